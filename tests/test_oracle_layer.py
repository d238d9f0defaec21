"""Pins for the CPU oracle's whole-layer wiring (CPU only).

The layer is pinned (a) against library routines in the special case they
cover (prefill-only batch: torch rms_norm / linear / causal
scaled_dot_product_attention, rotary embedding written as a complex product),
(b) by prefill <-> decode consistency, which ties the paged decode path to the
prefill path, and (c) by invariances: physical page permutation, GQA head
duplication, request-aligned batch splitting (nano-batch invariance, Sec. 3.7).
"""
import dataclasses

import numpy as np
import torch

from oracle import decoder_layer as orc
from paper_2408_12757_amd import workloads as wl


def small_model(**kw):
    base = dict(hidden=32, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn_inner=24, page_size=16,
                rope_theta=1e4, rms_eps=1e-5)
    base.update(kw)
    return wl.ModelDesc(**base)


def float_weights(m, seed, scale=0.3):
    r = np.random.default_rng(seed)
    E = m.experts
    return {
        "g_attn_norm": 1 + 0.1 * r.standard_normal(m.hidden),
        "w_qkv": scale * r.standard_normal((m.n_qkv, m.hidden)),
        "w_o": scale * r.standard_normal((m.hidden, m.q_dim)),
        "g_ffn_norm": 1 + 0.1 * r.standard_normal(m.hidden),
        "w_gate_up": scale * r.standard_normal((E, 2 * m.ffn_inner, m.hidden)),
        "w_down": scale * r.standard_normal((E, m.hidden, m.ffn_inner)),
        "w_router": r.standard_normal((E, m.hidden)) if m.is_moe else None,
    }


def mk_batch(q_lens, ctx, n_pf, page_size, seed=0, spare=3):
    return wl.batch_from_lengths(q_lens, ctx, n_pf, np.random.default_rng(seed), page_size, spare)


def random_pages(m, num_pages, seed):
    return np.random.default_rng(seed).standard_normal((num_pages, m.page_elems))


# ---------------------------------------------------- (a) library routines ---

def torch_prefill_layer(m, w, x, q_lens):
    """Prefill-only decoder layer from torch library routines, float64."""
    F = torch.nn.functional
    t = {k: (torch.from_numpy(np.asarray(v, np.float64)) if v is not None else None) for k, v in w.items()}
    xs = torch.from_numpy(x)
    h = F.rms_norm(xs, (m.hidden,), t["g_attn_norm"], eps=m.rms_eps)
    qkv = F.linear(h, t["w_qkv"])
    Hq, Hkv, dh = m.n_q_heads, m.n_kv_heads, m.head_dim
    outs = []
    off = 0
    for n in q_lens:
        seg = qkv[off:off + n]
        q = seg[:, :Hq * dh].reshape(n, Hq, dh)
        k = seg[:, Hq * dh:(Hq + Hkv) * dh].reshape(n, Hkv, dh)
        v = seg[:, (Hq + Hkv) * dh:].reshape(n, Hkv, dh)
        pos = torch.arange(n, dtype=torch.float64)
        inv = 1.0 / (m.rope_theta ** (torch.arange(0, dh, 2, dtype=torch.float64) / dh))
        rot = torch.polar(torch.ones(n, dh // 2, dtype=torch.float64), pos[:, None] * inv[None, :])

        def rope_c(u):                       # pair (i, i + dh/2) as a complex number
            z = torch.complex(u[..., :dh // 2], u[..., dh // 2:]) * rot[:, None, :]
            return torch.cat([z.real, z.imag], dim=-1)

        q, k = rope_c(q), rope_c(k)
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None],
                                           v.permute(1, 0, 2)[None], is_causal=True, enable_gqa=True)
        outs.append(o[0].permute(1, 0, 2).reshape(n, Hq * dh))
        off += n
    a = torch.cat(outs, 0)
    y = xs + F.linear(a, t["w_o"])
    h2 = F.rms_norm(y, (m.hidden,), t["g_ffn_norm"], eps=m.rms_eps)
    gu = F.linear(h2, t["w_gate_up"][0])
    f = F.silu(gu[:, :m.ffn_inner]) * gu[:, m.ffn_inner:]
    return (y + F.linear(f, t["w_down"][0])).numpy()


def test_prefill_only_layer_matches_torch_library_routines():
    m = small_model()
    w = float_weights(m, 21)
    q_lens = [7, 1, 10]
    b = mk_batch(q_lens, [0, 0, 0], 3, m.page_size)
    x = np.random.default_rng(22).standard_normal((b.n_tokens, m.hidden))
    pages = random_pages(m, b.num_pages, 23)
    z, k_new, v_new = orc.layer_forward(m, w, pages, b, x)
    ref = torch_prefill_layer(m, w, x, q_lens)
    np.testing.assert_allclose(z, ref, rtol=1e-10, atol=1e-11)


def test_layer_chain_matches_torch_library_routines_applied_in_sequence():
    """Consecutive layers: each layer has its own weights and its own pool, the output of one
    is the input of the next (Sec. 2.1).  A wrong hand-over (weights or pools swapped, an
    input reused) changes the result."""
    m = small_model()
    ws = [float_weights(m, 61 + l) for l in range(3)]
    q_lens = [6, 9]
    b = mk_batch(q_lens, [0, 0], 2, m.page_size)
    x = np.random.default_rng(62).standard_normal((b.n_tokens, m.hidden))
    pools = [random_pages(m, b.num_pages, 63 + l) for l in range(3)]
    z, ks, vs = orc.layers_forward(m, ws, pools, b, x)
    ref = x
    for w in ws:
        ref = torch_prefill_layer(m, w, ref, q_lens)
    np.testing.assert_allclose(z, ref, rtol=1e-9, atol=1e-10)
    assert len(ks) == 3 and len(vs) == 3
    # layer 0 of the chain is the single layer; the order of the layers matters
    z0, k0, v0 = orc.layer_forward(m, ws[0], pools[0], b, x)
    np.testing.assert_array_equal(ks[0], k0)
    z_swapped, _, _ = orc.layers_forward(m, ws[::-1], pools, b, x)
    assert np.max(np.abs(z_swapped - z)) > 1e-3


def test_residuals_present():
    m = small_model()
    w = float_weights(m, 24)
    b = mk_batch([5, 1, 1], [0, 6, 9], 1, m.page_size)
    x = np.random.default_rng(25).standard_normal((b.n_tokens, m.hidden))
    pages = random_pages(m, b.num_pages, 26)
    w0 = dict(w, w_o=np.zeros_like(w["w_o"]), w_down=np.zeros_like(w["w_down"]))
    z, _, _ = orc.layer_forward(m, w0, pages, b, x)
    np.testing.assert_array_equal(z, x)
    # W_down = 0 only: z = x + attention block, which differs from x
    w1 = dict(w, w_down=np.zeros_like(w["w_down"]))
    z1, _, _, parts = orc.layer_forward(m, w1, pages, b, x, return_parts=True)
    np.testing.assert_array_equal(z1, parts["y"])
    assert np.max(np.abs(z1 - x)) > 1e-3


# ------------------------------------------- (b) prefill <-> decode, paging ---

def write_rows_to_pages(m, pages, batch, r, k_rows, v_rows, start_pos=0):
    """Store K/V rows of request r at positions start_pos.. (append rule)."""
    P, Hkv, dh = m.page_size, m.n_kv_heads, m.head_dim
    pg = pages.reshape(pages.shape[0], 2, Hkv, P * dh)
    kidx, vidx = wl.page_block_index(dh, P)
    for i in range(k_rows.shape[0]):
        page, slot = orc.kv_slot(batch, m, r, start_pos + i)
        for h in range(Hkv):
            pg[page, 0, h][kidx[slot]] = k_rows[i, h]
            pg[page, 1, h][vidx[slot]] = v_rows[i, h]


def test_decode_equals_last_row_of_prefill():
    m = small_model()
    w = float_weights(m, 31)
    c = 9
    x = np.random.default_rng(32).standard_normal((c + 1, m.hidden))
    bp = mk_batch([c + 1], [0], 1, m.page_size)
    zp, kp, vp = orc.layer_forward(m, w, random_pages(m, bp.num_pages, 33), bp, x)
    # decode request whose cache holds the first c tokens' K/V (float pages: unrounded)
    bd = mk_batch([1], [c], 0, m.page_size, seed=5)
    pages = random_pages(m, bd.num_pages, 34)
    write_rows_to_pages(m, pages, bd, 0, kp[:c], vp[:c])
    zd, kd, vd = orc.layer_forward(m, w, pages, bd, x[c:c + 1])
    np.testing.assert_allclose(zd[0], zp[c], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(kd[0], kp[c], rtol=1e-12, atol=1e-13)


def test_chunked_prefill_with_prior_context_equals_full_prefill():
    m = small_model()
    w = float_weights(m, 35)
    n, c = 11, 6
    x = np.random.default_rng(36).standard_normal((n, m.hidden))
    bf = mk_batch([n], [0], 1, m.page_size)
    zf, kf, vf = orc.layer_forward(m, w, random_pages(m, bf.num_pages, 37), bf, x)
    bc = mk_batch([n - c], [c], 1, m.page_size, seed=9)
    pages = random_pages(m, bc.num_pages, 38)
    write_rows_to_pages(m, pages, bc, 0, kf[:c], vf[:c])
    zc, _, _ = orc.layer_forward(m, w, pages, bc, x[c:])
    np.testing.assert_allclose(zc, zf[c:], rtol=1e-11, atol=1e-12)


def test_page_permutation_invariance():
    m = small_model()
    w = float_weights(m, 41)
    b = mk_batch([6, 1, 1, 1], [0, 13, 4, 8], 1, m.page_size, seed=1, spare=5)
    x = np.random.default_rng(42).standard_normal((b.n_tokens, m.hidden))
    pages = random_pages(m, b.num_pages, 43)
    z, _, _ = orc.layer_forward(m, w, pages, b, x)
    perm = np.random.default_rng(44).permutation(b.num_pages)       # new id of old page i
    pages2 = np.empty_like(pages)
    pages2[perm] = pages
    b2 = dataclasses.replace(b, page_ids=perm[b.page_ids].astype(np.int32))
    z2, _, _ = orc.layer_forward(m, w, pages2, b2, x)
    np.testing.assert_array_equal(z, z2)


def test_gqa_equals_mha_with_duplicated_kv_heads():
    m = small_model(n_q_heads=4, n_kv_heads=2)
    G = 2
    w = float_weights(m, 51)
    b = mk_batch([5, 1, 1], [0, 7, 10], 1, m.page_size, seed=2)
    x = np.random.default_rng(52).standard_normal((b.n_tokens, m.hidden))
    pages = random_pages(m, b.num_pages, 53)
    z, _, _ = orc.layer_forward(m, w, pages, b, x)

    m2 = dataclasses.replace(m, n_kv_heads=4)
    dh, Hq = m.head_dim, m.n_q_heads
    wq = w["w_qkv"][:Hq * dh]
    wk = w["w_qkv"][Hq * dh:(Hq + 2) * dh].reshape(2, dh, m.hidden)
    wv = w["w_qkv"][(Hq + 2) * dh:].reshape(2, dh, m.hidden)
    w2 = dict(w, w_qkv=np.concatenate([wq, np.repeat(wk, G, axis=0).reshape(-1, m.hidden),
                                       np.repeat(wv, G, axis=0).reshape(-1, m.hidden)]))
    pg = pages.reshape(b.num_pages, 2, 2, -1)
    pages2 = np.repeat(pg, G, axis=2).reshape(b.num_pages, -1)
    z2, _, _ = orc.layer_forward(m2, w2, pages2, b, x)
    np.testing.assert_allclose(z, z2, rtol=1e-12, atol=1e-13)


# ------------------------------------------------ (c) nano-batch invariance ---

def test_request_aligned_split_gives_identical_rows():
    m = small_model()
    w = float_weights(m, 61)
    b = mk_batch([4, 3, 1, 1, 1, 1], [0, 5, 12, 3, 20, 7], 2, m.page_size, seed=3)
    x = np.random.default_rng(62).standard_normal((b.n_tokens, m.hidden))
    pages = random_pages(m, b.num_pages, 63)
    z, k, v = orc.layer_forward(m, w, pages, b, x)
    for reqs in ([0, 2, 3], [1, 4, 5], [5]):
        sub, tok, phys = wl.subset_batch(b, reqs)
        zs, ks, vs = orc.layer_forward(m, w, pages[phys], sub, x[tok])
        # equal up to the rounding order of the float64 matmul library
        np.testing.assert_allclose(zs, z[tok], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(ks, k[tok], rtol=1e-12, atol=1e-13)


def test_new_kv_rows_and_positions():
    # position of a token = ctx_len + index in its chunk; at position 0 the
    # rotary embedding is the identity, so k_new is the plain K projection
    m = small_model()
    w = float_weights(m, 71)
    b = mk_batch([3, 1], [0, 20], 1, m.page_size)
    x = np.random.default_rng(72).standard_normal((b.n_tokens, m.hidden))
    pages = random_pages(m, b.num_pages, 73)
    z, k, v, parts = orc.layer_forward(m, w, pages, b, x, return_parts=True)
    Hq, Hkv, dh = m.n_q_heads, m.n_kv_heads, m.head_dim
    plain = parts["h"] @ w["w_qkv"].T
    np.testing.assert_allclose(k[0].ravel(), plain[0, Hq * dh:(Hq + Hkv) * dh], rtol=1e-12)
    np.testing.assert_allclose(v.reshape(b.n_tokens, -1), plain[:, (Hq + Hkv) * dh:], rtol=1e-12)
    # decode token (row 3) sits at position 20: its K differs from the plain projection
    # by a rotation of exactly 20 rad in the first pair of every head
    kp = plain[3, Hq * dh:(Hq + Hkv) * dh].reshape(Hkv, dh)
    a, bb = kp[:, 0], kp[:, dh // 2]
    np.testing.assert_allclose(k[3, :, 0], a * np.cos(20.0) - bb * np.sin(20.0), rtol=1e-11)
    assert orc.kv_slot(b, m, 1, 20) == (int(b.page_ids[b.page_indptr[1] + 1]), 4)


def test_moe_layer_identical_experts_equals_dense_layer():
    m = small_model(n_experts=4, top_k=2)
    w = float_weights(m, 81)
    w["w_gate_up"] = np.repeat(w["w_gate_up"][:1], 4, axis=0)
    w["w_down"] = np.repeat(w["w_down"][:1], 4, axis=0)
    b = mk_batch([4, 1, 1], [0, 6, 2], 1, m.page_size)
    x = np.random.default_rng(82).standard_normal((b.n_tokens, m.hidden))
    pages = random_pages(m, b.num_pages, 83)
    z, _, _ = orc.layer_forward(m, w, pages, b, x)
    md = dataclasses.replace(m, n_experts=0, top_k=0)
    zd, _, _ = orc.layer_forward(md, w, pages, b, x)
    np.testing.assert_allclose(z, zd, rtol=1e-12, atol=1e-13)


def test_bf16_inputs_are_widened_exactly():
    cfg = wl.CONFIGS["C1"]
    m = cfg.model
    wb = wl.make_weights(m, cfg.seed)
    b = wl.make_batch(cfg.batch, cfg.seed + 2)
    xb = wl.make_x(b.n_tokens, m.hidden, cfg.seed + 1)
    pages = wl.make_kv_pages_host(m, b.num_pages, cfg.seed + 3)
    sub, tok, phys = wl.subset_batch(b, [0, 5, 9])
    z, _, _ = orc.layer_forward(m, wb, pages[phys], sub, xb[tok])
    wf = {k: (orc.widen(v) if v is not None else None) for k, v in wb.items()}
    z2, _, _ = orc.layer_forward(m, wf, orc.widen(pages[phys]), sub, orc.widen(xb[tok]))
    np.testing.assert_allclose(z, z2, rtol=1e-12, atol=1e-13)
    assert np.all(np.isfinite(z))
