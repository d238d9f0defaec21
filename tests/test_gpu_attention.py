"""GPU parity of the attention path on its own scale (Sec. 2.2 "Attention operations"):
rotary embedding + KV append + paged attention through the single-operation entry points of
the C ABI, on seeded random Q/K/V rows and pages, against the oracle's attention stage.

Two kinds of evidence:
  * every output row against the oracle, relative to that row's own magnitude (a row over
    9000 keys has values near 0.02; measured against the layer output it would vanish);
  * planted keys ("needles"): one cached key per (request, kv head) is made parallel to the
    rotated query of one q head with a score about 30 above the rest, at positions around
    every boundary the kernel has (page, 64-page id group, 2048-key chunk, last cached
    key, first key).  The softmax then puts weight 1 - 1e-9 on it and the output row must
    equal that key's V row - a closed form that an off-by-one, a wrong page order or a
    dropped chunk cannot satisfy at any context length.
The demonstration that these measures reject a wrong attention (zero output, uniform
weights, dropped key, wrong scale, wrong head mapping) runs on the CPU in
tests/test_parity_metric.py.
"""
import numpy as np
import pytest
import torch

from oracle import decoder_layer as orc
from paper_2408_12757_amd import binding as nf
from paper_2408_12757_amd import harness as hz
from paper_2408_12757_amd import workloads as wl

from cases import EDGE_CASES, edge_case_batch
from gpu_util import DEV, f64
from parity_metrics import REL_TOL, rms_report, row_rel_err, tensor_rel_err

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def ctx():
    c = nf.Context(0)
    yield c
    c.close()


def split_qkv(model, qkv):
    Hq, Hkv, dh = model.n_q_heads, model.n_kv_heads, model.head_dim
    B = qkv.shape[0]
    q = qkv[:, :Hq * dh].reshape(B, Hq, dh)
    k = qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(B, Hkv, dh)
    v = qkv[:, (Hq + Hkv) * dh:].reshape(B, Hkv, dh)
    return q, k, v


def positions(batch):
    pos = np.zeros(batch.n_tokens, np.int64)
    for r in range(batch.n_reqs):
        t0, t1 = int(batch.q_indptr[r]), int(batch.q_indptr[r + 1])
        pos[t0:t1] = int(batch.ctx_len[r]) + np.arange(t1 - t0)
    return pos


def needle_positions(c: int):
    cand = [0, 15, 16, 1023, 1024, 2047, 2048, 4095, 4096, 8191, c // 2, c - 2, c - 1]
    return sorted({p for p in cand if 0 <= p < c})


def plant_needles(model, batch, qkv_bits, pages_bits, round_index: int):
    """Overwrites one key per (request, kv head) - a cached one, the fresh key of the middle
    token of a prefill chunk, or the row's own fresh key, in turn - with a multiple of the
    rotated query of the request's last token (first q head of the group).  Returns [(token, q head, expected
    V row in float64)].  Input formatting only: the layout index map and the oracle's rotary
    embedding (used to aim the key), no attention arithmetic."""
    Hq, Hkv, dh, P = model.n_q_heads, model.n_kv_heads, model.head_dim, model.page_size
    G = Hq // Hkv
    kidx, vidx = wl.page_block_index(dh, P)
    pages = pages_bits.reshape(pages_bits.shape[0], 2, Hkv, P * dh)
    pos = positions(batch)
    q, k, v = split_qkv(model, f64(qkv_bits))
    q_rot = orc.rope(q, pos, model.rope_theta)
    expect = []
    for r in range(batch.n_reqs):
        t0, t1 = int(batch.q_indptr[r]), int(batch.q_indptr[r + 1])
        c = int(batch.ctx_len[r])
        t = t1 - 1                                   # the row that must find the needle
        plist = batch.page_ids[int(batch.page_indptr[r]):int(batch.page_indptr[r + 1])]
        cands = needle_positions(c)
        for hk in range(Hkv):
            hq = hk * G
            aim = q_rot[t, hq]
            sigma = np.linalg.norm(aim) / np.sqrt(dh)            # std of a random key's score
            gain = (30.0 + 6.0 * sigma) * np.sqrt(dh) / float(aim @ aim)
            mode = (round_index + hk) % 3
            col, vcol = (Hq + hk) * dh, (Hq + Hkv + hk) * dh
            if mode == 0 and t1 - t0 >= 3:
                # fresh key of the chunk's middle token: undo its own rotation
                j = t0 + (t1 - t0) // 2
                pre = orc.rope((gain * aim)[None, None, :], -pos[j:j + 1], model.rope_theta)[0, 0]
                qkv_bits[j, col:col + dh] = wl.f32_to_bf16_bits(pre.astype(np.float32))
                expect.append((t, hq, f64(qkv_bits[j, vcol:vcol + dh])))
            elif mode == 2 or not cands:
                # the row's own key (appended in this iteration): same position, so the
                # rotation leaves the product with its own query unchanged
                qkv_bits[t, col:col + dh] = wl.f32_to_bf16_bits((gain * q[t, hq]).astype(np.float32))
                expect.append((t, hq, f64(qkv_bits[t, vcol:vcol + dh])))
            else:
                p = cands[(round_index * Hkv + hk) % len(cands)]
                page, slot = int(plist[p // P]), p % P
                pages[page, 0, hk][kidx[slot]] = wl.f32_to_bf16_bits((gain * aim).astype(np.float32))
                expect.append((t, hq, f64(pages[page, 1, hk][vidx[slot]])))
    return expect


def oracle_attention(model, batch, pages_bits, qkv_bits):
    q, k, v = split_qkv(model, f64(qkv_bits))
    return orc.attention_stage(model, batch, pages_bits, q, k, v)       # q_rot, k_rot, attn


def gpu_attention(ctx, model, batch, args, qkv_bits, pages_bits, bounds, attn_wgs):
    """nf_op_rope_append on all rows, then nf_op_attention per nano-batch.  Returns the
    bits of (qkv after the call, attention output, pages after the call)."""
    B = batch.n_tokens
    pages = hz.bf16_tensor(pages_bits, DEV)
    qkv = hz.bf16_tensor(qkv_bits, DEV)
    attn = torch.full((B, model.q_dim), 7.0, dtype=torch.bfloat16, device=DEV)
    plan = nf.nf_plan_manual(ctx, model, args, bounds, False, 0, 0, attn_wgs)
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=DEV)
    for i in range(len(bounds) - 1):
        nf.nf_op_rope_append(ctx, model, pages.data_ptr(), batch.num_pages, args, plan, qkv.data_ptr(),
                             bounds[i], bounds[i + 1])
    for i in range(len(bounds) - 1):
        nf.nf_op_attention(ctx, model, pages.data_ptr(), batch.num_pages, args, plan, qkv.data_ptr(),
                           attn.data_ptr(), ws.data_ptr(), ws.numel(), i)
    torch.cuda.synchronize()
    plan.close()
    return hz.bf16_bits(qkv), hz.bf16_bits(attn), hz.bf16_bits(pages)


def compare_with_oracle(model, batch, qkv_bits, pages_bits, got_qkv, got_attn, got_pages, expect, tok=None):
    """tok: rows (of the tensors as given) to compare; the oracle inputs must already be
    restricted to them."""
    Hq, Hkv, dh = model.n_q_heads, model.n_kv_heads, model.head_dim
    q_rot, k_rot, attn = oracle_attention(model, batch, pages_bits, qkv_bits)
    B = batch.n_tokens
    g_attn = f64(got_attn).reshape(B, Hq, dh)
    fig = {"attn": tensor_rel_err(g_attn, attn), "attn_row": row_rel_err(g_attn, attn),
           "attn_rms": rms_report(g_attn, attn)}
    assert np.all(np.isfinite(g_attn))
    assert fig["attn"] <= REL_TOL and fig["attn_row"] <= REL_TOL, fig
    # rotated Q left in place, K and V rows in their page slots
    gq, _, _ = split_qkv(model, f64(got_qkv))
    fig["q"] = tensor_rel_err(gq, q_rot)
    assert fig["q"] <= REL_TOL / 2, fig
    if got_pages is not None:
        kg, vg = hz.read_kv_rows(got_pages, model, batch, np.arange(B))
        _, _, v = split_qkv(model, f64(qkv_bits))
        fig["k"], fig["v"] = tensor_rel_err(f64(kg), k_rot), tensor_rel_err(f64(vg), v)
        assert fig["k"] <= REL_TOL / 2 and fig["v"] == 0.0, fig
    worst = 0.0
    for t, hq, vrow in expect:
        worst = max(worst, float(np.max(np.abs(g_attn[t, hq] - vrow))))
    fig["needle"] = worst
    # weight of everything else <= n * exp(-30) ~ 1e-9; bf16 store of the output: half an ulp
    assert worst <= 2.0 ** -8 * 6.0, fig
    return fig


@pytest.mark.parametrize("name", ["page_edges", "long_ctx", "prefill_prior", "gqa8", "mha64", "prefill_only",
                                  "one_decode"])
def test_attention_ops_match_oracle_per_row(ctx, name):
    model, b, seed = edge_case_batch(name)
    rng = np.random.default_rng(seed + 50)
    args = hz.upload_batch(b, DEV)
    pages0 = wl.make_kv_pages_host(model, b.num_pages, seed + 3)
    structures = [([0, b.n_tokens], 0)]
    if b.n_tokens >= 4:
        structures += [([0, b.n_tokens // 2, b.n_tokens], -1), ([0, 1, b.n_tokens - 1, b.n_tokens], 3)]
    for rnd, (bounds, wgs) in enumerate(structures):
        # q rows with unit-variance elements give scores of standard deviation 1 against
        # N(0,1) keys: a softmax far from uniform, so wrong weights show
        qkv_bits = wl.f32_to_bf16_bits(rng.standard_normal((b.n_tokens, model.n_qkv)).astype(np.float32))
        pages_bits = pages0.copy()
        expect = plant_needles(model, b, qkv_bits, pages_bits, rnd)
        say(name, "bounds", bounds, "attn_wgs", wgs, "needles", len(expect))
        got = gpu_attention(ctx, model, b, args, qkv_bits, pages_bits, bounds, wgs)
        fig = compare_with_oracle(model, b, qkv_bits, pages_bits, *got, expect)
        say(name, fig)


def test_attention_without_needles_is_not_uniform_and_matches(ctx):
    """Plain random rows (no planted key) at long contexts: the oracle's softmax weights
    are far from uniform here, and the outputs agree per row."""
    model, b, seed = edge_case_batch("long_ctx")
    rng = np.random.default_rng(77)
    args = hz.upload_batch(b, DEV)
    pages_bits = wl.make_kv_pages_host(model, b.num_pages, seed + 3)
    qkv_bits = wl.f32_to_bf16_bits((1.5 * rng.standard_normal((b.n_tokens, model.n_qkv))).astype(np.float32))
    got = gpu_attention(ctx, model, b, args, qkv_bits, pages_bits, [0, b.n_tokens], 0)
    fig = compare_with_oracle(model, b, qkv_bits, pages_bits, *got, [])
    say("long_ctx, no needles", fig)
