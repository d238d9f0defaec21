"""Pins for the CPU oracle's individual operations.

Each test checks the oracle against something other than itself: brute force
in pure Python, a closed form, an invariant, or a library routine the special
case reduces to.  CPU only.
"""
import math

import numpy as np
import pytest
import torch

from oracle import decoder_layer as orc


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ dense ---

def test_dense_matches_naive_triple_loop():
    r = rng(1)
    T, N, K = 5, 7, 6
    x = r.standard_normal((T, K))
    w = r.standard_normal((N, K))
    y = orc.dense(x, w)
    assert y.shape == (T, N)
    for t in range(T):
        for n in range(N):
            acc = math.fsum(float(x[t, k]) * float(w[n, k]) for k in range(K))
            assert abs(y[t, n] - acc) <= 1e-13 * (1 + abs(acc))


def test_dense_one_hot_weight_picks_column():
    # w[n0, k0] = 1 : output column n0 is input column k0 (orientation of W[N, K])
    r = rng(2)
    x = r.standard_normal((4, 6))
    w = np.zeros((3, 6))
    w[2, 5] = 1.0
    y = orc.dense(x, w)
    assert np.array_equal(y[:, 2], x[:, 5])
    assert np.all(y[:, :2] == 0)


def test_dense_linearity():
    r = rng(3)
    x1, x2 = r.standard_normal((2, 3, 8))
    w = r.standard_normal((5, 8))
    np.testing.assert_allclose(orc.dense(2 * x1 - 3 * x2, w), 2 * orc.dense(x1, w) - 3 * orc.dense(x2, w),
                               rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- rmsnorm ---

def test_rmsnorm_constant_row_closed_form():
    D, c, eps = 16, 3.0, 1e-5
    g = np.linspace(0.5, 2.0, D)
    out = orc.rmsnorm(np.full((2, D), c), g, eps)
    np.testing.assert_allclose(out, np.broadcast_to(g * c / math.sqrt(c * c + eps), (2, D)), rtol=1e-14)


def test_rmsnorm_energy_identity_and_scale_invariance():
    r = rng(4)
    D, eps = 64, 1e-5
    x = r.standard_normal((3, D)) * 5
    g = 1 + 0.1 * r.standard_normal(D)
    out = orc.rmsnorm(x, g, eps)
    ms = np.mean(x ** 2, axis=1)
    np.testing.assert_allclose(np.mean((out / g) ** 2, axis=1), ms / (ms + eps), rtol=1e-12)
    # eps -> 0: invariant to the scale of x
    np.testing.assert_allclose(orc.rmsnorm(x, g, 0.0), orc.rmsnorm(7.5 * x, g, 0.0), rtol=1e-12)


def test_rmsnorm_matches_torch_rms_norm():
    r = rng(5)
    x = r.standard_normal((4, 32))
    g = r.standard_normal(32)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(orc.rmsnorm(x, g, 1e-5), ref, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------- rope ---

def test_rope_pos0_identity_and_norm_preserved():
    r = rng(6)
    v = r.standard_normal((3, 2, 8))
    np.testing.assert_array_equal(orc.rope(v, np.zeros(3, np.int64), 1e4), v)
    out = orc.rope(v, np.array([5, 17, 1234]), 1e4)
    half = 4
    np.testing.assert_allclose(out[..., :half] ** 2 + out[..., half:] ** 2,
                               v[..., :half] ** 2 + v[..., half:] ** 2, rtol=1e-12)


def test_rope_first_pair_rotates_by_pos_radians():
    # unit vector on element 0: pair (0, dh/2), frequency theta^0 = 1
    dh = 8
    v = np.zeros((1, 1, dh))
    v[0, 0, 0] = 1.0
    out = orc.rope(v, np.array([3]), 1e4)
    expect = np.zeros(dh)
    expect[0] = math.cos(3.0)
    expect[dh // 2] = math.sin(3.0)
    np.testing.assert_allclose(out[0, 0], expect, atol=1e-15)


def test_rope_frequency_of_second_pair_closed_form():
    # dh = 4, theta = 1e4: pair i=1 has frequency 1e4^(-2/4) = 0.01; pos 100 -> 1 rad
    v = np.zeros((1, 1, 4))
    v[0, 0, 3] = 1.0            # the "b" element of pair i=1 (elements 1 and 3)
    out = orc.rope(v, np.array([100]), 1e4)
    np.testing.assert_allclose(out[0, 0], [0.0, -math.sin(1.0), 0.0, math.cos(1.0)], atol=1e-14)


def test_rope_relative_position_property_and_inverse():
    r = rng(7)
    q = r.standard_normal((1, 1, 16))
    k = r.standard_normal((1, 1, 16))

    def dot(m, n):
        return float(np.sum(orc.rope(q, np.array([m]), 5e5) * orc.rope(k, np.array([n]), 5e5)))

    assert abs(dot(10, 3) - dot(107, 100)) < 1e-10
    assert abs(dot(10, 3) - dot(7, 0)) < 1e-10
    assert abs(dot(10, 3) - dot(3, 10)) > 1e-6      # sign of the relative offset matters
    back = orc.rope(orc.rope(q, np.array([41]), 1e4), np.array([-41]), 1e4)
    np.testing.assert_allclose(back, q, atol=1e-13)


# -------------------------------------------------------------- attention ---

def brute_attention(q, K, V):
    dh = len(q)
    s = [sum(q[d] * K[j][d] for d in range(dh)) / math.sqrt(dh) for j in range(len(K))]
    m = max(s)
    e = [math.exp(v - m) for v in s]
    tot = math.fsum(e)
    return [math.fsum(e[j] / tot * V[j][d] for j in range(len(K))) for d in range(len(V[0]))]


def test_attention_matches_brute_force():
    r = rng(8)
    q = r.standard_normal(8)
    K = r.standard_normal((11, 8))
    V = r.standard_normal((11, 8))
    np.testing.assert_allclose(orc.softmax_attention(q, K, V),
                               brute_attention(q.tolist(), K.tolist(), V.tolist()), rtol=1e-12, atol=1e-14)


def test_attention_special_cases():
    r = rng(9)
    q = r.standard_normal(4)
    V = r.standard_normal((5, 4))
    # one key: output is its value
    np.testing.assert_allclose(orc.softmax_attention(q, r.standard_normal((1, 4)), V[:1]), V[0], rtol=1e-15)
    # equal keys: mean of the values
    K = np.tile(r.standard_normal(4), (5, 1))
    np.testing.assert_allclose(orc.softmax_attention(q, K, V), V.mean(axis=0), rtol=1e-13)
    # a very negative score contributes nothing
    K2 = r.standard_normal((5, 4))
    K2[4] = -1e4 * q
    np.testing.assert_allclose(orc.softmax_attention(q, K2, V), orc.softmax_attention(q, K2[:4], V[:4]), rtol=1e-13)
    # adding the same constant to every score changes nothing
    u = q / np.dot(q, q) * 3.7
    np.testing.assert_allclose(orc.softmax_attention(q, K2[:4] + u, V[:4]),
                               orc.softmax_attention(q, K2[:4], V[:4]), rtol=1e-12)


def test_attention_scale_is_inverse_sqrt_head_dim():
    # two keys whose raw scores differ by sqrt(dh)*ln 3  ->  probabilities 3/4, 1/4
    dh = 16
    q = np.zeros(dh)
    q[0] = 1.0
    K = np.zeros((2, dh))
    K[0, 0] = math.sqrt(dh) * math.log(3.0)
    V = np.array([[1.0] + [0.0] * (dh - 1), [0.0, 1.0] + [0.0] * (dh - 2)])
    out = orc.softmax_attention(q, K, V)
    np.testing.assert_allclose(out[:2], [0.75, 0.25], rtol=1e-13)


# ----------------------------------------------------------------- swiglu ---

def test_silu_closed_forms():
    assert orc.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(orc.silu(np.array([math.log(3.0)])), [math.log(3.0) * 0.75], rtol=1e-15)
    a = np.linspace(-6, 6, 25)
    np.testing.assert_allclose(orc.silu(a), torch.nn.functional.silu(torch.from_numpy(a)).numpy(), rtol=1e-13)


def test_swiglu_gate_rows_first_then_up_rows():
    # I = 2, D = 3.  gate = [h0, h1], up = [h2, 1*h0]; down = identity-like
    wgu = np.array([[1, 0, 0], [0, 1, 0],      # gate rows
                    [0, 0, 1], [1, 0, 0.0]])   # up rows
    wd = np.array([[1, 0], [0, 1], [1, 1.0]])  # [D=3, I=2]
    h = np.array([[math.log(3.0), 0.0, 2.0]])
    f0 = math.log(3.0) * 0.75 * 2.0            # silu(h0)*h2
    f1 = 0.0                                   # silu(0)*h0
    np.testing.assert_allclose(orc.swiglu_ffn(h, wgu, wd), [[f0, f1, f0 + f1]], rtol=1e-14)
    assert np.all(orc.swiglu_ffn(np.zeros((2, 3)), wgu, wd) == 0)


# -------------------------------------------------------------------- moe ---

def test_route_topk_tie_and_order():
    logits = np.array([[0.5, 2.0, 2.0, -1.0],      # tie -> experts 1 then 2
                       [9.0, 1.0, 1.0, 1.0],       # tie for second place -> expert 1
                       [0.0, 0.0, math.log(3.0), 0.0]])
    idx, w = orc.route_topk(logits, 2)
    assert idx.tolist() == [[1, 2], [0, 1], [2, 0]]
    np.testing.assert_allclose(w[0], [0.5, 0.5])
    np.testing.assert_allclose(w[2], [0.75, 0.25], rtol=1e-14)
    assert w[1, 0] > 0.999


def test_moe_identical_experts_equals_dense_ffn():
    r = rng(10)
    D, I, E = 8, 6, 4
    wgu = r.standard_normal((2 * I, D))
    wd = r.standard_normal((D, I))
    h = r.standard_normal((5, D))
    wr = r.standard_normal((E, D))
    out, idx, wts, _ = orc.moe_ffn(h, wr, [wgu] * E, [wd] * E, 2)
    np.testing.assert_allclose(out, orc.swiglu_ffn(h, wgu, wd), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(wts.sum(axis=1), 1.0, rtol=1e-14)


def test_moe_selects_the_routed_expert_only():
    r = rng(11)
    D, I, E = 4, 3, 3
    wgus = [r.standard_normal((2 * I, D)) for _ in range(E)]
    wds = [r.standard_normal((D, I)) for _ in range(E)]
    h = np.abs(r.standard_normal((2, D))) + 0.1
    wr = np.zeros((E, D))
    wr[2] = 50.0            # expert 2 gets a huge logit, the rest tie at 0 -> expert 0 second
    out, idx, wts, _ = orc.moe_ffn(h, wr, wgus, wds, 2)
    assert idx.tolist() == [[2, 0], [2, 0]]
    np.testing.assert_allclose(out, orc.swiglu_ffn(h, wgus[2], wds[2]), rtol=1e-9)
    # an explicit choice overrides the argmax and re-normalises over the chosen logits
    out2, idx2, wts2, _ = orc.moe_ffn(h, np.zeros((E, D)), wgus, wds, 2, expert_choice=[[1, 0], [1, 0]])
    np.testing.assert_allclose(out2, 0.5 * orc.swiglu_ffn(h, wgus[1], wds[1]) + 0.5 * orc.swiglu_ffn(h, wgus[0], wds[0]),
                               rtol=1e-12)


# ------------------------------------------------------------- paged read ---

def test_gather_kv_layout():
    # The page block layouts, pinned element by element with the index formulas of the
    # interface: K (t, d) at ((d//32)*16 + t)*32 + d%32;
    # V (t, d) at ((((t//4)*(dh//32) + d//32)*16 + d%16)*2 + (d//16)%2)*4 + t%4.
    Hkv, dh, P = 2, 64, 16
    n_pages = 3
    pages = np.zeros((n_pages, 2, Hkv, P * dh))
    val = lambda p, h, t, d: 10000 * p + 1000 * h + 64 * t + d          # noqa: E731
    for p in range(n_pages):
        for h in range(Hkv):
            for t in range(P):
                for d in range(dh):
                    pages[p, 0, h, ((d // 32) * 16 + t) * 32 + d % 32] = val(p, h, t, d)
                    pages[p, 1, h, ((((t // 4) * (dh // 32) + d // 32) * 16 + d % 16) * 2 + (d // 16) % 2) * 4 + t % 4] = \
                        -val(p, h, t, d)
    # every position of a block is used exactly once
    assert len(np.unique(pages[0, 0, 0])) == P * dh and len(np.unique(pages[0, 1, 0])) == P * dh
    K, V = orc.gather_kv(pages.reshape(n_pages, -1), [2, 0], 21, Hkv, dh, P)
    assert K.shape == (21, Hkv, dh)
    for j in range(21):
        p = [2, 0][j // P]
        for h in range(Hkv):
            for d in range(dh):
                assert K[j, h, d] == val(p, h, j % P, d)
                assert V[j, h, d] == -val(p, h, j % P, d)


def test_widen_bf16_exact():
    bits = np.array([0x3F80, 0xC000, 0x3DCD, 0x0000], np.uint16)   # 1, -2, ~0.1001, 0
    out = orc.widen(bits)
    assert out.dtype == np.float64
    assert out[0] == 1.0 and out[1] == -2.0 and out[3] == 0.0
    assert out[2] == 0.10009765625
