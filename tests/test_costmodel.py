"""The flop/byte counters against the paper's worked example (Table 2)."""
import os

import numpy as np
import pytest

from paper_2408_12757_amd import costmodel as cm
from paper_2408_12757_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table2_cost_model.txt")


def table2():
    rows = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        rows[f[0]] = [float(v) for v in f[1:]]
    return rows


L, NGPU, B = 80, 8, 2048
M70 = wl.CONFIGS["C3"].model          # LLaMA-2-70B layer dimensions


def test_dense_ops_flops_and_bytes_match_table2():
    t2 = table2()
    shapes = {"KQV": (M70.n_qkv, M70.hidden), "O": (M70.hidden, M70.q_dim),
              "UG": (2 * M70.ffn_inner, M70.hidden), "D": (M70.hidden, M70.ffn_inner)}
    for op, (N, K) in shapes.items():
        gf = cm.gemm_flops(B, N, K) * L / 1e9
        gb = cm.gemm_bytes(B, N, K, 2) * L / 1e9
        assert abs(gf - t2[op][0]) <= 0.06, (op, gf)          # printed to 0.1 GFLOP
        assert abs(gb - t2[op][1]) <= 0.06, (op, gb)          # printed to 0.1 GB
        # estimated times with the paper's hardware constants
        assert abs(gf / (NGPU * 312e3) * 1e3 - t2[op][2]) <= 0.006, op
        assert abs(gb / (NGPU * 2000.0) * 1e3 - t2[op][3]) <= 0.01, op   # the paper divides the rounded GB


def test_layer_costs_agree_with_table2_for_a_70b_batch():
    # A batch with the paper's decode-attention flop count: 4 * keys * Hq * dh * L = 3665.9 GFLOP
    t2 = table2()
    keys = t2["DecAttn"][0] * 1e9 / (4 * M70.n_q_heads * M70.head_dim * L)
    n_dec = 1024
    ctx = np.full(n_dec, int(round(keys / n_dec)) - 1, np.int32)
    b = wl.batch_from_lengths(np.concatenate([[B - n_dec], np.ones(n_dec, np.int32)]),
                              np.concatenate([[0], ctx]), 1, np.random.default_rng(0))
    c = cm.layer_costs(M70, b)
    assert abs(c["DecAttn"].flops * L / 1e9 - t2["DecAttn"][0]) / t2["DecAttn"][0] < 1e-3
    # memory column: KV bytes of those keys (+ q/out); the paper prints 462.2 GB
    assert abs(c["DecAttn"].bytes * L / 1e9 - t2["DecAttn"][1]) / t2["DecAttn"][1] < 0.015
    for op in ("KQV", "O", "UG", "D"):
        assert abs(c[op].flops * L / 1e9 - t2[op][0]) <= 0.06
        assert abs(c[op].bytes * L / 1e9 - t2[op][1]) <= 0.06
    # decode attention is memory-bound, dense ops compute-bound on the paper's hardware
    assert c["DecAttn"].bytes / 2000e9 > c["DecAttn"].flops / 312e12
    assert c["UG"].flops / 312e12 > c["UG"].bytes / 2000e9
    t_est = c["DecAttn"].t_est(NGPU * 312e12, NGPU * 2000e9) * L * 1e3
    assert abs(t_est - t2["DecAttn"][3]) / t2["DecAttn"][3] < 0.015


def test_roofline_and_eq4_eq5():
    costs = {"a": cm.OpCost(2.5e15 * 1e-3, 1.0), "b": cm.OpCost(0.0, 8e12 * 2e-3)}
    r = cm.iteration_roofline(costs)
    assert r["bound"] == "hbm" and abs(r["t_roofline"] - 2e-3) < 1e-12 and abs(r["T_R"] - 2.0) < 1e-9
    # Eq. 5 with the inputs the paper names (280 TFLOP/s, 70e9 parameters) gives 2000 tokens/s/GPU;
    # the 1857 printed there corresponds to 260 TFLOP/s.  Both follow from the same formula.
    assert cm.optimal_throughput(280e12, 70e9) == pytest.approx(2000.0)
    assert cm.optimal_throughput(260e12, 70e9) == pytest.approx(1857.14, abs=0.01)
    # Eq. 4 on 8 x A100-80GB, 70B parameters, B_dense 2048: below 1 (compute-bound)
    tr = cm.t_ratio(8 * 312e12, 8 * 2000e9, 8 * 80e9, 70e9, 2048)
    assert tr == pytest.approx(156 * (640 / 70) / 4096, rel=1e-12) and tr < 1


def test_c2_batch_is_hbm_bound_on_mi355x():
    cfg = wl.CONFIGS["C2"]
    b = wl.make_batch(cfg.batch, cfg.seed + 2)
    assert b.n_tokens == 2048 and b.n_decode_reqs == 1792
    r = cm.iteration_roofline(cm.layer_costs(cfg.model, b))
    assert r["bound"] == "hbm"
    assert 0.9e12 < r["flops"] < 1.0e12
    assert 8e9 < r["bytes"] < 14e9
