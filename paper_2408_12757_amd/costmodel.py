"""Flop / byte accounting and the iteration roofline (host logic, no GPU).

Follows the paper's cost model: a dense operation on a batch of B tokens with
a weight [N, K] performs 2*B*N*K flops (Sec. 3.2, "Compute") and moves its
weight, its input and its output once (the "Mem Load" column of Table 2 is
S_type * (N*K + B*K + B*N)); decode attention reads the K and V of every
cached token once per kv head (Sec. 2.2, "Attention operations") and performs
4 flops per (cached token, q head, head dim element).  The estimated time of an
operation is max(T_compute, T_mem) with T = work / capacity (Sec. 3.4).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict

import numpy as np

# published MI355X peaks used for every roofline figure reported by the bench
MI355X_PEAK_BF16_FLOPS = 2.5e15
MI355X_PEAK_HBM_BPS = 8.0e12


def gemm_flops(B: int, N: int, K: int) -> float:
    return 2.0 * B * N * K


def gemm_bytes(B: int, N: int, K: int, s_type: int = 2) -> float:
    return float(s_type) * (N * K + B * K + B * N)


@dataclass
class OpCost:
    flops: float
    bytes: float

    def t_est(self, compute: float, membw: float) -> float:
        """max(T_compute, T_mem) in seconds (Sec. 3.4)."""
        return max(self.flops / compute, self.bytes / membw)


def attention_tokens(batch) -> "tuple[int, int]":
    """(sum over decode tokens of keys read, sum over prefill tokens of keys read).
    A token at position pos reads pos + 1 keys (itself included)."""
    q_indptr = np.asarray(batch.q_indptr, np.int64)
    ctx = np.asarray(batch.ctx_len, np.int64)
    npf = int(batch.n_prefill_reqs)
    dec = int(np.sum(ctx[npf:] + 1))
    pf = 0
    for r in range(npf):
        n = int(q_indptr[r + 1] - q_indptr[r])
        pf += n * int(ctx[r]) + n * (n + 1) // 2
    return dec, pf


def layer_costs(model, batch, s_type: int = 2) -> Dict[str, OpCost]:
    """Algorithmic work of one decoder layer on one dense batch.

    Weights are counted once per layer (not once per nano-batch), KV once per
    kv head (not once per q head); a MoE layer counts the flops of the top_k
    selected experts and the weights of all experts.
    """
    B = int(batch.n_tokens)
    D, Hq, Hkv, dh, I = model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim, model.ffn_inner
    E = max(1, model.n_experts)
    k = model.top_k if model.n_experts > 1 else 1
    nqkv = (Hq + 2 * Hkv) * dh
    dec_keys, pf_keys = attention_tokens(batch)
    kv_tok_bytes = 2 * Hkv * dh * s_type
    npf = int(batch.n_prefill_reqs)
    ctx = np.asarray(batch.ctx_len, np.int64)
    q_indptr = np.asarray(batch.q_indptr, np.int64)
    n_dec = int(batch.n_decode_reqs)
    n_pf_tok = int(q_indptr[npf])
    # prefill reads each request's keys once (cached prefix + own chunk)
    pf_read_tok = int(np.sum(ctx[:npf])) + n_pf_tok
    ops = {
        "KQV": OpCost(gemm_flops(B, nqkv, D), gemm_bytes(B, nqkv, D, s_type)),
        "O": OpCost(gemm_flops(B, D, Hq * dh), gemm_bytes(B, D, Hq * dh, s_type)),
        "UG": OpCost(k * gemm_flops(B, 2 * I, D),
                     s_type * (E * 2 * I * D + B * D + k * B * 2 * I)),
        "D": OpCost(k * gemm_flops(B, D, I), s_type * (E * D * I + k * B * I + B * D)),
        "DecAttn": OpCost(4.0 * dec_keys * Hq * dh,
                          kv_tok_bytes * dec_keys + 2 * n_dec * Hq * dh * s_type),
        "PfAttn": OpCost(4.0 * pf_keys * Hq * dh,
                         kv_tok_bytes * pf_read_tok + 2 * n_pf_tok * Hq * dh * s_type),
        "KVAppend": OpCost(0.0, kv_tok_bytes * B),
    }
    if model.n_experts > 1:
        ops["Router"] = OpCost(gemm_flops(B, E, D), gemm_bytes(B, E, D, s_type))
    return ops


def iteration_roofline(costs: Dict[str, OpCost], peak_flops: float = MI355X_PEAK_BF16_FLOPS,
                       peak_bw: float = MI355X_PEAK_HBM_BPS) -> Dict[str, float]:
    """Lower bound of one layer-iteration: max(total flops / peak, total bytes / peak)."""
    F = sum(c.flops for c in costs.values())
    Bt = sum(c.bytes for c in costs.values())
    t_c, t_m = F / peak_flops, Bt / peak_bw
    return {"flops": F, "bytes": Bt, "t_compute": t_c, "t_mem": t_m, "t_roofline": max(t_c, t_m),
            "bound": "mfma" if t_c >= t_m else "hbm", "T_R": t_m / t_c}


def optimal_throughput(compute: float, p_model: float) -> float:
    """Eq. 5: tokens/s when compute is fully used = Compute / (2 * P_model)."""
    return compute / (2.0 * p_model)


def t_ratio(compute: float, membw: float, memsize: float, p_model: float, b_dense: int) -> float:
    """Eq. 4: T_R = T_mem / T_compute = (Compute/MemBW) * (MemSize/P_model) / (2 * B_dense)."""
    return (compute / membw) * (memsize / p_model) / (2.0 * b_dense)
