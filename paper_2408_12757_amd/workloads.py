"""Seeded synthetic inputs for one decoder-layer iteration over a dense batch.

This module only *draws and formats data*: model shapes, random weights, a
dense batch of prefill + decode requests, context lengths, a page table and
KV-page contents.  It contains none of the decoder layer's arithmetic and is
imported neither by the CPU oracle nor by the HIP path; tests and the bench
hand its arrays to both.

bf16 tensors are carried on the host as ``numpy.uint16`` bit patterns.

Workload shapes follow the paper's description of a serving iteration: a
dense batch of B_dense tokens mixing the chunk of one or a few prefill
requests with one token from each of hundreds-to-thousands of decode
requests (Sec. 3.1 "Batch size", Sec. 4.2.1), a fragmented paged KV cache
(Sec. 4.2.2), and request lengths whose spread matches the dataset
statistics of Table 4 (coefficient of variation about 1, hence the
log-normal sigma of 0.83 used here).
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

PAGE_SIZE = 16
LOGNORMAL_SIGMA = 0.83


@dataclass(frozen=True)
class ModelDesc:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_inner: int
    n_experts: int = 0          # 0 or 1 = dense FFN
    top_k: int = 0
    page_size: int = PAGE_SIZE
    rms_eps: float = 1e-5
    rope_theta: float = 1e4

    @property
    def n_qkv(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def gqa(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def experts(self) -> int:
        return max(1, self.n_experts)

    @property
    def is_moe(self) -> bool:
        return self.n_experts > 1

    @property
    def page_elems(self) -> int:
        """bf16 elements in one page: K and V blocks of every kv head."""
        return 2 * self.n_kv_heads * self.page_size * self.head_dim


@dataclass(frozen=True)
class BatchSpec:
    """Recipe of one dense batch (see ``make_batch``)."""
    n_prefill_reqs: int
    prefill_len: int
    n_decode_reqs: int
    ctx_dist: str               # "uniform" | "lognormal"
    ctx_lo: int
    ctx_hi: int
    ctx_median: float = 0.0
    prefill_prior: int = 0      # tokens already cached for each prefill request


@dataclass(frozen=True)
class Config:
    name: str
    model: ModelDesc
    batch: BatchSpec
    seed: int
    granule: int                # nano-batch boundary granularity in tokens
    description: str = ""


CONFIGS: Dict[str, Config] = {
    "C1": Config(
        "C1",
        ModelDesc(hidden=512, n_q_heads=8, n_kv_heads=8, head_dim=64, ffn_inner=1408,
                  rope_theta=1e4),
        BatchSpec(4, 8, 32, "uniform", 16, 128),
        seed=1000, granule=16,
        description="tiny LLaMA-style layer, 64-token dense batch"),
    "C2": Config(
        "C2",
        ModelDesc(hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn_inner=14336,
                  rope_theta=5e5),
        BatchSpec(1, 256, 1792, "lognormal", 64, 8192, 1024.0),
        seed=2000, granule=128,
        description="LLaMA-3-8B layer, dense batch 2048"),
    "C3": Config(
        "C3",
        ModelDesc(hidden=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn_inner=28672,
                  rope_theta=1e4),
        BatchSpec(3, 128, 1664, "lognormal", 64, 4096, 1536.0),
        seed=3000, granule=128,
        description="LLaMA-2-70B layer on one GPU, dense batch 2048"),
    "C4": Config(
        "C4",
        ModelDesc(hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn_inner=14336,
                  n_experts=8, top_k=2, rope_theta=1e6),
        BatchSpec(1, 256, 1792, "lognormal", 64, 8192, 1024.0),
        seed=4000, granule=128,
        description="Mixtral-8x7B-style MoE layer, dense batch 2048"),
}


# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit formatting (data representation only)
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, std: float, mean: float = 0.0) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        v = rng.standard_normal(e - s, dtype=np.float32)
        v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        out[s:e] = f32_to_bf16_bits(v)
    return out.reshape(shape)


# ----------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------

def make_weights(m: ModelDesc, seed: int, std: float = 0.02) -> Dict[str, Optional[np.ndarray]]:
    """Random-init bf16 weights ~ N(0, std^2); norm gains ~ 1 + N(0, std^2).

    Layouts (row-major, the contraction dimension contiguous):
      g_attn_norm [D]; w_qkv [Nqkv, D] rows = Q heads, K heads, V heads;
      w_o [D, Hq*dh]; g_ffn_norm [D]; w_gate_up [E, 2I, D] gate rows then up
      rows; w_down [E, D, I]; w_router [E, D] (MoE only).
    """
    rng = np.random.default_rng(seed)
    E = m.experts
    w = {
        "g_attn_norm": _normal_bf16(rng, (m.hidden,), std, 1.0),
        "w_qkv": _normal_bf16(rng, (m.n_qkv, m.hidden), std),
        "w_o": _normal_bf16(rng, (m.hidden, m.q_dim), std),
        "g_ffn_norm": _normal_bf16(rng, (m.hidden,), std, 1.0),
        "w_gate_up": _normal_bf16(rng, (E, 2 * m.ffn_inner, m.hidden), std),
        "w_down": _normal_bf16(rng, (E, m.hidden, m.ffn_inner), std),
        "w_router": _normal_bf16(rng, (E, m.hidden), std) if m.is_moe else None,
    }
    return w


# ----------------------------------------------------------------------------
# dense batch + page table
# ----------------------------------------------------------------------------

@dataclass
class Batch:
    """Token order: prefill requests first (each contiguous), then one token per
    decode request.  ``ctx_len[r]`` counts tokens cached *before* this
    iteration; the request's page list covers ctx_len + q_len tokens."""
    n_tokens: int
    n_prefill_reqs: int
    n_decode_reqs: int
    q_indptr: np.ndarray      # int32 [n_reqs+1]
    ctx_len: np.ndarray       # int32 [n_reqs]
    page_indptr: np.ndarray   # int32 [n_reqs+1]
    page_ids: np.ndarray      # int32 [page_indptr[-1]]
    num_pages: int            # size of the physical page pool

    @property
    def n_reqs(self) -> int:
        return self.n_prefill_reqs + self.n_decode_reqs

    def q_len(self, r: int) -> int:
        return int(self.q_indptr[r + 1] - self.q_indptr[r])


def draw_ctx_lens(spec: BatchSpec, rng: np.random.Generator) -> np.ndarray:
    n = spec.n_decode_reqs
    if spec.ctx_dist == "uniform":
        return rng.integers(spec.ctx_lo, spec.ctx_hi + 1, size=n).astype(np.int32)
    if spec.ctx_dist == "lognormal":
        v = np.exp(rng.normal(np.log(spec.ctx_median), LOGNORMAL_SIGMA, size=n))
        return np.clip(np.rint(v), spec.ctx_lo, spec.ctx_hi).astype(np.int32)
    raise ValueError(spec.ctx_dist)


def make_batch(spec: BatchSpec, seed: int, page_size: int = PAGE_SIZE,
               sort_decode="none", spare_pages: int = 0) -> Batch:
    """Draw context lengths and a fragmented page table.

    Physical page ids are a seeded random permutation of the pool, so the
    pages of one request are scattered (Sec. 4.2.2).  ``sort_decode`` orders
    the decode requests of the batch by context length: "none" (as drawn), "asc"
    or "desc" (True = "desc").  The order of the requests in the dense batch is a
    batch-formation choice; the layer result per request does not depend on it.
    """
    rng = np.random.default_rng(seed)
    dec_ctx = draw_ctx_lens(spec, rng)
    if sort_decode is True:
        sort_decode = "desc"
    if sort_decode in ("asc", "desc"):
        dec_ctx = np.sort(dec_ctx)
        if sort_decode == "desc":
            dec_ctx = dec_ctx[::-1].copy()
    elif sort_decode not in (False, None, "none"):
        raise ValueError(sort_decode)
    q_lens = np.concatenate([np.full(spec.n_prefill_reqs, spec.prefill_len, np.int32),
                             np.ones(spec.n_decode_reqs, np.int32)])
    ctx = np.concatenate([np.full(spec.n_prefill_reqs, spec.prefill_prior, np.int32), dec_ctx])
    return batch_from_lengths(q_lens, ctx, spec.n_prefill_reqs, rng, page_size, spare_pages)


def batch_from_lengths(q_lens, ctx, n_prefill_reqs: int, rng: np.random.Generator,
                       page_size: int = PAGE_SIZE, spare_pages: int = 0) -> Batch:
    q_lens = np.asarray(q_lens, np.int32)
    ctx = np.asarray(ctx, np.int32)
    q_indptr = np.zeros(len(q_lens) + 1, np.int32)
    np.cumsum(q_lens, out=q_indptr[1:])
    n_pages_req = (ctx + q_lens + page_size - 1) // page_size
    page_indptr = np.zeros(len(q_lens) + 1, np.int32)
    np.cumsum(n_pages_req, out=page_indptr[1:])
    total = int(page_indptr[-1])
    num_pages = total + int(spare_pages)
    page_ids = rng.permutation(num_pages)[:total].astype(np.int32)
    return Batch(int(q_indptr[-1]), int(n_prefill_reqs), len(q_lens) - int(n_prefill_reqs),
                 q_indptr, ctx, page_indptr, page_ids, num_pages)


def make_request_stream(n_requests: int, seed: int, prompt_median: float = 512.0, prompt_max: int = 4096,
                        output_median: float = 256.0, output_max: int = 2048) -> "list[tuple[int, int]]":
    """Synthetic request stream of the 32-layer loop configuration: (prompt length, output
    length) pairs, both lognormal with the given medians and the length spread used for the
    contexts of the layer configurations, clipped to [1, max].  Stands in for the paper's
    datasets (only their length statistics matter to the loop)."""
    rng = np.random.default_rng(seed)
    p = np.clip(np.rint(np.exp(rng.normal(np.log(prompt_median), LOGNORMAL_SIGMA, size=n_requests))), 1, prompt_max)
    o = np.clip(np.rint(np.exp(rng.normal(np.log(output_median), LOGNORMAL_SIGMA, size=n_requests))), 1, output_max)
    return [(int(a), int(b)) for a, b in zip(p, o)]


def make_x(n_tokens: int, hidden: int, seed: int) -> np.ndarray:
    """Layer input activations, bf16 ~ N(0,1)."""
    return _normal_bf16(np.random.default_rng(seed), (n_tokens, hidden), 1.0)


def make_kv_pages_host(m: ModelDesc, num_pages: int, seed: int) -> np.ndarray:
    """KV pool [num_pages, page_elems] bf16 ~ N(0,1), generated on the host
    (small configs).  Every slot is filled, including slots past a request's
    context, so a kernel that reads beyond the context is caught."""
    return _normal_bf16(np.random.default_rng(seed), (num_pages, m.page_elems), 1.0)


def page_block_index(head_dim: int, page_size: int = PAGE_SIZE):
    """Index maps of the page block layouts of the library's interface: kidx[t, d] and
    vidx[t, d] give the position of element (token slot t, dimension d) inside the K block
    ([dh/32][16][32]) and the V block ([4][dh/32][16][2][4]).  Data formatting only."""
    assert page_size == 16
    t = np.arange(page_size)[:, None]
    d = np.arange(head_dim)[None, :]
    kidx = ((d // 32) * 16 + t) * 32 + d % 32
    vidx = ((((t // 4) * (head_dim // 32) + d // 32) * 16 + d % 16) * 2 + (d // 16) % 2) * 4 + t % 4
    return kidx, vidx


def subset_batch(b: Batch, reqs) -> "tuple[Batch, np.ndarray, np.ndarray]":
    """Restrict a batch to the listed requests (order kept as given).

    Returns (sub-batch with page ids renumbered 0..n-1, token indices of the
    original batch that were kept, original physical page ids in the order of
    the new numbering).  Requests are independent in a decoder layer, so the
    sub-batch result equals the corresponding rows of the full result.
    """
    reqs = np.asarray(reqs, np.int64)
    tok = np.concatenate([np.arange(b.q_indptr[r], b.q_indptr[r + 1]) for r in reqs]).astype(np.int64)
    phys = np.concatenate([b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]] for r in reqs]).astype(np.int64)
    q_lens = np.array([b.q_len(int(r)) for r in reqs], np.int32)
    n_pages_req = np.array([b.page_indptr[r + 1] - b.page_indptr[r] for r in reqs], np.int32)
    q_indptr = np.zeros(len(reqs) + 1, np.int32)
    np.cumsum(q_lens, out=q_indptr[1:])
    page_indptr = np.zeros(len(reqs) + 1, np.int32)
    np.cumsum(n_pages_req, out=page_indptr[1:])
    n_pf = int(np.sum(reqs < b.n_prefill_reqs))
    assert np.all(reqs[:n_pf] < b.n_prefill_reqs) and np.all(reqs[n_pf:] >= b.n_prefill_reqs), \
        "keep prefill requests first"
    sub = Batch(int(q_indptr[-1]), n_pf, len(reqs) - n_pf, q_indptr, b.ctx_len[reqs].astype(np.int32),
                page_indptr, np.arange(len(phys), dtype=np.int32), len(phys))
    return sub, tok, phys


def config(name: str) -> Config:
    return CONFIGS[name]


def with_batch(cfg: Config, **kw) -> Config:
    return dataclasses.replace(cfg, batch=dataclasses.replace(cfg.batch, **kw))
