"""Thin ctypes binding of libnanoflow.so (the C ABI declared in include/nf.h).

Argument marshalling only: every step of the layer runs in the library's HIP
kernels.  PyTorch is used by callers for device memory and streams; this module
takes raw device pointers (``tensor.data_ptr()``) and ``hipStream_t`` handles.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import json
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnanoflow.so")

NF_OK, NF_EINVAL, NF_ESHAPE, NF_EWORKSPACE, NF_EPAGES, NF_EHIP, NF_EPLAN, NF_ENOMEM, NF_EIO, NF_ESCRATCH = 0, -1, -2, -3, -4, -5, -6, -7, -8, -9
NF_EPI_NONE, NF_EPI_RESIDUAL, NF_EPI_SWIGLU = 0, 1, 2

EXPORTS = [
    "nf_ctx_create", "nf_ctx_destroy", "nf_last_hip_error", "nf_strerror", "nf_ctx_num_cus", "nf_check_batch",
    "nf_ctx_set_trace", "nf_ctx_read_trace", "nf_ctx_lane_stream", "nf_ctx_mask_stream", "nf_tune_set",
    "nf_nano_ops_dependent", "nf_profile", "nf_search_pipeline", "nf_simulate_pipeline", "nf_plan_nanobatches", "nf_plan_manual", "nf_plan_describe", "nf_plan_destroy",
    "nf_workspace_bytes", "nf_plan_workspace_bytes", "nf_workspace_region", "nf_layer_forward",
    "nf_op_rmsnorm", "nf_op_gemm", "nf_gemm_segments", "nf_op_rope_append", "nf_op_attention", "nf_measure_peaks",
    "nf_layers_workspace_bytes", "nf_layers_forward",
    "nf_sched_create", "nf_sched_destroy", "nf_sched_submit", "nf_sched_next_batch", "nf_sched_complete",
    "nf_sched_get_stats", "nf_ctx_set_kv_offload", "nf_op_embedding", "nf_op_argmax", "nf_op_attention_static",
    "nf_attention_static_bytes", "nf_plan_manual_ops", "nf_probe_load_latency", "nf_simulate_pipeline_ops",
    "nf_plan_manual_parts", "nf_simulate_pipeline_parts", "nf_op_move_pages", "nf_plan_search",
]


class nf_model_desc(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn_inner", C.c_int32), ("n_experts", C.c_int32),
                ("top_k", C.c_int32), ("page_size", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float)]


class nf_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g_attn_norm", "w_qkv", "w_o", "g_ffn_norm", "w_gate_up",
                                          "w_down", "w_router")]


class nf_kv_cache(C.Structure):
    _fields_ = [("pages", C.c_void_p), ("num_pages", C.c_int64)]


class nf_batch(C.Structure):
    _fields_ = [("n_tokens", C.c_int32), ("n_prefill_reqs", C.c_int32), ("n_decode_reqs", C.c_int32),
                ("q_indptr", C.c_void_p), ("ctx_len", C.c_void_p), ("page_indptr", C.c_void_p),
                ("page_ids", C.c_void_p), ("host_q_indptr", C.c_void_p), ("host_ctx_len", C.c_void_p),
                ("host_page_indptr", C.c_void_p), ("host_page_ids", C.c_void_p)]


class nf_partitions(C.Structure):
    _fields_ = [("n", C.c_int32 * 5), ("bounds", (C.c_int32 * 9) * 5)]


class nf_pipeline_desc(C.Structure):
    _fields_ = [("n_nano", C.c_int32), ("bounds", C.c_int32 * 9), ("overlap", C.c_int32), ("attn_wgs", C.c_int32),
                ("gemm_tile", C.c_int32), ("reserved", C.c_int32), ("nano_attn_wgs", C.c_int32 * 8),
                ("order", C.c_int32 * 8), ("parts", nf_partitions), ("est_us", C.c_double),
                ("est_us_stage1", C.c_double), ("est_us_unsplit", C.c_double)]


class nf_search_options(C.Structure):
    _fields_ = [("max_nano", C.c_int32), ("granule", C.c_int32), ("layers", C.c_int32), ("rank", C.c_int32),
                ("refine", C.c_int32), ("max_parts", C.c_int32), ("reserved", C.c_int32 * 2)]


class nf_nano_spec(C.Structure):
    _fields_ = [("attn_wgs", C.c_int32), ("gemm_tile", C.c_int32 * 4), ("launch_pos", C.c_int32),
                ("reserved", C.c_int32 * 2)]


class nf_trace_rec(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("op", C.c_int32), ("nano", C.c_int32), ("tok_begin", C.c_int32),
                ("tok_end", C.c_int32), ("start_ms", C.c_float), ("ms", C.c_float)]


KERNEL_NAMES = ["rmsnorm", "gemm", "rope_append", "attention", "attn_merge", "moe_route", "moe_combine"]
OP_NAMES = ["KQV", "ATTN", "O", "UG", "D"]


class NfError(RuntimeError):
    def __init__(self, status: int, where: str, hip: int = 0):
        self.status = status
        self.hip = hip
        msg = lib().nf_strerror(status).decode()
        super().__init__(f"{where}: {msg} (status {status}" + (f", hipError {hip})" if hip else ")"))


_lib = None


def lib() -> C.CDLL:
    """Loads the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -c 'import __graft_entry__ as g; g.build()'` (there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    P = C.POINTER
    L.nf_ctx_create.argtypes = [i32, P(vp)]
    L.nf_ctx_destroy.argtypes = [vp]
    L.nf_ctx_destroy.restype = None
    L.nf_last_hip_error.argtypes = [vp]
    L.nf_strerror.argtypes = [i32]
    L.nf_strerror.restype = C.c_char_p
    L.nf_ctx_num_cus.argtypes = [vp]
    L.nf_ctx_set_trace.argtypes = [vp, i32]
    L.nf_ctx_read_trace.argtypes = [vp, P(nf_trace_rec), i32]
    L.nf_ctx_lane_stream.argtypes = [vp, i32, i32, i32, P(vp)]
    L.nf_ctx_mask_stream.argtypes = [vp, P(C.c_uint32), i32, P(vp)]
    L.nf_tune_set.argtypes = [C.c_char_p, i32]
    L.nf_check_batch.argtypes = [P(nf_model_desc), P(nf_batch), C.c_int64]
    L.nf_profile.argtypes = [vp, P(nf_model_desc), i32, i32, C.c_char_p]
    L.nf_nano_ops_dependent.argtypes = [i32] * 6
    L.nf_search_pipeline.argtypes = [P(nf_model_desc), P(nf_batch), C.c_char_p, i32, i32, P(nf_pipeline_desc)]
    L.nf_simulate_pipeline.argtypes = [P(nf_model_desc), P(nf_batch), C.c_char_p, i32, P(C.c_int32), i32, i32,
                                       P(C.c_double)]
    L.nf_simulate_pipeline_ops.argtypes = [P(nf_model_desc), P(nf_batch), C.c_char_p, i32, P(C.c_int32), P(C.c_int32),
                                           P(C.c_int32), P(C.c_double)]
    L.nf_plan_nanobatches.argtypes = [vp, P(nf_model_desc), P(nf_batch), i32, i32, P(vp)]
    L.nf_plan_search.argtypes = [vp, P(nf_model_desc), P(nf_batch), P(nf_search_options), P(vp)]
    L.nf_plan_manual.argtypes = [vp, P(nf_model_desc), P(nf_batch), i32, P(C.c_int32), i32, i32, i32, i32, P(vp)]
    L.nf_plan_manual_ops.argtypes = [vp, P(nf_model_desc), P(nf_batch), i32, P(C.c_int32), i32, i32, i32,
                                     P(nf_nano_spec), P(vp)]
    L.nf_plan_manual_parts.argtypes = [vp, P(nf_model_desc), P(nf_batch), P(nf_partitions), i32, i32, i32,
                                       P(C.c_int32), P(C.c_int32), P(vp)]
    L.nf_simulate_pipeline_parts.argtypes = [P(nf_model_desc), P(nf_batch), C.c_char_p, P(nf_partitions), i32,
                                             P(C.c_int32), P(C.c_double)]
    L.nf_op_move_pages.argtypes = [vp, sz, C.c_int64, vp, i32, vp, i32, vp]
    L.nf_probe_load_latency.argtypes = [vp, i32, i32, vp, vp]
    L.nf_plan_describe.argtypes = [vp, C.c_char_p, sz]
    L.nf_plan_destroy.argtypes = [vp]
    L.nf_plan_destroy.restype = None
    L.nf_workspace_bytes.argtypes = [P(nf_model_desc), i32, i32]
    L.nf_workspace_bytes.restype = sz
    L.nf_plan_workspace_bytes.argtypes = [vp]
    L.nf_plan_workspace_bytes.restype = sz
    L.nf_workspace_region.argtypes = [vp, C.c_char_p, P(sz), P(sz)]
    L.nf_layer_forward.argtypes = [vp, P(nf_model_desc), P(nf_layer_weights), P(nf_kv_cache), P(nf_batch), vp,
                                   vp, vp, vp, sz, vp]
    L.nf_layers_workspace_bytes.argtypes = [vp, i32]
    L.nf_layers_workspace_bytes.restype = sz
    L.nf_layers_forward.argtypes = [vp, P(nf_model_desc), i32, P(nf_layer_weights), P(nf_kv_cache), P(nf_batch), vp,
                                    vp, vp, vp, sz, vp]
    L.nf_op_rmsnorm.argtypes = [vp, vp, vp, i32, i32, C.c_float, vp]
    L.nf_op_gemm.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp]
    L.nf_gemm_segments.argtypes = [i32, i32, i32]
    L.nf_gemm_segments.restype = i32
    L.nf_op_rope_append.argtypes = [vp, P(nf_model_desc), P(nf_kv_cache), P(nf_batch), vp, vp, i32, i32, vp]
    L.nf_op_attention.argtypes = [vp, P(nf_model_desc), P(nf_kv_cache), P(nf_batch), vp, vp, vp, vp, sz, i32, vp]
    L.nf_op_attention_static.argtypes = [vp, P(nf_model_desc), P(nf_kv_cache), P(nf_batch), vp, vp, vp, i32, vp]
    L.nf_attention_static_bytes.argtypes = []
    L.nf_attention_static_bytes.restype = sz
    _lib = L
    return L


def model_desc(m) -> nf_model_desc:
    return nf_model_desc(m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_inner, m.n_experts, m.top_k,
                         m.page_size, m.rms_eps, m.rope_theta)


def _check(status: int, where: str, ctx: "Optional[Context]" = None):
    if status != NF_OK:
        raise NfError(status, where, lib().nf_last_hip_error(ctx.handle) if ctx is not None else 0)


def _np_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


class Context:
    def __init__(self, device: int = 0):
        h = C.c_void_p()
        _check(lib().nf_ctx_create(device, C.byref(h)), "nf_ctx_create")
        self.handle = h

    @property
    def num_cus(self) -> int:
        return lib().nf_ctx_num_cus(self.handle)

    def lane_stream(self, lane: int, first_cu: int, n_cus: int) -> int:
        h = C.c_void_p()
        _check(lib().nf_ctx_lane_stream(self.handle, lane, first_cu, n_cus, C.byref(h)), "nf_ctx_lane_stream", self)
        return h.value or 0

    def mask_stream(self, cu_bits) -> int:
        """Stream restricted to the listed CU bit indices."""
        words = (self.num_cus + 31) // 32
        mask = (C.c_uint32 * words)()
        for b in cu_bits:
            mask[b >> 5] |= 1 << (b & 31)
        h = C.c_void_p()
        _check(lib().nf_ctx_mask_stream(self.handle, mask, words, C.byref(h)), "nf_ctx_mask_stream", self)
        return h.value or 0

    def set_trace(self, level: int):
        _check(lib().nf_ctx_set_trace(self.handle, int(level)), "nf_ctx_set_trace", self)

    def read_trace(self, max_recs: int = 4096):
        """Waits for the traced kernels and returns a list of dict records."""
        arr = (nf_trace_rec * max_recs)()
        n = lib().nf_ctx_read_trace(self.handle, arr, max_recs)
        _check(min(n, 0), "nf_ctx_read_trace", self)
        return [dict(kernel=KERNEL_NAMES[r.kernel], op=OP_NAMES[r.op], nano=r.nano, tok_begin=r.tok_begin,
                     tok_end=r.tok_end, start_ms=r.start_ms, ms=r.ms) for r in arr[:min(n, max_recs)]]

    def close(self):
        if self.handle:
            lib().nf_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class BatchArgs:
    """nf_batch plus the arrays it points to (kept alive here).

    ``dev`` maps q_indptr / ctx_len / page_indptr / page_ids to device pointers
    (ints); the host mirrors are numpy int32 arrays.
    """

    def __init__(self, n_tokens, n_prefill_reqs, n_decode_reqs, host_q_indptr, host_ctx_len,
                 host_page_indptr, host_page_ids, dev: dict, keepalive=None):
        self.h_q = _np_i32(host_q_indptr)
        self.h_c = _np_i32(host_ctx_len)
        self.h_pi = _np_i32(host_page_indptr)
        self.h_pid = _np_i32(host_page_ids) if host_page_ids is not None else None
        self.keepalive = keepalive
        self.struct = nf_batch(
            int(n_tokens), int(n_prefill_reqs), int(n_decode_reqs),
            dev["q_indptr"], dev["ctx_len"], dev["page_indptr"], dev["page_ids"],
            self.h_q.ctypes.data, self.h_c.ctypes.data, self.h_pi.ctypes.data,
            self.h_pid.ctypes.data if self.h_pid is not None else None)


class Plan:
    def __init__(self, ctx: Context, handle):
        self.ctx = ctx
        self.handle = handle

    def describe(self) -> dict:
        n = lib().nf_plan_describe(self.handle, None, 0)
        _check(min(n, 0), "nf_plan_describe")
        buf = C.create_string_buffer(n + 1)
        lib().nf_plan_describe(self.handle, buf, n + 1)
        return json.loads(buf.value.decode())

    @property
    def workspace_bytes(self) -> int:
        return int(lib().nf_plan_workspace_bytes(self.handle))

    def workspace_region(self, name: str):
        """(offset, bytes) of a named intermediate inside the workspace."""
        off, nb = C.c_size_t(), C.c_size_t()
        _check(lib().nf_workspace_region(self.handle, name.encode(), C.byref(off), C.byref(nb)), "nf_workspace_region")
        return off.value, nb.value

    def close(self):
        if self.handle:
            lib().nf_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def nf_plan_manual(ctx: Context, model, batch: BatchArgs, bounds: Sequence[int], overlap: bool = False,
                   attn_cus: int = 0, gemm_cus: int = 0, attn_wgs: int = 0) -> Plan:
    b = _np_i32(bounds)
    h = C.c_void_p()
    md = model_desc(model)
    _check(lib().nf_plan_manual(ctx.handle, C.byref(md), C.byref(batch.struct), len(b) - 1,
                                b.ctypes.data_as(C.POINTER(C.c_int32)), int(bool(overlap)), int(attn_cus),
                                int(gemm_cus), int(attn_wgs), C.byref(h)), "nf_plan_manual", ctx)
    return Plan(ctx, h)


def nf_plan_manual_ops(ctx: Context, model, batch: BatchArgs, bounds: Sequence[int], overlap: bool,
                       attn_wgs: Sequence[int], gemm_tiles: "Optional[Sequence[Sequence[int]]]" = None,
                       attn_cus: int = 0, gemm_cus: int = 0, launch_pos: "Optional[Sequence[int]]" = None) -> Plan:
    """attn_wgs[i] and gemm_tiles[i] = (KQV, O, Up/Gate, Down) implementations of nano-batch i;
    launch_pos[i] = its position in the launch order (None = index order)."""
    b = _np_i32(bounds)
    n = len(b) - 1
    spec = (nf_nano_spec * n)()
    for i in range(n):
        spec[i].attn_wgs = int(attn_wgs[i])
        spec[i].launch_pos = int(launch_pos[i]) if launch_pos is not None else 0
        for k in range(4):
            spec[i].gemm_tile[k] = int(gemm_tiles[i][k]) if gemm_tiles is not None else 0
    h = C.c_void_p()
    md = model_desc(model)
    _check(lib().nf_plan_manual_ops(ctx.handle, C.byref(md), C.byref(batch.struct), n,
                                    b.ctypes.data_as(C.POINTER(C.c_int32)), int(bool(overlap)), int(attn_cus),
                                    int(gemm_cus), spec, C.byref(h)), "nf_plan_manual_ops", ctx)
    return Plan(ctx, h)


PART_KINDS = ("KQV", "ATTN", "O", "UG", "D")


def _partitions(parts) -> nf_partitions:
    """parts: five boundary lists (KQV, attention, O, Up/Gate, Down) or a dict keyed by PART_KINDS."""
    if isinstance(parts, dict):
        parts = [parts[k] for k in PART_KINDS]
    c = nf_partitions()
    for k in range(5):
        b = [int(v) for v in parts[k]]
        if not 2 <= len(b) <= 9:
            raise ValueError("an operation has 1..8 nano-operations")
        c.n[k] = len(b) - 1
        for i, v in enumerate(b):
            c.bounds[k][i] = v
    return c


def nf_plan_manual_parts(ctx: Context, model, batch: BatchArgs, parts, overlap: bool,
                         attn_wgs: "Optional[Sequence[int]]" = None, gemm_tile: "Optional[Sequence[int]]" = None,
                         attn_cus: int = 0, gemm_cus: int = 0) -> Plan:
    """A partition per operation; attn_wgs[i] = share of attention nano-operation i; gemm_tile = (KQV, O,
    Up/Gate, Down) implementations."""
    c = _partitions(parts)
    w = _np_i32(attn_wgs) if attn_wgs is not None else None
    g = _np_i32(gemm_tile) if gemm_tile is not None else None
    if w is not None and len(w) != c.n[1]:
        raise ValueError("attn_wgs needs one entry per attention nano-operation")
    if g is not None and len(g) != 4:
        raise ValueError("gemm_tile needs four entries")
    h = C.c_void_p()
    md = model_desc(model)
    _check(lib().nf_plan_manual_parts(ctx.handle, C.byref(md), C.byref(batch.struct), C.byref(c), int(bool(overlap)),
                                      int(attn_cus), int(gemm_cus),
                                      w.ctypes.data_as(C.POINTER(C.c_int32)) if w is not None else None,
                                      g.ctypes.data_as(C.POINTER(C.c_int32)) if g is not None else None, C.byref(h)),
           "nf_plan_manual_parts", ctx)
    return Plan(ctx, h)


def nf_simulate_pipeline_parts(model, batch: BatchArgs, parts, overlap: bool,
                               rp_rows: "Optional[Sequence[int]]" = None, profile_path: Optional[str] = None) -> float:
    md = model_desc(model)
    c = _partitions(parts)
    r = _np_i32(rp_rows) if rp_rows is not None else None
    if r is not None and len(r) != c.n[1]:
        raise ValueError("rp_rows needs one entry per attention nano-operation")
    est = C.c_double()
    _check(lib().nf_simulate_pipeline_parts(C.byref(md), C.byref(batch.struct),
                                            profile_path.encode() if profile_path else None, C.byref(c),
                                            int(bool(overlap)),
                                            r.ctypes.data_as(C.POINTER(C.c_int32)) if r is not None else None,
                                            C.byref(est)), "nf_simulate_pipeline_parts")
    return est.value


def nf_plan_nanobatches(ctx: Context, model, batch: BatchArgs, max_nano: int = 0, granule: int = 128) -> Plan:
    h = C.c_void_p()
    md = model_desc(model)
    _check(lib().nf_plan_nanobatches(ctx.handle, C.byref(md), C.byref(batch.struct), int(max_nano), int(granule),
                                     C.byref(h)), "nf_plan_nanobatches", ctx)
    return Plan(ctx, h)


def nf_plan_search(ctx: Context, model, batch: BatchArgs, max_nano: int = 0, granule: int = 128, layers: int = 1,
                   rank: int = 0, refine: int = 2, max_parts: int = 0) -> Plan:
    """nf_plan_nanobatches with the search's knobs given here instead of through nf_tune_set."""
    h = C.c_void_p()
    md = model_desc(model)
    opt = nf_search_options(int(max_nano), int(granule), int(layers), int(rank), int(refine), int(max_parts))
    _check(lib().nf_plan_search(ctx.handle, C.byref(md), C.byref(batch.struct), C.byref(opt), C.byref(h)),
           "nf_plan_search", ctx)
    return Plan(ctx, h)


def nf_search_pipeline(model, batch: BatchArgs, profile_path: Optional[str] = None, max_nano: int = 0,
                       granule: int = 128) -> dict:
    md = model_desc(model)
    out = nf_pipeline_desc()
    _check(lib().nf_search_pipeline(C.byref(md), C.byref(batch.struct), profile_path.encode() if profile_path else None,
                                    int(max_nano), int(granule), C.byref(out)), "nf_search_pipeline")
    return dict(bounds=[int(out.bounds[i]) for i in range(out.n_nano + 1)], overlap=int(out.overlap),
                attn_wgs=int(out.attn_wgs), gemm_tile=int(out.gemm_tile), est_us=out.est_us, est_us_stage1=out.est_us_stage1,
                est_us_unsplit=out.est_us_unsplit, nano_attn_wgs=[int(out.nano_attn_wgs[i]) for i in range(out.n_nano)],
                order=[int(out.order[i]) for i in range(out.n_nano)],
                parts=[[int(out.parts.bounds[k][i]) for i in range(out.parts.n[k] + 1)] for k in range(5)]
                if out.parts.n[0] > 0 else None)


def nf_simulate_pipeline(model, batch: BatchArgs, bounds: Sequence[int], overlap: bool, rp_row: int = -1,
                         profile_path: Optional[str] = None) -> float:
    md = model_desc(model)
    b = _np_i32(bounds)
    est = C.c_double()
    _check(lib().nf_simulate_pipeline(C.byref(md), C.byref(batch.struct), profile_path.encode() if profile_path else None,
                                      len(b) - 1, b.ctypes.data_as(C.POINTER(C.c_int32)), int(bool(overlap)),
                                      int(rp_row), C.byref(est)), "nf_simulate_pipeline")
    return est.value


def nf_simulate_pipeline_ops(model, batch: BatchArgs, bounds: Sequence[int], rp_rows: Sequence[int],
                             order: Optional[Sequence[int]], profile_path: str) -> float:
    md = model_desc(model)
    b, r = _np_i32(bounds), _np_i32(rp_rows)
    o = _np_i32(order) if order is not None else None
    est = C.c_double()
    _check(lib().nf_simulate_pipeline_ops(C.byref(md), C.byref(batch.struct), profile_path.encode(), len(b) - 1,
                                          b.ctypes.data_as(C.POINTER(C.c_int32)), r.ctypes.data_as(C.POINTER(C.c_int32)),
                                          o.ctypes.data_as(C.POINTER(C.c_int32)) if o is not None else None,
                                          C.byref(est)), "nf_simulate_pipeline_ops")
    return est.value


def nf_profile(ctx: Context, model, max_tokens: int, granule: int = 128, cache_path: Optional[str] = None):
    md = model_desc(model)
    _check(lib().nf_profile(ctx.handle, C.byref(md), int(max_tokens), int(granule),
                            cache_path.encode() if cache_path else None), "nf_profile", ctx)


class nf_peaks(C.Structure):
    _fields_ = [("mfma_bf16_tflops", C.c_double), ("mfma_bf16_tflops_zero_operands", C.c_double),
                ("hbm_read_gbs", C.c_double), ("n_cus", C.c_int32), ("reserved", C.c_int32)]


def nf_measure_peaks(ctx: Context) -> dict:
    """Measured MFMA and HBM ceilings of the device (about a second of GPU time, 4 GiB of scratch)."""
    pk = nf_peaks()
    _check(lib().nf_measure_peaks(ctx.handle, C.byref(pk)), "nf_measure_peaks", ctx)
    return {"mfma_bf16_tflops": pk.mfma_bf16_tflops,
            "mfma_bf16_tflops_zero_operands": pk.mfma_bf16_tflops_zero_operands,
            "hbm_read_gbs": pk.hbm_read_gbs, "n_cus": pk.n_cus}


def nf_op_embedding(token_ids_ptr, from_slot_ptr, slot_tokens_ptr, table_ptr, table_rows, out_ptr, n_rows, width,
                    stream=0):
    f = lib().nf_op_embedding
    f.argtypes = [C.c_void_p] * 4 + [C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    _check(f(token_ids_ptr, from_slot_ptr, slot_tokens_ptr, table_ptr, int(table_rows), out_ptr, int(n_rows),
             int(width), stream), "nf_op_embedding")


def nf_op_move_pages(pool_ptr, page_bytes, num_pages, page_ids_ptr, n_pages, staging_ptr, scatter, stream=0):
    """Gather (scatter = False) pool pages into a contiguous device buffer, or scatter them back."""
    _check(lib().nf_op_move_pages(pool_ptr, int(page_bytes), int(num_pages), page_ids_ptr, int(n_pages), staging_ptr,
                                  int(bool(scatter)), stream), "nf_op_move_pages")


def nf_op_argmax(logits_ptr, n_rows, vocab, out_index_ptr, out_ptr, stream=0):
    f = lib().nf_op_argmax
    f.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
    _check(f(logits_ptr, int(n_rows), int(vocab), out_index_ptr, out_ptr, stream), "nf_op_argmax")


def nf_ctx_set_kv_offload(ctx: Context, host_ptr: Optional[int], layer_stride_bytes: int = 0):
    """Switches the simultaneous KV offload on (host_ptr = address of pinned host memory) or off (None)."""
    f = lib().nf_ctx_set_kv_offload
    f.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
    _check(f(ctx.handle, host_ptr, int(layer_stride_bytes)), "nf_ctx_set_kv_offload", ctx)


def nf_tune_set(key: str, value: int):
    _check(lib().nf_tune_set(key.encode(), int(value)), "nf_tune_set")


def nf_check_batch(model, batch: BatchArgs, num_pages: int) -> int:
    """Returns the status code (no exception): host-only validation."""
    md = model_desc(model)
    return int(lib().nf_check_batch(C.byref(md), C.byref(batch.struct), int(num_pages)))


def nf_workspace_bytes(model, max_tokens: int, max_context: int) -> int:
    md = model_desc(model)
    return int(lib().nf_workspace_bytes(C.byref(md), int(max_tokens), int(max_context)))


def weights_struct(ptrs: dict) -> nf_layer_weights:
    return nf_layer_weights(*[ptrs.get(n) for n, _ in nf_layer_weights._fields_])


def nf_layer_forward(ctx: Context, model, weights: nf_layer_weights, pages_ptr: int, num_pages: int,
                     batch: BatchArgs, plan: Optional[Plan], x_in_ptr: int, x_out_ptr: int, workspace_ptr: int,
                     workspace_bytes: int, stream: int = 0):
    md = model_desc(model)
    kv = nf_kv_cache(pages_ptr, int(num_pages))
    _check(lib().nf_layer_forward(ctx.handle, C.byref(md), C.byref(weights), C.byref(kv), C.byref(batch.struct),
                                  plan.handle if plan is not None else None, x_in_ptr, x_out_ptr, workspace_ptr,
                                  int(workspace_bytes), stream), "nf_layer_forward", ctx)


def nf_layers_workspace_bytes(plan: Plan, n_layers: int) -> int:
    return int(lib().nf_layers_workspace_bytes(plan.handle, int(n_layers)))


def nf_layers_forward(ctx: Context, model, weights: "list[nf_layer_weights]", pages_ptrs: "list[int]", num_pages: int,
                      batch: BatchArgs, plan: Plan, x_in_ptr: int, x_out_ptr: int, workspace_ptr: int,
                      workspace_bytes: int, stream: int = 0):
    """n consecutive layers (layer l uses weights[l] and the pool at pages_ptrs[l]) with one plan."""
    n = len(weights)
    if len(pages_ptrs) != n:
        raise ValueError("one KV pool per layer")
    md = model_desc(model)
    w_arr = (nf_layer_weights * n)(*weights)
    kv_arr = (nf_kv_cache * n)(*[nf_kv_cache(p, int(num_pages)) for p in pages_ptrs])
    _check(lib().nf_layers_forward(ctx.handle, C.byref(md), n, w_arr, kv_arr, C.byref(batch.struct), plan.handle,
                                   x_in_ptr, x_out_ptr, workspace_ptr, int(workspace_bytes), stream),
           "nf_layers_forward", ctx)


def nf_op_rmsnorm(x_ptr, g_ptr, out_ptr, n_tokens, hidden, eps, stream=0):
    _check(lib().nf_op_rmsnorm(x_ptr, g_ptr, out_ptr, int(n_tokens), int(hidden), float(eps), stream), "nf_op_rmsnorm")


def nf_gemm_segments(N: int, K: int, epilogue: int = NF_EPI_NONE) -> int:
    return int(lib().nf_gemm_segments(int(N), int(K), int(epilogue)))


def nf_op_gemm(x_ptr, w_ptr, out_ptr, residual_ptr, M, N, K, epilogue=NF_EPI_NONE, stream=0):
    _check(lib().nf_op_gemm(x_ptr, w_ptr, out_ptr, residual_ptr, int(M), int(N), int(K), int(epilogue), stream),
           "nf_op_gemm")


def nf_op_rope_append(ctx, model, pages_ptr, num_pages, batch: BatchArgs, plan: Plan, qkv_ptr, tok_begin, tok_end,
                      stream=0):
    md = model_desc(model)
    kv = nf_kv_cache(pages_ptr, int(num_pages))
    _check(lib().nf_op_rope_append(ctx.handle, C.byref(md), C.byref(kv), C.byref(batch.struct), plan.handle, qkv_ptr,
                                   int(tok_begin), int(tok_end), stream), "nf_op_rope_append", ctx)


def nf_op_attention(ctx, model, pages_ptr, num_pages, batch: BatchArgs, plan: Plan, qkv_ptr, attn_out_ptr,
                    workspace_ptr, workspace_bytes, nano_index=0, stream=0):
    md = model_desc(model)
    kv = nf_kv_cache(pages_ptr, int(num_pages))
    _check(lib().nf_op_attention(ctx.handle, C.byref(md), C.byref(kv), C.byref(batch.struct), plan.handle, qkv_ptr,
                                 attn_out_ptr, workspace_ptr, int(workspace_bytes), int(nano_index), stream),
           "nf_op_attention", ctx)


def nf_probe_load_latency(ctx: Context, n_workgroups: int, iters: int, out_ptr: int, stream=0):
    _check(lib().nf_probe_load_latency(ctx.handle, int(n_workgroups), int(iters), out_ptr, stream),
           "nf_probe_load_latency", ctx)


def nf_attention_static_bytes() -> int:
    return int(lib().nf_attention_static_bytes())


def nf_op_attention_static(ctx, model, pages_ptr, num_pages, batch: BatchArgs, plan: Plan, qkv_ptr, attn_out_ptr,
                           nano_index=0, stream=0):
    md = model_desc(model)
    kv = nf_kv_cache(pages_ptr, int(num_pages))
    _check(lib().nf_op_attention_static(ctx.handle, C.byref(md), C.byref(kv), C.byref(batch.struct), plan.handle,
                                        qkv_ptr, attn_out_ptr, int(nano_index), stream), "nf_op_attention_static", ctx)


# ------------------------------------------------------------ continuous batching ---

class nf_sched_config(C.Structure):
    _fields_ = [("dense_batch", C.c_int32), ("page_size", C.c_int32), ("num_pages", C.c_int64),
                ("max_requests", C.c_int32), ("max_chunk", C.c_int32), ("reserve_pages", C.c_int32),
                ("avg_decode_len", C.c_float)]


class nf_sched_batch(C.Structure):
    _I32P, _I64P = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    _fields_ = [("iteration", C.c_int64), ("n_tokens", C.c_int32), ("n_prefill_reqs", C.c_int32),
                ("n_decode_reqs", C.c_int32), ("q_indptr", _I32P), ("ctx_len", _I32P), ("page_indptr", _I32P),
                ("page_ids", _I32P), ("request_ids", _I64P),
                ("n_swap_out", C.c_int32), ("swap_out_req", _I64P), ("swap_out_indptr", _I32P),
                ("swap_out_pages", _I32P),
                ("n_swap_in", C.c_int32), ("swap_in_req", _I64P), ("swap_in_indptr", _I32P), ("swap_in_pages", _I32P),
                ("n_released", C.c_int32), ("released_req", _I64P),
                ("n_finished", C.c_int32), ("finished_req", _I64P)]


class nf_sched_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "iterations_formed", "iterations_completed", "submitted", "finished", "waiting", "resident", "swapped",
        "prefill_tokens", "decode_tokens", "wasted_decode_tokens", "swap_outs", "swap_ins", "free_pages")] + [
        ("avg_decode_len", C.c_double)]


def _np_from(ptr, n, dtype):
    if n <= 0:
        return np.zeros(0, dtype)
    return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dtype, copy=True)


class FormedBatch:
    """Host copy of one batch formed by the scheduler."""

    def __init__(self, b: nf_sched_batch):
        n = b.n_prefill_reqs + b.n_decode_reqs
        self.iteration = int(b.iteration)
        self.n_tokens, self.n_prefill_reqs, self.n_decode_reqs = int(b.n_tokens), int(b.n_prefill_reqs), int(b.n_decode_reqs)
        self.q_indptr = _np_from(b.q_indptr, n + 1, np.int32)
        self.ctx_len = _np_from(b.ctx_len, n, np.int32)
        self.page_indptr = _np_from(b.page_indptr, n + 1, np.int32)
        self.page_ids = _np_from(b.page_ids, int(self.page_indptr[-1]) if n else 0, np.int32)
        self.request_ids = _np_from(b.request_ids, n, np.int64)

        def groups(cnt, req, indptr, pages):
            req = _np_from(req, cnt, np.int64)
            ip = _np_from(indptr, cnt + 1, np.int32)
            pg = _np_from(pages, int(ip[-1]) if cnt else 0, np.int32)
            return [(int(req[i]), pg[ip[i]:ip[i + 1]].copy()) for i in range(cnt)]
        self.swap_out = groups(b.n_swap_out, b.swap_out_req, b.swap_out_indptr, b.swap_out_pages)
        self.swap_in = groups(b.n_swap_in, b.swap_in_req, b.swap_in_indptr, b.swap_in_pages)
        self.released = [int(x) for x in _np_from(b.released_req, b.n_released, np.int64)]
        self.finished = [int(x) for x in _np_from(b.finished_req, b.n_finished, np.int64)]


class Scheduler:
    """Continuous-batching scheduler of the library (host only)."""

    def __init__(self, dense_batch: int, page_size: int, num_pages: int, max_requests: int, max_chunk: int = 0,
                 reserve_pages: int = 0, avg_decode_len: float = 256.0):
        L = lib()
        L.nf_sched_create.argtypes = [C.POINTER(nf_sched_config), C.POINTER(C.c_void_p)]
        L.nf_sched_destroy.argtypes = [C.c_void_p]
        L.nf_sched_destroy.restype = None
        L.nf_sched_submit.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int64)]
        L.nf_sched_next_batch.argtypes = [C.c_void_p, C.POINTER(nf_sched_batch)]
        L.nf_sched_complete.argtypes = [C.c_void_p, C.c_int64]
        L.nf_sched_get_stats.argtypes = [C.c_void_p, C.POINTER(nf_sched_stats)]
        cfg = nf_sched_config(int(dense_batch), int(page_size), int(num_pages), int(max_requests), int(max_chunk),
                              int(reserve_pages), float(avg_decode_len))
        h = C.c_void_p()
        _check(L.nf_sched_create(C.byref(cfg), C.byref(h)), "nf_sched_create")
        self.handle = h

    def submit(self, prompt_len: int, output_len: int) -> int:
        rid = C.c_int64()
        _check(lib().nf_sched_submit(self.handle, int(prompt_len), int(output_len), C.byref(rid)), "nf_sched_submit")
        return int(rid.value)

    def next_batch(self) -> FormedBatch:
        b = nf_sched_batch()
        _check(lib().nf_sched_next_batch(self.handle, C.byref(b)), "nf_sched_next_batch")
        return FormedBatch(b)

    def complete(self, iteration: int):
        _check(lib().nf_sched_complete(self.handle, int(iteration)), "nf_sched_complete")

    def stats(self) -> dict:
        st = nf_sched_stats()
        _check(lib().nf_sched_get_stats(self.handle, C.byref(st)), "nf_sched_get_stats")
        return {n: getattr(st, n) for n, _ in nf_sched_stats._fields_}

    def close(self):
        if self.handle:
            lib().nf_sched_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
