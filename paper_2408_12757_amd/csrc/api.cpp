// C ABI: context management, workspace layout, and the nano-operation executor that
// enqueues the layer's kernels on the caller's stream or on the two lane streams
// (paper Sec. 5: nano-operations are launched in the searched order and their
// dependencies are enforced with events).
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "nf_internal.h"

// ------------------------------------------------------------------ context ---

extern "C" int nf_ctx_create(int device, nf_ctx** out) try {
  if (!out) return NF_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return NF_EHIP;
  nf_ctx* c = new (std::nothrow) nf_ctx();
  if (!c) return NF_ENOMEM;
  c->device = device;
  hipError_t e = hipSetDevice(device);
  hipDeviceProp_t prop;
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
  if (e != hipSuccess) {
    delete c;
    return NF_EHIP;
  }
  c->num_cus = prop.multiProcessorCount;
  // the device address of the static scratch array, looked up with this device current
  e = nf_attention_static_scratch(device, &c->static_parts, &c->static_parts_bytes);
  if (e != hipSuccess) {
    delete c;
    return NF_EHIP;
  }
  *out = c;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" void nf_ctx_destroy(nf_ctx* ctx) {
  if (!ctx) return;
  for (auto& t : ctx->trace) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  for (hipEvent_t e : ctx->event_pool) (void)hipEventDestroy(e);
  for (auto& kv : ctx->streams) (void)hipStreamDestroy(kv.second);
  for (hipEvent_t e : ctx->offload_events) (void)hipEventDestroy(e);
  for (auto& r : ctx->retired_plans) {
    (void)hipEventSynchronize(r.second);
    (void)hipEventDestroy(r.second);
    nf_plan_destroy(r.first);
  }
  // the caller must have drained the streams it used with this context
  if (ctx->null_plan) nf_plan_destroy(ctx->null_plan);
  if (ctx->offload_stream) (void)hipStreamDestroy(ctx->offload_stream);
  nf_profile_free(ctx);
  delete ctx;
}

extern "C" int nf_last_hip_error(const nf_ctx* ctx) { return ctx ? ctx->last_hip : 0; }
extern "C" int nf_ctx_num_cus(const nf_ctx* ctx) { return ctx ? ctx->num_cus : 0; }

extern "C" const char* nf_strerror(int status) {
  switch (status) {
    case NF_OK: return "ok";
    case NF_EINVAL: return "invalid argument";
    case NF_ESHAPE: return "unsupported model or batch shape";
    case NF_EWORKSPACE: return "workspace too small";
    case NF_EPAGES: return "page table does not cover the batch";
    case NF_EHIP: return "HIP call failed";
    case NF_EPLAN: return "plan does not match the batch or is malformed";
    case NF_ENOMEM: return "host allocation failed";
    case NF_EIO: return "profile cache i/o failed";
    case NF_ESCRATCH: return "problem exceeds the built-in scratch of the allocation-free entry point";
    default: return "unknown status";
  }
}

// Lane streams, one per (lane, CU range).  n_cus = 0: an ordinary non-blocking stream.
// Otherwise a stream whose kernels may only run on CU bits [first_cu, first_cu + n_cus)
// of the device's CU mask.
int nf_get_lane_stream(nf_ctx* ctx, int lane, int first_cu, int n_cus, hipStream_t* out) {
  if (n_cus < 0 || first_cu < 0 || first_cu + n_cus > ctx->num_cus) return NF_EINVAL;
  const long key = ((long)lane << 40) | ((long)first_cu << 20) | (long)n_cus;
  auto it = ctx->streams.find(key);
  if (it != ctx->streams.end()) {
    *out = it->second;
    return NF_OK;
  }
  hipStream_t s = nullptr;
  if (n_cus == 0) {
    NF_HIP(ctx, hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
  } else {
    const int words = (ctx->num_cus + 31) / 32;
    std::vector<uint32_t> mask((size_t)words, 0u);
    for (int b = first_cu; b < first_cu + n_cus; ++b) mask[b >> 5] |= 1u << (b & 31);
    NF_HIP(ctx, hipExtStreamCreateWithCUMask(&s, (uint32_t)words, mask.data()));
  }
  ctx->streams[key] = s;
  *out = s;
  return NF_OK;
}

extern "C" int nf_ctx_lane_stream(nf_ctx* ctx, int lane, int first_cu, int n_cus, void** out) {
  if (!ctx || !out || lane < 0 || lane >= NF_LANES) return NF_EINVAL;
  hipStream_t s = nullptr;
  int rc = nf_get_lane_stream(ctx, lane, first_cu, n_cus, &s);
  *out = (void*)s;
  return rc;
}

extern "C" int nf_ctx_mask_stream(nf_ctx* ctx, const uint32_t* mask, int words, void** out) {
  if (!ctx || !out || !mask || words < 1 || words > 32) return NF_EINVAL;
  hipStream_t s = nullptr;
  NF_HIP(ctx, hipExtStreamCreateWithCUMask(&s, (uint32_t)words, mask));
  ctx->streams[(7L << 40) + (long)ctx->streams.size()] = s;
  *out = (void*)s;
  return NF_OK;
}

extern "C" int nf_tune_set(const char* key, int value) {
  if (!key) return NF_EINVAL;
  if (!strcmp(key, "attention.variant")) {
    if (value < 0 || value > 7) return NF_EINVAL;
    nf_set_attention_variant(value);
    return NF_OK;
  }
  if (!strcmp(key, "offload.dma")) {
    if (value < 0 || value > 1) return NF_EINVAL;
    nf_set_offload_dma(value);
    return NF_OK;
  }
  if (!strcmp(key, "search.rank")) {
    if (value < 0 || value > 64) return NF_EINVAL;
    nf_set_search_rank(value);
    return NF_OK;
  }
  if (!strcmp(key, "search.refine")) {
    if (value < 0 || value > 2) return NF_EINVAL;
    nf_set_search_refine(value);
    return NF_OK;
  }
  if (!strcmp(key, "search.max_parts")) {
    if (value < 0 || value > 8) return NF_EINVAL;
    nf_set_search_max_parts(value);
    return NF_OK;
  }
  if (!strcmp(key, "search.layers")) {
    if (value < 1 || value > 16) return NF_EINVAL;
    nf_set_search_layers(value);
    return NF_OK;
  }
  if (!strcmp(key, "gemm.grouped_tile")) {
    if (value != 0 && value != 1 && value != 7 && value != 9 && value != 11 && value != 12 && value != 13 && value != 19 &&
        value != 21)
      return NF_EINVAL;
    nf_set_grouped_gemm_tile(value);
    return NF_OK;
  }
  if (!strcmp(key, "gemm.ksplit")) {
    if (value < 0 || value > 2) return NF_EINVAL;
    nf_set_gemm_ksplit(value);
    return NF_OK;
  }
  if (!strcmp(key, "gemm.tile")) {
    if (value < 0 || value > 25) return NF_EINVAL;
    nf_set_gemm_tile(value);
    return NF_OK;
  }
  return NF_EINVAL;
}

extern "C" int nf_ctx_set_kv_offload(nf_ctx* ctx, void* host_rows, size_t layer_stride_bytes) {
  if (!ctx) return NF_EINVAL;
  if (host_rows && (layer_stride_bytes % 16 != 0 || ((uintptr_t)host_rows & 15) != 0)) return NF_EINVAL;
  if (host_rows && !ctx->offload_stream) {
    NF_HIP(ctx, hipSetDevice(ctx->device));
    NF_HIP(ctx, hipStreamCreateWithFlags(&ctx->offload_stream, hipStreamNonBlocking));
  }
  ctx->offload_host = host_rows;
  ctx->offload_layer_stride = host_rows ? layer_stride_bytes : 0;
  return NF_OK;
}

// ---------------------------------------------------------------- workspace ---

namespace {

struct Workspace {
  char* h;     // [B, D]   normalised activations (both norms)
  char* qkv;   // [B, Nqkv]
  char* attn;  // [B, Hq*dh]
  char* y;     // [B, D]   x + attention block
  char* f;     // [B*k, I] silu(gate) * up  (k = 1 dense, top_k for experts: rows sorted by expert)
  float* parts;
  // mixture of experts only
  int32_t* expert_ids;     // [B, k]
  float* expert_w;         // [B, k]
  int32_t* slot_of;        // [B, k] sorted row of (token, k)
  int32_t* row_token;      // [B*k]  token of a sorted row
  int32_t* expert_offset;  // [NF_MAX_NANO_OFFSETS][E + 1] per nano-batch
  char* expert_out;        // [B*k, D]
  float* expert_partial;   // [2][B*k, D] fp32 sums of the K halves when the experts' down projection has two segments
  // dense models whose down projection is a two-segment operation: [2][B, D] fp32 sums of the
  // two K halves, for nano-batches that run the halves on different workgroups
  float* down_partial;
  size_t total;
};

constexpr int kMaxNanoOffsets = 64;

Workspace layout_workspace(const nf_model_desc* m, int n_tokens, size_t n_parts, char* base) {
  Workspace w;
  const size_t B = (size_t)std::max(1, n_tokens);
  const size_t nqkv = (size_t)(m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base + off;
    off += nf_align256(bytes);
    return p;
  };
  w.h = take(B * m->hidden * 2);
  w.qkv = take(B * nqkv * 2);
  w.attn = take(B * (size_t)m->n_q_heads * m->head_dim * 2);
  w.y = take(B * m->hidden * 2);
  const bool moe = m->n_experts > 1;
  const size_t k = moe ? (size_t)m->top_k : 1;
  w.f = take(B * k * (size_t)m->ffn_inner * 2);
  w.parts = (float*)take(n_parts * m->n_kv_heads * nf_attn_part_floats(m->head_dim) * sizeof(float));
  w.expert_ids = (int32_t*)take(moe ? B * k * 4 : 0);
  w.expert_w = (float*)take(moe ? B * k * 4 : 0);
  w.slot_of = (int32_t*)take(moe ? B * k * 4 : 0);
  w.row_token = (int32_t*)take(moe ? B * k * 4 : 0);
  w.expert_offset = (int32_t*)take(moe ? (size_t)kMaxNanoOffsets * (m->n_experts + 1) * 4 : 0);
  const bool moe_two_seg = moe && nf_gemm_k_segments(m->hidden, m->ffn_inner, NF_EPI_NONE) == 2;
  w.expert_out = take(moe && !moe_two_seg ? B * k * (size_t)m->hidden * 2 : 0);
  w.expert_partial = moe_two_seg ? (float*)take(2 * B * k * (size_t)m->hidden * sizeof(float)) : nullptr;
  const bool two_seg = !moe && nf_gemm_k_segments(m->hidden, m->ffn_inner, NF_EPI_RESIDUAL) == 2;
  w.down_partial = two_seg ? (float*)take(2 * B * m->hidden * sizeof(float)) : nullptr;
  w.total = off;
  return w;
}

size_t max_parts_bound(const nf_model_desc* m, int max_tokens, int max_context) {
  const size_t per_group = ((size_t)std::max(0, max_context) + 16 + NF_ATTN_CHUNK - 1) / NF_ATTN_CHUNK + 1;
  return (size_t)std::max(1, max_tokens) * per_group;
}

}  // namespace

extern "C" size_t nf_workspace_bytes(const nf_model_desc* model, int max_tokens, int max_context) {
  if (nf_validate_model(model) != NF_OK || max_tokens < 0) return 0;
  return layout_workspace(model, max_tokens, max_parts_bound(model, max_tokens, max_context), nullptr).total;
}

extern "C" size_t nf_plan_workspace_bytes(const nf_plan* plan) {
  if (!plan) return 0;
  return layout_workspace(&plan->model, plan->n_tokens, (size_t)std::max(1, plan->total_parts), nullptr).total;
}

extern "C" int nf_workspace_region(const nf_plan* plan, const char* name, size_t* offset, size_t* bytes) {
  if (!plan || !name || !offset || !bytes) return NF_EINVAL;
  const nf_model_desc* m = &plan->model;
  const Workspace w = layout_workspace(m, plan->n_tokens, (size_t)std::max(1, plan->total_parts), nullptr);
  const size_t B = (size_t)plan->n_tokens, k = m->n_experts > 1 ? (size_t)m->top_k : 1;
  const size_t nqkv = (size_t)(m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
  struct {
    const char* n;
    const void* p;
    size_t b;
  } tab[] = {{"h", w.h, B * m->hidden * 2},
             {"qkv", w.qkv, B * nqkv * 2},
             {"attn", w.attn, B * (size_t)m->n_q_heads * m->head_dim * 2},
             {"y", w.y, B * m->hidden * 2},
             {"f", w.f, B * k * m->ffn_inner * 2},
             {"moe.expert_ids", w.expert_ids, m->n_experts > 1 ? B * k * 4 : 0},
             {"moe.expert_w", w.expert_w, m->n_experts > 1 ? B * k * 4 : 0},
             {"moe.slot_of", w.slot_of, m->n_experts > 1 ? B * k * 4 : 0}};
  for (auto& t : tab) {
    if (!strcmp(t.n, name)) {
      *offset = (size_t)reinterpret_cast<uintptr_t>(t.p);  // laid out from a null base: the address is the offset
      *bytes = t.b;
      return NF_OK;
    }
  }
  return NF_EINVAL;
}

// -------------------------------------------------------------------- trace ---

extern "C" int nf_ctx_set_trace(nf_ctx* ctx, int level) {
  if (!ctx || level < 0 || level > 2) return NF_EINVAL;
  ctx->trace_level = level;
  return NF_OK;
}

extern "C" int nf_ctx_read_trace(nf_ctx* ctx, nf_trace_rec* recs, int max_recs) try {
  if (!ctx || max_recs < 0 || (max_recs > 0 && !recs)) return NF_EINVAL;
  const int n = (int)ctx->trace.size();
  for (int i = 0; i < n; ++i) {
    NfTraceSlot& t = ctx->trace[i];
    NF_HIP(ctx, hipEventSynchronize(t.stop));
    NF_HIP(ctx, hipEventElapsedTime(&t.rec.ms, t.start, t.stop));
    NF_HIP(ctx, hipEventSynchronize(t.start));
    NF_HIP(ctx, hipEventElapsedTime(&t.rec.start_ms, ctx->trace[0].start, t.start));
    if (i < max_recs) recs[i] = t.rec;
  }
  for (auto& t : ctx->trace) {
    ctx->event_pool.push_back(t.start);
    ctx->event_pool.push_back(t.stop);
  }
  ctx->trace.clear();
  return n;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

// ----------------------------------------------------------------- executor ---

namespace {

hipError_t trace_event(nf_ctx* ctx, hipEvent_t* e) {
  if (!ctx->event_pool.empty()) {
    *e = ctx->event_pool.back();
    ctx->event_pool.pop_back();
    return hipSuccess;
  }
  return hipEventCreate(e);
}

// Brackets the kernels launched by `fn` with timing events when the trace level asks for it.
template <typename F>
hipError_t traced(nf_ctx* ctx, int kernel, const NfNanoOp& op, hipStream_t s, F fn) {
  const bool on = ctx->trace_level >= 2 || (ctx->trace_level == 1 && kernel == NF_K_ATTENTION);
  if (!on) return fn();
  NfTraceSlot t;
  t.rec = nf_trace_rec{kernel, op.kind, op.nano, op.tok_begin, op.tok_end, 0.f, 0.f};
  hipError_t e = trace_event(ctx, &t.start);
  if (e != hipSuccess) return e;
  e = trace_event(ctx, &t.stop);
  if (e != hipSuccess) return e;
  e = hipEventRecord(t.start, s);
  if (e != hipSuccess) return e;
  e = fn();
  if (e != hipSuccess) return e;
  e = hipEventRecord(t.stop, s);
  ctx->trace.push_back(t);
  return e;
}

struct LayerArgs {
  const nf_model_desc* m;
  const nf_layer_weights* w;
  nf_kv_cache* kv;
  const nf_batch* b;
  const char* x_in;
  char* x_out;
  Workspace ws;
};

hipError_t launch_nano_op(nf_ctx* ctx, const nf_plan* p, const NfNanoOp& op, const LayerArgs& a, hipStream_t s) {
  const nf_model_desc* m = a.m;
  const int t0 = op.tok_begin, M = op.tok_end - op.tok_begin;
  if (M <= 0) return hipSuccess;
  const size_t D = m->hidden, I = m->ffn_inner;
  const size_t nqkv = (size_t)(m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
  const size_t qdim = (size_t)m->n_q_heads * m->head_dim;
  hipError_t e = hipSuccess;
  switch (op.kind) {
    case NF_OP_KQV:
      e = traced(ctx, NF_K_RMSNORM, op, s, [&] {
        return nf_launch_rmsnorm(a.x_in + t0 * D * 2, a.w->g_attn_norm, a.ws.h + t0 * D * 2, M, (int)D, m->rms_eps, s);
      });
      if (e != hipSuccess) return e;
      e = traced(ctx, NF_K_GEMM, op, s, [&] {
        return nf_launch_gemm(a.ws.h + t0 * D * 2, a.w->w_qkv, a.ws.qkv + t0 * nqkv * 2, nullptr, M, (int)nqkv, (int)D,
                              NF_EPI_NONE, op.gemm_tile, s);
      });
      if (e != hipSuccess) return e;
      return traced(ctx, NF_K_ROPE_APPEND, op, s, [&] {
        return nf_launch_rope_append(a.ws.qkv, a.kv->pages, p->d_tok_req, a.b->q_indptr, a.b->ctx_len,
                                     a.b->page_indptr, a.b->page_ids, t0, op.tok_end, m->n_q_heads, m->n_kv_heads,
                                     m->head_dim, m->rope_theta, ctx->offload_host != nullptr, s);
      });
    case NF_OP_ATTN: {
      const NfAttnShape shp{m->n_q_heads, m->n_kv_heads, m->head_dim, (int32_t)nqkv};
      e = traced(ctx, NF_K_ATTENTION, op, s, [&] {
        return nf_launch_attention(a.ws.qkv, a.kv->pages, a.b->page_indptr, a.b->page_ids,
                                   p->d_items + p->item_off[op.nano], p->item_cnt[op.nano], shp, a.ws.parts,
                                   a.ws.attn, op.attn_wgs, s, p->item_pages[op.nano], ctx->num_cus);
      });
      if (e != hipSuccess) return e;
      return traced(ctx, NF_K_ATTN_MERGE, op, s, [&] {
        return nf_launch_attention_merge(a.ws.parts, p->d_groups + p->group_off[op.nano], p->group_cnt[op.nano], shp,
                                         a.ws.attn, s);
      });
    }
    case NF_OP_O:
      return traced(ctx, NF_K_GEMM, op, s, [&] {
        return nf_launch_gemm(a.ws.attn + t0 * qdim * 2, a.w->w_o, a.ws.y + t0 * D * 2, a.x_in + t0 * D * 2, M, (int)D,
                              (int)qdim, NF_EPI_RESIDUAL, op.gemm_tile, s);
      });
    case NF_OP_UG:
      e = traced(ctx, NF_K_RMSNORM, op, s, [&] {
        return nf_launch_rmsnorm(a.ws.y + t0 * D * 2, a.w->g_ffn_norm, a.ws.h + t0 * D * 2, M, (int)D, m->rms_eps, s);
      });
      if (e != hipSuccess) return e;
      if (m->n_experts > 1) {
        // gate routing, grouping of the (token, expert) rows, grouped Up/Gate GEMM
        const int E = m->n_experts, k = m->top_k;
        int32_t* eoff = a.ws.expert_offset + (size_t)op.nano * (E + 1);
        e = traced(ctx, NF_K_MOE_ROUTE, op, s, [&] {
          hipError_t r = nf_launch_moe_router(a.ws.h, a.w->w_router, a.ws.expert_ids, a.ws.expert_w, t0, op.tok_end,
                                              (int)D, E, k, s);
          if (r != hipSuccess) return r;
          return nf_launch_moe_scatter(a.ws.expert_ids, t0, op.tok_end, E, k, eoff, a.ws.row_token, a.ws.slot_of, s);
        });
        if (e != hipSuccess) return e;
        return traced(ctx, NF_K_GEMM, op, s, [&] {
          return nf_launch_grouped_gemm(a.ws.h, a.w->w_gate_up, a.ws.f, M * k, (int)I, (int)D, NF_EPI_SWIGLU, eoff,
                                        a.ws.row_token, E, (long long)(2 * I * D), s);
        });
      }
      return traced(ctx, NF_K_GEMM, op, s, [&] {
        return nf_launch_gemm(a.ws.h + t0 * D * 2, a.w->w_gate_up, a.ws.f + t0 * I * 2, nullptr, M, (int)I, (int)D,
                              NF_EPI_SWIGLU, op.gemm_tile, s);
      });
    case NF_OP_D:
      if (m->n_experts > 1) {
        const int E = m->n_experts, k = m->top_k;
        const int32_t* eoff = a.ws.expert_offset + (size_t)op.nano * (E + 1);
        const size_t Bk = (size_t)std::max(1, a.b->n_tokens) * k;
        const NfGemmSplit moe_split{a.ws.expert_partial, (long long)(Bk * D)};
        e = traced(ctx, NF_K_GEMM, op, s, [&] {
          return nf_launch_grouped_gemm(a.ws.f, a.w->w_down, a.ws.expert_out, M * k, (int)D, (int)I, NF_EPI_NONE, eoff,
                                        nullptr, E, (long long)(D * I), s, moe_split);
        });
        if (e != hipSuccess) return e;
        return traced(ctx, NF_K_MOE_COMBINE, op, s, [&] {
          return nf_launch_moe_combine(a.ws.y, a.ws.expert_out, a.ws.slot_of, a.ws.expert_w, a.x_out, t0, op.tok_end,
                                       (int)D, k, s, moe_split.partial, moe_split.seg_stride);
        });
      }
      return traced(ctx, NF_K_GEMM, op, s, [&] {
        // rows t0.. of both halves' sums: nano-operations on different rows never share scratch
        const size_t B = (size_t)std::max(1, a.b->n_tokens);
        const NfGemmSplit split{a.ws.down_partial ? a.ws.down_partial + t0 * D : nullptr, (long long)(B * D)};
        return nf_launch_gemm(a.ws.f + t0 * I * 2, a.w->w_down, a.x_out + t0 * D * 2, a.ws.y + t0 * D * 2, M, (int)D,
                              (int)I, NF_EPI_RESIDUAL, op.gemm_tile, s, split);
      });
    default:
      return hipErrorInvalidValue;
  }
}

// Runs the plan on n_layers consecutive layers (a[l] holds layer l's weights, cache and
// input / output buffers; the workspace is shared).  Overlapped plans are pipelined across
// the layer boundary as the paper's pipelines are (Sec. 4.1, Fig. 6: the operations of the
// next layer follow without a global join): the KQV nano-operation of a token range in layer
// l + 1 is issued right behind the Down nano-operation of the same range in layer l, so the
// attention of that range can run beside the remaining GEMMs of layer l.  This is safe with
// one shared workspace because (i) every buffer is indexed by token row and the nano-batches
// are disjoint row ranges, (ii) the operations of one range form a chain, and (iii) the
// layers own distinct KV pools.  Events alternate between two sets from layer to layer: a
// hoisted KQV re-records its event before the late operations of the previous layer have
// enqueued their waits.
// Simultaneous KV offload (Sec. 4.2.2): once the attention nano-operation of a token range is
// done, the K and V parts of its qkv rows (rotary embedding applied) are copied to the host by
// a small kernel on a stream of its own, so the copy runs during the dense operations that
// follow.  (Starting it right behind the KQV nano-operation cost 5 % of the 8B layer instead
// of 3 %: the copy kernel then occupies CUs just when the attention kernel's persistent
// workgroups are placed, and a fixed work schedule ends with its slowest workgroup.)  `done`
// receives the event the copy records; whoever overwrites those qkv rows next (the same
// range's KQV of the next layer) and the end of the call wait for it.
struct Offload {
  nf_ctx* ctx;
  size_t cursor = 0;
  bool on() const { return ctx->offload_host != nullptr; }
  hipError_t event(hipEvent_t* e) {
    if (cursor == ctx->offload_events.size()) {
      hipEvent_t n = nullptr;
      hipError_t r = hipEventCreateWithFlags(&n, hipEventDisableTiming);
      if (r != hipSuccess) return r;
      ctx->offload_events.push_back(n);
    }
    *e = ctx->offload_events[cursor++];
    return hipSuccess;
  }
  hipError_t after_attention(const NfNanoOp& op, const LayerArgs& a, int layer, hipStream_t s, hipEvent_t* done) {
    hipEvent_t ready = nullptr;
    hipError_t r = event(&ready);
    if (r == hipSuccess) r = hipEventRecord(ready, s);
    if (r == hipSuccess) r = hipStreamWaitEvent(ctx->offload_stream, ready, 0);
    if (r == hipSuccess)
      r = nf_launch_kv_offload(a.ws.qkv, (char*)ctx->offload_host + (size_t)layer * ctx->offload_layer_stride,
                               op.tok_begin, op.tok_end, a.m->n_q_heads, a.m->n_kv_heads, a.m->head_dim,
                               ctx->offload_stream);
    if (r == hipSuccess) r = event(done);
    if (r == hipSuccess) r = hipEventRecord(*done, ctx->offload_stream);
    return r;
  }
};

int run_layers(nf_ctx* ctx, const nf_plan* p, const LayerArgs* a, int n_layers, hipStream_t user) {
  Offload off{ctx};
  // per attention nano-op: the latest offload copy of its qkv rows.  A KQV nano-op overwrites qkv
  // rows, so it waits for the copies of the attention nano-ops whose rows it shares.
  std::vector<hipEvent_t> copied(p->ops.size(), nullptr);
  auto wait_for_copies = [&](const NfNanoOp& kqv, hipStream_t s) -> hipError_t {
    for (size_t j = 0; j < p->ops.size(); ++j) {
      const NfNanoOp& at = p->ops[j];
      if (at.kind != NF_OP_ATTN || !copied[j]) continue;
      if (std::max(at.tok_begin, kqv.tok_begin) >= std::min(at.tok_end, kqv.tok_end)) continue;
      hipError_t e = hipStreamWaitEvent(s, copied[j], 0);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  };
  if (!p->overlap) {
    for (int l = 0; l < n_layers; ++l)
      for (size_t i = 0; i < p->ops.size(); ++i) {
        const NfNanoOp& op = p->ops[i];
        if (op.kind == NF_OP_KQV) NF_HIP(ctx, wait_for_copies(op, user));
        NF_HIP(ctx, launch_nano_op(ctx, p, op, a[l], user));
        if (op.kind == NF_OP_ATTN && off.on()) NF_HIP(ctx, off.after_attention(op, a[l], l, user, &copied[i]));
      }
    for (hipEvent_t e : copied)
      if (e) NF_HIP(ctx, hipStreamWaitEvent(user, e, 0));
    return NF_OK;
  }
  // fork: the lane streams start after everything already enqueued on the caller's stream
  NF_HIP(ctx, hipEventRecord(p->ev_fork, user));
  for (int l = 0; l < NF_LANES; ++l) NF_HIP(ctx, hipStreamWaitEvent(p->lane_stream[l], p->ev_fork, 0));
  auto emit = [&](int layer, size_t i, int after_prev_layer_op) -> int {
    const NfNanoOp& op = p->ops[i];
    hipStream_t s = p->lane_stream[op.lane];
    const std::vector<hipEvent_t>& ev = (layer & 1) ? p->events_alt : p->events;
    for (int d : op.deps) NF_HIP(ctx, hipStreamWaitEvent(s, ev[d], 0));
    if (after_prev_layer_op >= 0 && p->ops[after_prev_layer_op].lane != op.lane) {
      const std::vector<hipEvent_t>& pev = ((layer - 1) & 1) ? p->events_alt : p->events;
      NF_HIP(ctx, hipStreamWaitEvent(s, pev[after_prev_layer_op], 0));
    }
    if (op.kind == NF_OP_KQV) NF_HIP(ctx, wait_for_copies(op, s));
    NF_HIP(ctx, launch_nano_op(ctx, p, op, a[layer], s));
    if (op.kind == NF_OP_ATTN && off.on()) NF_HIP(ctx, off.after_attention(op, a[layer], layer, s, &copied[i]));
    if (op.record) NF_HIP(ctx, hipEventRecord(ev[i], s));
    return NF_OK;
  };
  std::vector<char> down_done((size_t)std::max(1, p->n_tokens));  // rows whose Down nano-op of this layer is issued
  std::vector<char> hoisted(p->ops.size());                       // next layer's KQV nano-ops already issued
  for (int l = 0; l < n_layers; ++l) {
    std::fill(down_done.begin(), down_done.end(), 0);
    std::fill(hoisted.begin(), hoisted.end(), 0);
    for (size_t i = 0; i < p->ops.size(); ++i) {
      const NfNanoOp& op = p->ops[i];
      if (l > 0 && op.kind == NF_OP_KQV) continue;  // issued behind the previous layer's Down
      int rc = emit(l, i, -1);
      if (rc) return rc;
      if (op.kind == NF_OP_D && l + 1 < n_layers) {
        // the next layer's KQV nano-ops whose rows are now all complete (with equal partitions:
        // the one of the same range)
        for (int t = op.tok_begin; t < op.tok_end; ++t) down_done[(size_t)t] = 1;
        for (size_t j = 0; j < p->ops.size(); ++j) {
          const NfNanoOp& nx = p->ops[j];
          if (nx.kind != NF_OP_KQV || hoisted[j]) continue;
          bool complete = true;
          for (int t = nx.tok_begin; t < nx.tok_end && complete; ++t) complete = down_done[(size_t)t] != 0;
          if (!complete) continue;
          hoisted[j] = 1;
          rc = emit(l + 1, j, (int)i);
          if (rc) return rc;
        }
      }
    }
  }
  // join: the caller's stream continues after both lanes (and the offload copies) have drained
  for (int l = 0; l < NF_LANES; ++l) {
    NF_HIP(ctx, hipEventRecord(p->ev_join[l], p->lane_stream[l]));
    NF_HIP(ctx, hipStreamWaitEvent(user, p->ev_join[l], 0));
  }
  for (hipEvent_t e : copied)
    if (e) NF_HIP(ctx, hipStreamWaitEvent(user, e, 0));
  return NF_OK;
}

int check_weights(const nf_model_desc* model, const nf_layer_weights* w) {
  if (!w->g_attn_norm || !w->w_qkv || !w->w_o || !w->g_ffn_norm || !w->w_gate_up || !w->w_down ||
      (model->n_experts > 1 && !w->w_router))
    return NF_EINVAL;
  return NF_OK;
}

// The unsplit plan a plan = NULL call runs with.  It is kept in the context and reused while the
// batch stays the same.  When the batch changes, the old plan cannot be freed at once - kernels
// already enqueued on the caller's stream may still read its work lists - and the call must not
// wait for them either (it returns after enqueueing): the old plan is parked with an event
// recorded on the caller's stream and freed by a later call once that event has passed.  Only
// a caller more than eight batches ahead of the GPU waits (for the oldest parked plan).
int null_plan_for(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch, hipStream_t user,
                  const nf_plan** out) {
  nf_plan* cur = ctx->null_plan;
  if (cur && cur->n_tokens == batch->n_tokens && cur->batch_sig == nf_batch_signature(batch) &&
      memcmp(&cur->model, model, sizeof(nf_model_desc)) == 0) {
    *out = cur;
    return NF_OK;
  }
  for (size_t i = 0; i < ctx->retired_plans.size();) {
    auto& r = ctx->retired_plans[i];
    const bool oldest_must_go = ctx->retired_plans.size() > 8 && i == 0;
    if (oldest_must_go) NF_HIP(ctx, hipEventSynchronize(r.second));
    if (oldest_must_go || hipEventQuery(r.second) == hipSuccess) {
      (void)hipEventDestroy(r.second);
      nf_plan_destroy(r.first);
      ctx->retired_plans.erase(ctx->retired_plans.begin() + (long)i);
    } else {
      ++i;
    }
  }
  if (cur) {
    hipEvent_t e = nullptr;
    NF_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    NF_HIP(ctx, hipEventRecord(e, user));
    ctx->retired_plans.emplace_back(cur, e);
    ctx->null_plan = nullptr;
  }
  const int32_t bounds[2] = {0, batch->n_tokens};
  nf_plan* fresh = nullptr;
  int rc = nf_plan_manual(ctx, model, batch, 1, bounds, 0, 0, 0, 0, &fresh);
  if (rc) return rc;
  ctx->null_plan = fresh;
  *out = fresh;
  return NF_OK;
}

}  // namespace

extern "C" int nf_layer_forward(nf_ctx* ctx, const nf_model_desc* model, const nf_layer_weights* weights,
                                nf_kv_cache* kv, const nf_batch* batch, const nf_plan* plan, const void* x_in,
                                void* x_out, void* workspace, size_t workspace_bytes, void* hip_stream) try {
  if (!ctx || !weights || !kv || !batch) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  if (!kv->pages || kv->num_pages < 0) return NF_EINVAL;
  rc = nf_validate_batch(model, batch, kv->num_pages);
  if (rc) return rc;
  if (batch->n_tokens == 0) return NF_OK;
  if (!x_in || !x_out || x_in == x_out || !workspace) return NF_EINVAL;
  if (check_weights(model, weights) != NF_OK) return NF_EINVAL;
  hipStream_t user = (hipStream_t)hip_stream;

  if (!plan) {
    rc = null_plan_for(ctx, model, batch, user, &plan);
    if (rc) return rc;
  }
  rc = NF_OK;
  if ((int)plan->bounds.size() - 1 > kMaxNanoOffsets) rc = NF_EPLAN;
  if (plan->n_tokens != batch->n_tokens || plan->batch_sig != nf_batch_signature(batch) ||
      memcmp(&plan->model, model, sizeof(nf_model_desc)) != 0)
    rc = NF_EPLAN;
  if (rc == NF_OK && workspace_bytes < nf_plan_workspace_bytes(plan)) rc = NF_EWORKSPACE;
  if (rc == NF_OK && ctx->offload_host && ctx->offload_layer_stride != 0 &&
      (size_t)batch->n_tokens * 2 * model->n_kv_heads * model->head_dim * 2 > ctx->offload_layer_stride)
    rc = NF_EINVAL;
  if (rc == NF_OK) {
    LayerArgs a;
    a.m = model;
    a.w = weights;
    a.kv = kv;
    a.b = batch;
    a.x_in = (const char*)x_in;
    a.x_out = (char*)x_out;
    a.ws = layout_workspace(model, batch->n_tokens, (size_t)std::max(1, plan->total_parts), (char*)workspace);
    rc = run_layers(ctx, plan, &a, 1, user);
  }
  return rc;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" size_t nf_layers_workspace_bytes(const nf_plan* plan, int n_layers) {
  if (!plan || n_layers < 1) return 0;
  const size_t x_bytes = nf_align256((size_t)std::max(1, plan->n_tokens) * plan->model.hidden * 2);
  return nf_align256(nf_plan_workspace_bytes(plan)) + (n_layers > 1 ? 2 * x_bytes : 0);
}

extern "C" int nf_layers_forward(nf_ctx* ctx, const nf_model_desc* model, int n_layers,
                                 const nf_layer_weights* weights, nf_kv_cache* kv, const nf_batch* batch,
                                 const nf_plan* plan, const void* x_in, void* x_out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) try {
  if (!ctx || !weights || !kv || !batch || !plan || n_layers < 1) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  for (int l = 0; l < n_layers; ++l) {
    if (!kv[l].pages || kv[l].num_pages < 0) return NF_EINVAL;
    if (check_weights(model, &weights[l]) != NF_OK) return NF_EINVAL;
    // the pipelining across the layer boundary relies on distinct pools (and so does the model)
    for (int k = 0; k < l; ++k)
      if (kv[k].pages == kv[l].pages) return NF_EINVAL;
    rc = nf_validate_batch(model, batch, kv[l].num_pages);
    if (rc) return rc;
  }
  if (batch->n_tokens == 0) return NF_OK;
  if (!x_in || !x_out || x_in == x_out || !workspace) return NF_EINVAL;
  if ((int)plan->bounds.size() - 1 > kMaxNanoOffsets) return NF_EPLAN;
  if (plan->n_tokens != batch->n_tokens || plan->batch_sig != nf_batch_signature(batch) ||
      memcmp(&plan->model, model, sizeof(nf_model_desc)) != 0)
    return NF_EPLAN;
  if (workspace_bytes < nf_layers_workspace_bytes(plan, n_layers)) return NF_EWORKSPACE;
  if (ctx->offload_host && (size_t)batch->n_tokens * 2 * model->n_kv_heads * model->head_dim * 2 > ctx->offload_layer_stride)
    return NF_EINVAL;
  const size_t x_bytes = nf_align256((size_t)batch->n_tokens * model->hidden * 2);
  char* mid[2] = {(char*)workspace + nf_align256(nf_plan_workspace_bytes(plan)), nullptr};
  mid[1] = mid[0] + x_bytes;
  std::vector<LayerArgs> args((size_t)n_layers);
  for (int l = 0; l < n_layers; ++l) {
    LayerArgs& a = args[l];
    a.m = model;
    a.w = &weights[l];
    a.kv = &kv[l];
    a.b = batch;
    a.x_in = l == 0 ? (const char*)x_in : mid[(l - 1) & 1];
    a.x_out = l == n_layers - 1 ? (char*)x_out : mid[l & 1];
    a.ws = layout_workspace(model, batch->n_tokens, (size_t)std::max(1, plan->total_parts), (char*)workspace);
  }
  return run_layers(ctx, plan, args.data(), n_layers, (hipStream_t)hip_stream);
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

// --------------------------------------------------------- single operations ---

extern "C" int nf_op_rmsnorm(const void* x, const void* g, void* out, int n_tokens, int hidden, float eps,
                             void* hip_stream) {
  if (!x || !g || !out || n_tokens < 0 || hidden <= 0) return NF_EINVAL;
  if (hidden % 8) return NF_ESHAPE;
  return nf_launch_rmsnorm(x, g, out, n_tokens, hidden, eps, (hipStream_t)hip_stream) == hipSuccess ? NF_OK : NF_EHIP;
}

extern "C" int nf_gemm_segments(int N, int K, int epilogue) {
  if (N <= 0 || K <= 0 || epilogue < NF_EPI_NONE || epilogue > NF_EPI_SWIGLU || K % 64 || N % 64) return 0;
  return nf_gemm_k_segments(N, K, epilogue);
}

extern "C" int nf_op_gemm(const void* x, const void* w, void* out, const void* residual, int M, int N, int K,
                          int epilogue, void* hip_stream) {
  if (!x || !w || !out || M < 0 || N <= 0 || K <= 0) return NF_EINVAL;
  if (epilogue < NF_EPI_NONE || epilogue > NF_EPI_SWIGLU) return NF_EINVAL;
  if (epilogue == NF_EPI_RESIDUAL && !residual) return NF_EINVAL;
  if (K % 64 || N % 64) return NF_ESHAPE;
  return nf_launch_gemm(x, w, out, residual, M, N, K, epilogue, 0, (hipStream_t)hip_stream) == hipSuccess ? NF_OK
                                                                                                         : NF_EHIP;
}

extern "C" int nf_op_rope_append(nf_ctx* ctx, const nf_model_desc* model, nf_kv_cache* kv, const nf_batch* batch,
                                 const nf_plan* plan, void* qkv, int tok_begin, int tok_end, void* hip_stream) {
  if (!ctx || !kv || !batch || !plan || !qkv) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, kv->num_pages);
  if (rc) return rc;
  if (plan->batch_sig != nf_batch_signature(batch)) return NF_EPLAN;
  if (tok_begin < 0 || tok_end > batch->n_tokens || tok_begin > tok_end) return NF_EINVAL;
  NF_HIP(ctx, nf_launch_rope_append(qkv, kv->pages, plan->d_tok_req, batch->q_indptr, batch->ctx_len,
                                    batch->page_indptr, batch->page_ids, tok_begin, tok_end, model->n_q_heads,
                                    model->n_kv_heads, model->head_dim, model->rope_theta, 0,
                                    (hipStream_t)hip_stream));
  return NF_OK;
}

namespace {

// Shared body of nf_op_attention and nf_op_attention_static: validation on the host mirrors,
// then the attention kernel and the merge kernel with `parts` as the partial-result buffer.
int op_attention(nf_ctx* ctx, const nf_model_desc* model, const nf_kv_cache* kv, const nf_batch* batch,
                 const nf_plan* plan, const void* qkv, void* attn_out, float* parts, size_t parts_bytes,
                 int too_small, int nano_index, hipStream_t s) {
  if (!ctx || !kv || !batch || !plan || !qkv || !attn_out || !parts) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, kv->num_pages);
  if (rc) return rc;
  if (plan->batch_sig != nf_batch_signature(batch)) return NF_EPLAN;
  if (nano_index < 0 || nano_index + 1 >= (int)plan->bounds.size()) return NF_EINVAL;
  const size_t need = nf_align256((size_t)std::max(1, plan->total_parts) * model->n_kv_heads *
                                  nf_attn_part_floats(model->head_dim) * sizeof(float));
  if (parts_bytes < need) return too_small;
  const int32_t nqkv = (model->n_q_heads + 2 * model->n_kv_heads) * model->head_dim;
  const NfAttnShape shp{model->n_q_heads, model->n_kv_heads, model->head_dim, nqkv};
  NF_HIP(ctx, nf_launch_attention(qkv, kv->pages, batch->page_indptr, batch->page_ids,
                                  plan->d_items + plan->item_off[nano_index], plan->item_cnt[nano_index], shp,
                                  parts, attn_out, plan->nano_attn_wgs[nano_index], s, plan->item_pages[nano_index],
                                  ctx->num_cus));
  NF_HIP(ctx, nf_launch_attention_merge(parts, plan->d_groups + plan->group_off[nano_index],
                                        plan->group_cnt[nano_index], shp, attn_out, s));
  return NF_OK;
}

}  // namespace

extern "C" int nf_op_attention(nf_ctx* ctx, const nf_model_desc* model, const nf_kv_cache* kv, const nf_batch* batch,
                               const nf_plan* plan, const void* qkv, void* attn_out, void* workspace,
                               size_t workspace_bytes, int nano_index, void* hip_stream) {
  return op_attention(ctx, model, kv, batch, plan, qkv, attn_out, (float*)workspace, workspace_bytes, NF_EWORKSPACE,
                      nano_index, (hipStream_t)hip_stream);
}

extern "C" size_t nf_attention_static_bytes(void) { return NF_ATTN_STATIC_BYTES; }

extern "C" int nf_op_attention_static(nf_ctx* ctx, const nf_model_desc* model, const nf_kv_cache* kv,
                                      const nf_batch* batch, const nf_plan* plan, const void* qkv, void* attn_out,
                                      int nano_index, void* hip_stream) {
  if (!ctx) return NF_EINVAL;
  // ctx->static_parts is the address hipGetSymbolAddress returned for ctx->device at nf_ctx_create
  return op_attention(ctx, model, kv, batch, plan, qkv, attn_out, ctx->static_parts, ctx->static_parts_bytes,
                      NF_ESCRATCH, nano_index, (hipStream_t)hip_stream);
}

extern "C" int nf_op_embedding(const int32_t* token_ids, const int32_t* from_slot, const int32_t* slot_tokens,
                               const void* table, int table_rows, void* out, int n_rows, int width,
                               void* hip_stream) {
  if (!token_ids || !table || !out || n_rows < 0 || table_rows < 1 || width < 8) return NF_EINVAL;
  if ((from_slot != nullptr) != (slot_tokens != nullptr)) return NF_EINVAL;
  if (width % 8) return NF_ESHAPE;
  return nf_launch_gather_rows(token_ids, from_slot, slot_tokens, table, table_rows, out, n_rows, width,
                               (hipStream_t)hip_stream) == hipSuccess
             ? NF_OK
             : NF_EHIP;
}

extern "C" int nf_op_argmax(const void* logits, int n_rows, int vocab, const int32_t* out_index, int32_t* out,
                            void* hip_stream) {
  if (!logits || !out || n_rows < 0 || vocab < 8) return NF_EINVAL;
  if (vocab % 8) return NF_ESHAPE;
  return nf_launch_argmax(logits, n_rows, vocab, out_index, out, (hipStream_t)hip_stream) == hipSuccess ? NF_OK
                                                                                                        : NF_EHIP;
}

extern "C" int nf_op_move_pages(void* pool, size_t page_bytes, int64_t num_pages, const int32_t* page_ids, int n_pages,
                                void* staging, int scatter, void* hip_stream) {
  if (!pool || !staging || n_pages < 0 || num_pages < 0 || (n_pages > 0 && !page_ids)) return NF_EINVAL;
  if (page_bytes == 0 || page_bytes % 16) return NF_ESHAPE;
  return nf_launch_move_pages(pool, page_bytes, (long)num_pages, page_ids, n_pages, staging, scatter ? 1 : 0,
                              (hipStream_t)hip_stream) == hipSuccess
             ? NF_OK
             : NF_EHIP;
}
