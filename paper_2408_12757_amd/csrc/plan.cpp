// Plans: validation of a dense batch, construction of the nano-operation list with
// its dependencies (paper Sec. 4.1.2 "Constraints on dependencies"), the device work
// lists of the attention nano-operations, and the explicit-structure entry point.
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "nf_internal.h"
#include "planner.h"

// Device buffers of destroyed plans are kept for the next plans instead of being returned to
// the driver: hipFree waits for the whole device, which would stall a caller that forms the
// next batch while the current iteration is still running (Sec. 4.2.1, asynchronous
// scheduling).  A handful of buffers per process; the rest is freed.
namespace {
struct BlobPool {
  struct Blob {
    void* p;
    size_t bytes;
    int device;
  };
  std::mutex mu;
  std::vector<Blob> free_list;
  hipError_t acquire(int device, size_t bytes, void** out, size_t* got) {
    {
      std::lock_guard<std::mutex> g(mu);
      int best = -1;
      for (size_t i = 0; i < free_list.size(); ++i) {
        const Blob& b = free_list[i];
        if (b.device == device && b.bytes >= bytes && b.bytes <= 4 * bytes + (1u << 20) &&
            (best < 0 || b.bytes < free_list[best].bytes))
          best = (int)i;
      }
      if (best >= 0) {
        *out = free_list[best].p;
        *got = free_list[best].bytes;
        free_list.erase(free_list.begin() + best);
        return hipSuccess;
      }
    }
    const size_t rounded = (bytes + bytes / 4 + 65535) & ~(size_t)65535;
    *got = rounded;
    return hipMalloc(out, rounded);
  }
  void release(int device, void* p, size_t bytes) {
    {
      std::lock_guard<std::mutex> g(mu);
      if (free_list.size() < 16) {
        free_list.push_back(Blob{p, bytes, device});
        return;
      }
    }
    (void)hipFree(p);
  }
};
BlobPool g_blobs;
}  // namespace


size_t nf_align256(size_t v) { return (v + 255) & ~(size_t)255; }

int nf_validate_model(const nf_model_desc* m) {
  if (!m) return NF_EINVAL;
  if (m->hidden <= 0 || m->n_q_heads <= 0 || m->n_kv_heads <= 0 || m->ffn_inner <= 0) return NF_EINVAL;
  if (m->page_size != 16) return NF_ESHAPE;
  if (m->head_dim != 64 && m->head_dim != 128) return NF_ESHAPE;
  if (m->n_q_heads % m->n_kv_heads) return NF_ESHAPE;
  if (m->n_q_heads / m->n_kv_heads > 16) return NF_ESHAPE;
  if (m->hidden % 64 || m->ffn_inner % 64) return NF_ESHAPE;
  if (m->n_experts > 1 && (m->top_k < 1 || m->top_k > m->n_experts || m->top_k > 4 || m->n_experts > 64))
    return NF_ESHAPE;
  return NF_OK;
}

int nf_validate_batch(const nf_model_desc* m, const nf_batch* b, int64_t num_pages) {
  if (!b) return NF_EINVAL;
  if (b->n_tokens < 0 || b->n_prefill_reqs < 0 || b->n_decode_reqs < 0) return NF_EINVAL;
  const int n_reqs = b->n_prefill_reqs + b->n_decode_reqs;
  if (b->n_tokens == 0 && n_reqs == 0) return NF_OK;
  if (!b->host_q_indptr || !b->host_ctx_len || !b->host_page_indptr) return NF_EINVAL;
  if (!b->q_indptr || !b->ctx_len || !b->page_indptr || !b->page_ids) return NF_EINVAL;
  if (b->host_q_indptr[0] != 0 || b->host_q_indptr[n_reqs] != b->n_tokens) return NF_ESHAPE;
  if (b->host_page_indptr[0] != 0) return NF_EPAGES;
  for (int r = 0; r < n_reqs; ++r) {
    const int ql = b->host_q_indptr[r + 1] - b->host_q_indptr[r];
    if (ql < 1) return NF_ESHAPE;
    if (r >= b->n_prefill_reqs && ql != 1) return NF_ESHAPE;  // decode requests carry one token
    if (b->host_ctx_len[r] < 0) return NF_ESHAPE;
    const int np = b->host_page_indptr[r + 1] - b->host_page_indptr[r];
    if (np < 0) return NF_EPAGES;
    if ((int64_t)np * m->page_size < (int64_t)b->host_ctx_len[r] + ql) return NF_EPAGES;
  }
  if (b->host_page_ids) {
    const int total = b->host_page_indptr[n_reqs];
    for (int i = 0; i < total; ++i)
      if (b->host_page_ids[i] < 0 || (int64_t)b->host_page_ids[i] >= num_pages) return NF_EPAGES;
  }
  return NF_OK;
}

extern "C" int nf_check_batch(const nf_model_desc* model, const nf_batch* batch, int64_t num_pages) {
  int rc = nf_validate_model(model);
  if (rc) return rc;
  if (num_pages < 0) return NF_EINVAL;
  return nf_validate_batch(model, batch, num_pages);
}

uint64_t nf_batch_signature(const nf_batch* b) {
  uint64_t h = 1469598103934665603ull;
  auto mix = [&h](uint64_t v) {
    h ^= v;
    h *= 1099511628211ull;
  };
  const int n_reqs = b->n_prefill_reqs + b->n_decode_reqs;
  mix((uint64_t)b->n_tokens);
  mix((uint64_t)b->n_prefill_reqs);
  mix((uint64_t)n_reqs);
  for (int r = 0; r <= n_reqs && b->host_q_indptr; ++r) mix((uint64_t)b->host_q_indptr[r]);
  for (int r = 0; r < n_reqs && b->host_ctx_len; ++r) mix((uint64_t)b->host_ctx_len[r]);
  return h;
}

// Parent operations (Sec. 2.1): attention needs KQV of the same tokens (and, for a
// prefill request, of the request's earlier tokens); O needs attention; Up/Gate needs O;
// Down needs Up/Gate.
static bool is_parent(int parent, int child) {
  return (parent == NF_OP_KQV && child == NF_OP_ATTN) || (parent == NF_OP_ATTN && child == NF_OP_O) ||
         (parent == NF_OP_O && child == NF_OP_UG) || (parent == NF_OP_UG && child == NF_OP_D);
}

// Dependency rule of Sec. 4.1.2: two nano-operations are dependent iff their parent
// operations are dependent and their token ranges intersect.
extern "C" int nf_nano_ops_dependent(int parent_kind, int child_kind, int b0, int e0, int b1, int e1) {
  if (!is_parent(parent_kind, child_kind)) return 0;
  return std::max(b0, b1) < std::min(e0, e1) ? 1 : 0;
}

void nf_plan_default_order(nf_plan* p, int overlap, const int* order) {
  const int n = (int)p->bounds.size() - 1;
  p->ops.clear();
  p->nano_order.clear();
  if (order)
    for (int k = 0; k < n; ++k) p->nano_order.push_back(order[k]);
  auto add = [&](int kind, int k) {
    const int i = order ? order[k] : k;
    NfNanoOp op;
    op.kind = kind;
    op.nano = i;
    op.tok_begin = p->bounds[i];
    op.tok_end = p->bounds[i + 1];
    op.lane = (overlap && kind == NF_OP_ATTN) ? NF_LANE_ATTN : NF_LANE_GEMM;
    p->ops.push_back(op);
  };
  if (!overlap) {
    for (int i = 0; i < n; ++i)
      for (int k = 0; k < NF_OP_KINDS; ++k) add(k, i);
  } else {
    for (int i = 0; i < n; ++i) {
      add(NF_OP_KQV, i);
      add(NF_OP_ATTN, i);
    }
    for (int i = 0; i < n; ++i) {
      add(NF_OP_O, i);
      add(NF_OP_UG, i);
      add(NF_OP_D, i);
    }
  }
  p->overlap = overlap;
}

int nf_plan_finalize(nf_ctx* ctx, nf_plan* p, const nf_batch* batch) {
  const nf_model_desc& m = p->model;
  const int n_reqs = batch->n_prefill_reqs + batch->n_decode_reqs;
  const int n_nano = (int)p->bounds.size() - 1;
  p->n_tokens = batch->n_tokens;
  p->n_reqs = n_reqs;
  p->n_prefill_reqs = batch->n_prefill_reqs;
  p->batch_sig = nf_batch_signature(batch);
  // resource share of every attention nano-operation (Sec. 4.1.1: each nano-operation has its
  // own R): the plan-wide default unless the caller gave one per nano-batch
  if ((int)p->nano_attn_wgs.size() != n_nano) p->nano_attn_wgs.assign((size_t)n_nano, p->attn_wgs);
  for (NfNanoOp& op : p->ops)
    if (op.kind == NF_OP_ATTN) op.attn_wgs = p->nano_attn_wgs[op.nano];

  // token -> request
  std::vector<int32_t> tok_req((size_t)std::max(1, batch->n_tokens));
  for (int r = 0; r < n_reqs; ++r)
    for (int t = batch->host_q_indptr[r]; t < batch->host_q_indptr[r + 1]; ++t) tok_req[t] = r;

  // ---- dependencies between nano-operations -----------------------------------------------
  // Two nano-operations depend on each other iff their parents do and their token ranges
  // intersect.  An attention nano-op whose range starts inside a prefill request also reads
  // the K/V that request appended in earlier ranges, so its range is extended back to the
  // request's first token before the test.
  for (size_t a = 0; a < p->ops.size(); ++a) {
    NfNanoOp& oa = p->ops[a];
    oa.deps.clear();
    int eb = oa.tok_begin;
    if (oa.kind == NF_OP_ATTN && oa.tok_begin < oa.tok_end) eb = batch->host_q_indptr[tok_req[oa.tok_begin]];
    for (size_t b = 0; b < a; ++b) {
      NfNanoOp& ob = p->ops[b];
      if (!nf_nano_ops_dependent(ob.kind, oa.kind, ob.tok_begin, ob.tok_end,
                                 oa.kind == NF_OP_ATTN ? eb : oa.tok_begin, oa.tok_end))
        continue;
      if (ob.lane != oa.lane) {
        oa.deps.push_back((int)b);
        ob.record = true;
      }
    }
  }
  // every nano-op's inputs must be produced earlier in launch order
  for (size_t a = 0; a < p->ops.size(); ++a) {
    const NfNanoOp& oa = p->ops[a];
    if (oa.kind == NF_OP_KQV || oa.tok_begin >= oa.tok_end) continue;
    int lo = oa.tok_begin;
    if (oa.kind == NF_OP_ATTN) lo = batch->host_q_indptr[tok_req[oa.tok_begin]];
    std::vector<char> cov((size_t)(oa.tok_end - lo), 0);
    for (size_t b = 0; b < a; ++b) {
      const NfNanoOp& ob = p->ops[b];
      if (!is_parent(ob.kind, oa.kind)) continue;
      for (int t = std::max(lo, ob.tok_begin); t < std::min(oa.tok_end, ob.tok_end); ++t) cov[t - lo] = 1;
    }
    for (char c : cov)
      if (!c) return NF_EPLAN;
  }

  // ---- attention work lists -----------------------------------------------------------------
  const int G = m.n_q_heads / m.n_kv_heads;
  const int T = std::max(1, 16 / G);
  std::vector<NfAttnItem> items;
  std::vector<NfAttnGroup> groups;
  p->item_off.assign(n_nano, 0);
  p->item_cnt.assign(n_nano, 0);
  p->item_pages.assign(n_nano, 0);
  p->group_off.assign(n_nano, 0);
  p->group_cnt.assign(n_nano, 0);
  int part = 0;
  for (int i = 0; i < n_nano; ++i) {
    const int b = p->bounds[i], e = p->bounds[i + 1];
    p->item_off[i] = (int)items.size();
    p->group_off[i] = (int)groups.size();
    int t = b;
    while (t < e) {
      const int r = tok_req[t];
      const int q0 = batch->host_q_indptr[r], q1 = batch->host_q_indptr[r + 1];
      const int n_tok = std::min(T, std::min(e, q1) - t);
      const int pos0 = batch->host_ctx_len[r] + (t - q0);
      const int keys = pos0 + n_tok;
      const int n_parts = (keys + NF_ATTN_CHUNK - 1) / NF_ATTN_CHUNK;
      // rows whose keys fit one chunk need no merge: the attention kernel finishes them
      if (n_parts > 1) groups.push_back(NfAttnGroup{t, n_tok, part, n_parts});
      for (int j = 0; j < n_parts; ++j) {
        NfAttnItem it;
        it.req = r;
        it.tok0 = t;
        it.n_tok = n_tok;
        it.pos0 = pos0;
        it.key_begin = j * NF_ATTN_CHUNK;
        it.key_end = std::min(keys, (j + 1) * NF_ATTN_CHUNK);
        it.part = n_parts > 1 ? part + j : -1;
        it.pad = 0;
        items.push_back(it);
      }
      if (n_parts > 1) part += n_parts;
      t += n_tok;
    }
    p->item_cnt[i] = (int)items.size() - p->item_off[i];
    for (size_t k = (size_t)p->item_off[i]; k < items.size(); ++k)
      p->item_pages[i] += ((items[k].key_end + 15) >> 4) - (items[k].key_begin >> 4);
    p->group_cnt[i] = (int)groups.size() - p->group_off[i];
    // longest work first: the hardware dispatches workgroups in index order
    std::stable_sort(items.begin() + p->item_off[i], items.end(), [](const NfAttnItem& x, const NfAttnItem& y) {
      return (x.key_end - x.key_begin) > (y.key_end - y.key_begin);
    });
  }
  p->total_parts = part;

  // ---- upload ---------------------------------------------------------------------------------
  const size_t sz_tok = nf_align256(tok_req.size() * sizeof(int32_t));
  const size_t sz_items = nf_align256(std::max<size_t>(1, items.size()) * sizeof(NfAttnItem));
  const size_t sz_groups = nf_align256(std::max<size_t>(1, groups.size()) * sizeof(NfAttnGroup));
  NF_HIP(ctx, hipSetDevice(ctx->device));
  p->device = ctx->device;
  NF_HIP(ctx, g_blobs.acquire(ctx->device, sz_tok + sz_items + sz_groups, &p->dev_blob, &p->dev_blob_bytes));
  char* base = (char*)p->dev_blob;
  p->d_tok_req = (int32_t*)base;
  p->d_items = (NfAttnItem*)(base + sz_tok);
  p->d_groups = (NfAttnGroup*)(base + sz_tok + sz_items);
  NF_HIP(ctx, hipMemcpy(p->d_tok_req, tok_req.data(), tok_req.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  if (!items.empty())
    NF_HIP(ctx, hipMemcpy(p->d_items, items.data(), items.size() * sizeof(NfAttnItem), hipMemcpyHostToDevice));
  if (!groups.empty())
    NF_HIP(ctx, hipMemcpy(p->d_groups, groups.data(), groups.size() * sizeof(NfAttnGroup), hipMemcpyHostToDevice));

  // ---- streams and events ----------------------------------------------------------------------
  if (p->overlap) {
    for (int l = 0; l < NF_LANES; ++l) {
      int rc = nf_get_lane_stream(ctx, l, p->lane_cu_first[l], p->lane_cus[l], &p->lane_stream[l]);
      if (rc != NF_OK) return rc;
      NF_HIP(ctx, hipEventCreateWithFlags(&p->ev_join[l], hipEventDisableTiming));
    }
    NF_HIP(ctx, hipEventCreateWithFlags(&p->ev_fork, hipEventDisableTiming));
    p->events.assign(p->ops.size(), nullptr);
    p->events_alt.assign(p->ops.size(), nullptr);
    for (size_t a = 0; a < p->ops.size(); ++a) {
      // the last operation of a token range also records: in a multi-layer run the next
      // layer's first operation on that range may sit on the other lane
      if (p->ops[a].kind == NF_OP_D) p->ops[a].record = true;
      if (!p->ops[a].record) continue;
      NF_HIP(ctx, hipEventCreateWithFlags(&p->events[a], hipEventDisableTiming));
      NF_HIP(ctx, hipEventCreateWithFlags(&p->events_alt[a], hipEventDisableTiming));
    }
  }
  return NF_OK;
}

static int check_bounds(const nf_batch* batch, int n_nano, const int32_t* bounds) {
  if (n_nano < 1 || !bounds) return NF_EINVAL;
  if (bounds[0] != 0 || bounds[n_nano] != batch->n_tokens) return NF_EPLAN;
  for (int i = 0; i < n_nano; ++i)
    if (bounds[i + 1] <= bounds[i] && !(batch->n_tokens == 0 && n_nano == 1)) return NF_EPLAN;
  return NF_OK;
}

extern "C" int nf_plan_manual(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch, int n_nano,
                              const int32_t* bounds, int overlap, int attn_cus, int gemm_cus, int attn_wgs,
                              nf_plan** out) try {
  if (!ctx || !out) return NF_EINVAL;
  *out = nullptr;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, INT64_MAX);
  if (rc) return rc;
  rc = check_bounds(batch, n_nano, bounds);
  if (rc) return rc;
  if (attn_cus < 0 || gemm_cus < 0 || attn_cus > ctx->num_cus || gemm_cus > ctx->num_cus || attn_wgs < -1)
    return NF_EINVAL;
  nf_plan* p = new (std::nothrow) nf_plan();
  if (!p) return NF_ENOMEM;
  // released on every early exit, also when a container throws
  struct Guard {
    nf_plan* p;
    ~Guard() { nf_plan_destroy(p); }
  } guard{p};
  p->model = *model;
  p->bounds.assign(bounds, bounds + n_nano + 1);
  p->origin = "manual";
  p->attn_wgs = attn_wgs;
  nf_plan_default_order(p, overlap ? 1 : 0);
  // attention lane owns CU bits [0, attn_cus); the GEMM lane the gemm_cus bits that follow
  // (or the whole chip when gemm_cus = 0)
  p->lane_cus[NF_LANE_ATTN] = attn_cus;
  p->lane_cu_first[NF_LANE_ATTN] = 0;
  p->lane_cus[NF_LANE_GEMM] = gemm_cus;
  p->lane_cu_first[NF_LANE_GEMM] = (gemm_cus && attn_cus + gemm_cus <= ctx->num_cus) ? attn_cus : 0;
  rc = nf_plan_finalize(ctx, p, batch);
  if (rc) return rc;
  guard.p = nullptr;
  *out = p;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_plan_manual_ops(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch, int n_nano,
                                  const int32_t* bounds, int overlap, int attn_cus, int gemm_cus,
                                  const nf_nano_spec* spec, nf_plan** out) try {
  if (!ctx || !out || !spec) return NF_EINVAL;
  *out = nullptr;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, INT64_MAX);
  if (rc) return rc;
  rc = check_bounds(batch, n_nano, bounds);
  if (rc) return rc;
  if (attn_cus < 0 || gemm_cus < 0 || attn_cus > ctx->num_cus || gemm_cus > ctx->num_cus) return NF_EINVAL;
  // launch order: spec[i].launch_pos = position of nano-batch i (all zero = index order); it must
  // be a permutation, and nf_plan_finalize refuses one that launches an attention nano-operation
  // before a KQV nano-operation it depends on
  std::vector<int> order;
  bool any_pos = false;
  for (int i = 0; i < n_nano; ++i) any_pos = any_pos || spec[i].launch_pos != 0;
  if (any_pos) {
    order.assign((size_t)n_nano, -1);
    for (int i = 0; i < n_nano; ++i) {
      const int k = spec[i].launch_pos;
      if (k < 0 || k >= n_nano || order[k] >= 0) return NF_EPLAN;
      order[k] = i;
    }
  }
  for (int i = 0; i < n_nano; ++i) {
    if (spec[i].attn_wgs < -1) return NF_EINVAL;
    for (int k = 0; k < 4; ++k)
      if (spec[i].gemm_tile[k] < 0 || spec[i].gemm_tile[k] > 25) return NF_EINVAL;
  }
  nf_plan* p = new (std::nothrow) nf_plan();
  if (!p) return NF_ENOMEM;
  struct Guard {
    nf_plan* p;
    ~Guard() { nf_plan_destroy(p); }
  } guard{p};
  p->model = *model;
  p->bounds.assign(bounds, bounds + n_nano + 1);
  p->origin = "manual";
  p->attn_wgs = spec[0].attn_wgs;
  for (int i = 0; i < n_nano; ++i) p->nano_attn_wgs.push_back(spec[i].attn_wgs);
  nf_plan_default_order(p, overlap ? 1 : 0, order.empty() ? nullptr : order.data());
  for (NfNanoOp& op : p->ops) {
    static const int slot[NF_OP_KINDS] = {0, -1, 1, 2, 3};
    if (slot[op.kind] >= 0) op.gemm_tile = spec[op.nano].gemm_tile[slot[op.kind]];
  }
  p->lane_cus[NF_LANE_ATTN] = attn_cus;
  p->lane_cu_first[NF_LANE_ATTN] = 0;
  p->lane_cus[NF_LANE_GEMM] = gemm_cus;
  p->lane_cu_first[NF_LANE_GEMM] = (gemm_cus && attn_cus + gemm_cus <= ctx->num_cus) ? attn_cus : 0;
  rc = nf_plan_finalize(ctx, p, batch);
  if (rc) return rc;
  guard.p = nullptr;
  *out = p;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_plan_manual_parts(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch,
                                    const nf_partitions* parts, int overlap, int attn_cus, int gemm_cus,
                                    const int32_t* attn_wgs, const int32_t* gemm_tile, nf_plan** out) try {
  if (!ctx || !out || !parts) return NF_EINVAL;
  *out = nullptr;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, INT64_MAX);
  if (rc) return rc;
  if (attn_cus < 0 || gemm_cus < 0 || attn_cus > ctx->num_cus || gemm_cus > ctx->num_cus) return NF_EINVAL;
  if (batch->n_tokens == 0) {  // nothing to split
    const int32_t none[2] = {0, 0};
    return nf_plan_manual(ctx, model, batch, 1, none, overlap, attn_cus, gemm_cus, 0, out);
  }
  NfParts pp;
  for (int k = 0; k < NF_OP_KINDS; ++k) {
    if (parts->n[k] < 1 || parts->n[k] > NF_MAX_PARTS) return NF_EPLAN;
    rc = check_bounds(batch, parts->n[k], parts->bounds[k]);
    if (rc) return rc;
    pp[(size_t)k].assign(parts->bounds[k], parts->bounds[k] + parts->n[k] + 1);
  }
  // the (token, expert) rows of a Down nano-operation are those its Up/Gate nano-operation grouped
  if (model->n_experts > 1 && pp[NF_OP_UG] != pp[NF_OP_D]) return NF_EPLAN;
  for (int i = 0; attn_wgs && i < parts->n[NF_OP_ATTN]; ++i)
    if (attn_wgs[i] < -1) return NF_EINVAL;
  for (int k = 0; gemm_tile && k < 4; ++k)
    if (gemm_tile[k] < 0 || gemm_tile[k] > NF_MAX_TILE) return NF_EINVAL;
  std::vector<NfEmitOp> emit;
  if (!nf_emission_order(pp, &emit)) return NF_EPLAN;
  nf_plan* p = new (std::nothrow) nf_plan();
  if (!p) return NF_ENOMEM;
  struct Guard {
    nf_plan* p;
    ~Guard() { nf_plan_destroy(p); }
  } guard{p};
  p->model = *model;
  p->origin = "manual";
  p->bounds = pp[NF_OP_ATTN];  // the attention work lists and shares are per attention nano-operation
  for (int k = 0; k < NF_OP_KINDS; ++k) p->parts[k] = pp[(size_t)k];
  p->attn_wgs = attn_wgs ? attn_wgs[0] : 0;
  for (int i = 0; i < parts->n[NF_OP_ATTN]; ++i) p->nano_attn_wgs.push_back(attn_wgs ? attn_wgs[i] : 0);
  p->overlap = overlap ? 1 : 0;
  for (const NfEmitOp& e : emit) {
    static const int slot[NF_OP_KINDS] = {0, -1, 1, 2, 3};
    NfNanoOp op;
    op.kind = e.kind;
    op.nano = e.index;
    op.tok_begin = e.tok_begin;
    op.tok_end = e.tok_end;
    op.lane = (p->overlap && e.kind == NF_OP_ATTN) ? NF_LANE_ATTN : NF_LANE_GEMM;
    if (gemm_tile && slot[e.kind] >= 0) op.gemm_tile = gemm_tile[slot[e.kind]];
    p->ops.push_back(op);
  }
  p->lane_cus[NF_LANE_ATTN] = attn_cus;
  p->lane_cu_first[NF_LANE_ATTN] = 0;
  p->lane_cus[NF_LANE_GEMM] = gemm_cus;
  p->lane_cu_first[NF_LANE_GEMM] = (gemm_cus && attn_cus + gemm_cus <= ctx->num_cus) ? attn_cus : 0;
  rc = nf_plan_finalize(ctx, p, batch);
  if (rc) return rc;
  guard.p = nullptr;
  *out = p;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" void nf_plan_destroy(nf_plan* p) {
  if (!p) return;
  for (hipEvent_t e : p->events)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : p->events_alt)
    if (e) (void)hipEventDestroy(e);
  if (p->ev_fork) (void)hipEventDestroy(p->ev_fork);
  for (int l = 0; l < NF_LANES; ++l)
    if (p->ev_join[l]) (void)hipEventDestroy(p->ev_join[l]);
  if (p->dev_blob) g_blobs.release(p->device, p->dev_blob, p->dev_blob_bytes);
  delete p;
}

static std::string list_json(const std::vector<int>& v) {
  std::string s = "[";
  for (size_t i = 0; i < v.size(); ++i) s += (i ? ", " : "") + std::to_string(v[i]);
  return s + "]";
}

static const char* kind_name(int k) {
  static const char* n[] = {"KQV", "ATTN", "O", "UG", "D"};
  return (k >= 0 && k < NF_OP_KINDS) ? n[k] : "?";
}

extern "C" int nf_plan_describe(const nf_plan* p, char* buf, size_t buf_len) try {
  if (!p) return NF_EINVAL;
  std::string s = "{\"origin\": \"" + p->origin + "\", \"n_tokens\": " + std::to_string(p->n_tokens) +
                  ", \"overlap\": " + std::to_string(p->overlap) + ", \"bounds\": [";
  for (size_t i = 0; i < p->bounds.size(); ++i) s += (i ? ", " : "") + std::to_string(p->bounds[i]);
  s += "], \"attn_cus\": " + std::to_string(p->lane_cus[NF_LANE_ATTN]) +
       ", \"gemm_cus\": " + std::to_string(p->lane_cus[NF_LANE_GEMM]) +
       ", \"attn_wgs\": " + std::to_string(p->attn_wgs) + ", \"nano_attn_wgs\": " + list_json(p->nano_attn_wgs) +
       ", \"order\": " + list_json(p->nano_order) + ", \"partitions\": [" + list_json(p->parts[0]) + ", " +
       list_json(p->parts[1]) + ", " + list_json(p->parts[2]) + ", " + list_json(p->parts[3]) + ", " +
       list_json(p->parts[4]) + "], \"attn_parts\": " + std::to_string(p->total_parts) + ", \"est_time_us\": " + std::to_string(p->est_time_us) +
       ", \"ops\": [";
  for (size_t a = 0; a < p->ops.size(); ++a) {
    const NfNanoOp& o = p->ops[a];
    s += std::string(a ? ", " : "") + "{\"op\": \"" + kind_name(o.kind) + "\", \"nano\": " + std::to_string(o.nano) +
         ", \"range\": [" + std::to_string(o.tok_begin) + ", " + std::to_string(o.tok_end) +
         "], \"lane\": " + std::to_string(o.lane) +
         (o.kind == NF_OP_ATTN ? ", \"attn_wgs\": " + std::to_string(o.attn_wgs)
                               : ", \"gemm_tile\": " + std::to_string(o.gemm_tile)) +
         ", \"deps\": [";
    for (size_t d = 0; d < o.deps.size(); ++d) s += (d ? ", " : "") + std::to_string(o.deps[d]);
    s += "]}";
  }
  s += "]}";
  if (buf && buf_len) {
    const size_t n = std::min(buf_len - 1, s.size());
    memcpy(buf, s.data(), n);
    buf[n] = 0;
  }
  return (int)s.size();
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}
