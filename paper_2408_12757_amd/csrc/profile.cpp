// Auto-search, GPU part (paper Sec. 4.1.1): interference-free kernel profiling over batch
// sizes and implementations, pairwise GEMM || attention interference profiling that yields
// the R -> P table, and the entry points that turn a search result into a plan.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "nf_internal.h"
#include "planner.h"

// Objective of the search: 1 = one layer on its own; n > 1 = time per layer of n consecutive
// layers (process-wide tuning knob "search.layers").
static int g_search_layers = 1;
void nf_set_search_layers(int n) { g_search_layers = n; }
int nf_search_layers() { return g_search_layers; }
// Which of the ranked candidates the search returns (tuning knob "search.rank").
static int g_search_rank = 0;
void nf_set_search_rank(int r) { g_search_rank = r; }
static int g_search_refine = 2;
void nf_set_search_refine(int v) { g_search_refine = v; }
static int g_search_max_parts = 0;
void nf_set_search_max_parts(int v) { g_search_max_parts = v; }

void nf_profile_free(nf_ctx* ctx) {
  delete ctx->profile;
  ctx->profile = nullptr;
}

namespace {

constexpr int kTiles[] = {1, 7, 11, 12, 13, 17, 19, 20, 21, 22, 23, 24, 25};  // GEMM implementations (see gemm.hip / gemm_dl.hip)
constexpr int kAttnWgSettings[] = {64, 96, 128, 160, 192, 256, 512};

struct Scratch {
  std::vector<void*> ptrs;
  nf_ctx* ctx;
  explicit Scratch(nf_ctx* c) : ctx(c) {}
  ~Scratch() {
    for (void* p : ptrs) (void)hipFree(p);
  }
  void* get(size_t bytes, int fill) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
    ptrs.push_back(p);
    if (hipMemset(p, fill, bytes) != hipSuccess) return nullptr;
    return p;
  }
  // bf16 buffer of pseudo-random values: dense-kernel speed depends on the data (constant
  // inputs run up to 20 % faster than activations and weights do), so timing buffers are varied
  void* get_random(size_t bytes, float stddev) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
    ptrs.push_back(p);
    if (nf_launch_fill_random(p, bytes / 2, (uint32_t)ptrs.size() * 7919u, stddev, nullptr) != hipSuccess) return nullptr;
    if (hipDeviceSynchronize() != hipSuccess) return nullptr;
    return p;
  }
};

// Average milliseconds of `reps` calls of fn on stream s (one untimed call first).
template <typename F>
int time_ms(nf_ctx* ctx, hipStream_t s, int reps, F fn, double* out_ms) {
  hipEvent_t e0, e1;
  NF_HIP(ctx, hipEventCreate(&e0));
  NF_HIP(ctx, hipEventCreate(&e1));
  int rc = fn();
  if (rc == NF_OK && hipStreamSynchronize(s) != hipSuccess) rc = NF_EHIP;
  if (rc == NF_OK && hipEventRecord(e0, s) != hipSuccess) rc = NF_EHIP;
  for (int i = 0; i < reps && rc == NF_OK; ++i) rc = fn();
  if (rc == NF_OK && hipEventRecord(e1, s) != hipSuccess) rc = NF_EHIP;
  if (rc == NF_OK && hipEventSynchronize(e1) != hipSuccess) rc = NF_EHIP;
  float ms = 0.f;
  if (rc == NF_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = NF_EHIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *out_ms = ms / reps;
  return rc;
}

struct DenseShape {
  int N, K, epi;
};

void dense_shapes(const nf_model_desc* m, DenseShape* s) {
  const int nqkv = (m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
  const int qd = m->n_q_heads * m->head_dim;
  s[NF_DENSE_KQV] = DenseShape{nqkv, m->hidden, NF_EPI_NONE};
  s[NF_DENSE_O] = DenseShape{m->hidden, qd, NF_EPI_RESIDUAL};
  s[NF_DENSE_UG] = DenseShape{m->ffn_inner, m->hidden, NF_EPI_SWIGLU};
  s[NF_DENSE_D] = DenseShape{m->hidden, m->ffn_inner, NF_EPI_RESIDUAL};
}

// Synthetic decode-only batch for attention profiling: n_req requests of ctx cached tokens,
// pages numbered consecutively.
struct SynthBatch {
  std::vector<int32_t> q_indptr, ctx_len, page_indptr, page_ids;
  int32_t *d_q = nullptr, *d_c = nullptr, *d_pi = nullptr, *d_pid = nullptr;
  nf_batch b{};
  int64_t num_pages = 0;
};

int make_synth_batch(nf_ctx* ctx, Scratch& sc, int n_req, int ctx_tokens, SynthBatch* sb) {
  sb->q_indptr.resize(n_req + 1);
  sb->ctx_len.assign(n_req, ctx_tokens);
  sb->page_indptr.resize(n_req + 1);
  const int ppr = (ctx_tokens + 1 + 15) / 16;
  for (int r = 0; r <= n_req; ++r) {
    sb->q_indptr[r] = r;
    sb->page_indptr[r] = r * ppr;
  }
  sb->page_ids.resize((size_t)n_req * ppr);
  for (size_t i = 0; i < sb->page_ids.size(); ++i) sb->page_ids[i] = (int32_t)i;
  sb->num_pages = (int64_t)sb->page_ids.size();
  auto up = [&](const std::vector<int32_t>& v, int32_t** d) {
    *d = (int32_t*)sc.get(std::max<size_t>(4, v.size() * 4), 0);
    if (!*d) return NF_EHIP;
    return hipMemcpy(*d, v.data(), v.size() * 4, hipMemcpyHostToDevice) == hipSuccess ? NF_OK : NF_EHIP;
  };
  int rc = up(sb->q_indptr, &sb->d_q);
  if (!rc) rc = up(sb->ctx_len, &sb->d_c);
  if (!rc) rc = up(sb->page_indptr, &sb->d_pi);
  if (!rc) rc = up(sb->page_ids, &sb->d_pid);
  if (rc) {
    ctx->last_hip = (int)hipGetLastError();
    return rc;
  }
  sb->b = nf_batch{n_req, 0, n_req, sb->d_q, sb->d_c, sb->d_pi, sb->d_pid,
                   sb->q_indptr.data(), sb->ctx_len.data(), sb->page_indptr.data(), sb->page_ids.data()};
  return NF_OK;
}

int measure(nf_ctx* ctx, const nf_model_desc* m, int max_tokens, int granule, NfProfile* p) {
  NF_HIP(ctx, hipSetDevice(ctx->device));
  Scratch sc(ctx);
  hipStream_t sg = nullptr, sa = nullptr;
  int rc = nf_get_lane_stream(ctx, NF_LANE_GEMM, 0, 0, &sg);
  if (!rc) rc = nf_get_lane_stream(ctx, NF_LANE_ATTN, 0, 0, &sa);
  if (rc) return rc;
  nf_profile_analytic(p, m, max_tokens, granule);
  DenseShape shp[NF_DENSE_OPS];
  dense_shapes(m, shp);
  const int steps = (int)p->dense_us[0].size();
  const size_t Mmax = (size_t)steps * granule;

  // ---- interference-free dense operations: every batch size x every tile shape ----
  size_t max_in = 0, max_out = 0, max_w = 0;
  for (int o = 0; o < NF_DENSE_OPS; ++o) {
    max_in = std::max(max_in, Mmax * shp[o].K * 2);
    max_out = std::max(max_out, Mmax * shp[o].N * 2);
    max_w = std::max(max_w, (size_t)shp[o].N * (shp[o].epi == NF_EPI_SWIGLU ? 2 : 1) * shp[o].K * 2);
  }
  void* x = sc.get_random(max_in, 1.0f);
  void* y = sc.get(max_out, 0);
  void* res = sc.get_random(max_out, 1.0f);
  // alternate so weights are not cache-warm
  void* w[2] = {sc.get_random(max_w, 0.02f), sc.get_random(max_w, 0.02f)};
  // scratch of the two-segment operations, as the layer's workspace provides it
  void* partial = sc.get(2 * Mmax * (size_t)m->hidden * sizeof(float), 0);
  if (!x || !y || !res || !w[0] || !w[1] || !partial) {
    ctx->last_hip = (int)hipErrorOutOfMemory;
    return NF_EHIP;
  }
  const NfGemmSplit split{m->n_experts > 1 ? nullptr : (float*)partial, (long long)(Mmax * (size_t)m->hidden)};
  for (int o = 0; o < NF_DENSE_OPS; ++o) {
    for (int i = 0; i < steps; ++i) {
      const int M = (i + 1) * granule;
      double best = 1e300;
      int best_tile = 1;
      for (int tile : kTiles) {
        // the 192-column forms have no SwiGLU epilogue and need 192 | N: such an operation would
        // run (and be listed under) the implementation they fall back to
        if ((tile == 20 || tile == 23 || tile == 24) && (shp[o].epi == NF_EPI_SWIGLU || shp[o].N % 192 != 0)) continue;
        int flip = 0;
        double ms = 0;
        rc = time_ms(ctx, sg, 6, [&] {
          flip ^= 1;
          return nf_launch_gemm(x, w[flip], y, res, M, shp[o].N, shp[o].K, shp[o].epi, tile, sg, split) == hipSuccess
                     ? NF_OK
                     : NF_EHIP;
        }, &ms);
        if (rc) return rc;
        if (i == 0) p->tile_us[tile][o].assign(steps, 0.0);
        p->tile_us[tile][o][i] = ms * 1e3;
        if (ms < best) {
          best = ms;
          best_tile = tile;
        }
      }
      p->dense_us[o][i] = best * 1e3;
      p->dense_tile[o][i] = best_tile;
    }
  }

  // ---- interference-free attention: long contexts for the per-byte cost, short for the fixed cost ----
  const int n_req = std::max(16, std::min(max_tokens, 512));
  const size_t page_bytes = (size_t)2 * m->n_kv_heads * 16 * m->head_dim * 2;
  const int32_t nqkv = (m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
  void* qkv = sc.get_random((size_t)n_req * nqkv * 2, 1.0f);
  void* aout = sc.get((size_t)n_req * m->n_q_heads * m->head_dim * 2, 0);
  if (!qkv || !aout) return NF_EHIP;
  const NfAttnShape ash{m->n_q_heads, m->n_kv_heads, m->head_dim, nqkv};
  double t_short_ms = 0, t_long_ms[sizeof(kAttnWgSettings) / sizeof(int)] = {0};
  double long_mb = 0;
  nf_plan* plans[2] = {nullptr, nullptr};
  SynthBatch sb[2];
  void* pool = nullptr;
  float* parts = nullptr;
  const int ctx_tokens[2] = {48, 2047};
  for (int v = 1; v >= 0 && !rc; --v) {
    rc = make_synth_batch(ctx, sc, n_req, ctx_tokens[v], &sb[v]);
    if (rc) break;
    if (v == 1) {
      pool = sc.get_random((size_t)sb[1].num_pages * page_bytes, 1.0f);
      if (!pool) return NF_EHIP;
    }
    const int32_t bounds[2] = {0, n_req};
    rc = nf_plan_manual(ctx, m, &sb[v].b, 1, bounds, 0, 0, 0, 0, &plans[v]);
    if (rc) break;
    if (v == 1) {
      // (no partial results at all when every context fits one chunk)
      parts = (float*)sc.get(std::max<size_t>(256, (size_t)plans[1]->total_parts * m->n_kv_heads *
                                                       nf_attn_part_floats(m->head_dim) * 4), 0);
      if (!parts) rc = NF_EHIP;
    }
  }
  auto attn_call = [&](int v, int wgs, hipStream_t s) {
    hipError_t e = nf_launch_attention(qkv, pool, sb[v].d_pi, sb[v].d_pid, plans[v]->d_items, plans[v]->item_cnt[0],
                                       ash, parts, aout, wgs, s, plans[v]->item_pages[0]);
    if (e == hipSuccess)
      e = nf_launch_attention_merge(parts, plans[v]->d_groups, plans[v]->group_cnt[0], ash, aout, s);
    return e == hipSuccess ? NF_OK : NF_EHIP;
  };
  const int n_set = (int)(sizeof(kAttnWgSettings) / sizeof(int));
  double best_long = 1e300;
  if (!rc) rc = time_ms(ctx, sa, 5, [&] { return attn_call(0, 0, sa); }, &t_short_ms);
  for (int k = 0; k < n_set && !rc; ++k) {
    rc = time_ms(ctx, sa, 3, [&] { return attn_call(1, kAttnWgSettings[k], sa); }, &t_long_ms[k]);
    best_long = std::min(best_long, t_long_ms[k]);
  }
  if (!rc) {
    long_mb = (double)n_req * (ctx_tokens[1] + 1) * (page_bytes / 16) / 1e6;
    const double short_mb = (double)n_req * (ctx_tokens[0] + 1) * (page_bytes / 16) / 1e6;
    p->attn_us_per_mb = std::max(1e-6, (best_long - t_short_ms) * 1e3 / (long_mb - short_mb));
    p->attn_fixed_us = std::max(1.0, t_short_ms * 1e3 - p->attn_us_per_mb * short_mb);
  }

  // ---- the small row-wise kernels at n_req tokens: per-token cost, launch cost assumed 4 us each ----
  if (!rc) {
    double t_rms = 0, t_rope = 0, t_merge = 0;
    rc = time_ms(ctx, sg, 5, [&] {
      return nf_launch_rmsnorm(x, res, y, n_req, m->hidden, m->rms_eps, sg) == hipSuccess ? NF_OK : NF_EHIP;
    }, &t_rms);
    if (!rc)
      rc = time_ms(ctx, sg, 5, [&] {
        return nf_launch_rope_append(qkv, pool, plans[1]->d_tok_req, sb[1].d_q, sb[1].d_c, sb[1].d_pi, sb[1].d_pid, 0,
                                     n_req, m->n_q_heads, m->n_kv_heads, m->head_dim, m->rope_theta, 0, sg) == hipSuccess
                   ? NF_OK
                   : NF_EHIP;
      }, &t_rope);
    if (!rc)
      rc = time_ms(ctx, sg, 5, [&] {
        return nf_launch_attention_merge(parts, plans[1]->d_groups, plans[1]->group_cnt[0], ash, aout, sg) == hipSuccess
                   ? NF_OK
                   : NF_EHIP;
      }, &t_merge);
    if (!rc) {
      const double fixed = 4.0;
      auto per_tok = [&](double ms) { return std::max(0.0, ms * 1e3 - fixed) / n_req; };
      p->misc_kqv[0] = 2 * fixed;
      p->misc_kqv[1] = per_tok(t_rms) + per_tok(t_rope);
      p->misc_rest[0] = fixed;
      p->misc_rest[1] = per_tok(t_rms);
      p->misc_attn[0] = fixed;
      p->misc_attn[1] = per_tok(t_merge);
    }
  }

  // ---- latency of a dependency across the two lanes: a chain of tiny kernels that alternates
  // between the streams (event record, event wait) against the same chain on one stream ----
  if (!rc) {
    constexpr int kHops = 16;
    std::vector<hipEvent_t> ev(2 * kHops);
    for (auto& e : ev)
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) rc = NF_EHIP;
    auto tiny = [&](hipStream_t s) { return nf_launch_rmsnorm(x, res, y, 1, m->hidden, m->rms_eps, s); };
    double t_same = 0, t_cross = 0;
    if (!rc)
      rc = time_ms(ctx, sg, 3, [&] {
        for (int i = 0; i < 2 * kHops; ++i)
          if (tiny(sg) != hipSuccess) return NF_EHIP;
        return NF_OK;
      }, &t_same);
    if (!rc)
      rc = time_ms(ctx, sg, 3, [&] {
        for (int i = 0; i < kHops; ++i) {
          hipError_t e = tiny(sg);
          if (e == hipSuccess) e = hipEventRecord(ev[2 * i], sg);
          if (e == hipSuccess) e = hipStreamWaitEvent(sa, ev[2 * i], 0);
          if (e == hipSuccess) e = tiny(sa);
          if (e == hipSuccess) e = hipEventRecord(ev[2 * i + 1], sa);
          if (e == hipSuccess) e = hipStreamWaitEvent(sg, ev[2 * i + 1], 0);
          if (e != hipSuccess) return NF_EHIP;
        }
        return NF_OK;
      }, &t_cross);
    (void)hipDeviceSynchronize();
    for (auto& e : ev) (void)hipEventDestroy(e);
    if (!rc) p->sync_us = std::max(0.0, (t_cross - t_same) * 1e3 / (2 * kHops));
  }

  // ---- pairwise interference: the GEMM work of a two-nano-batch pipeline (O, Up/Gate, Down and
  // the next KQV on half of the batch, in every tile shape) || attention with k persistent
  // workgroups.  Performance is normalised to the best stand-alone implementation of each
  // kernel.  One "GEMM" below is that group of four. ----
  if (!rc) {
    const int half_steps = std::max(1, steps / 2);
    const int M = half_steps * granule;
    double g_best_ms = 0;
    for (int o = 0; o < NF_DENSE_OPS; ++o) g_best_ms += p->dense_us[o][half_steps - 1] / 1e3;
    const int kPairTiles[] = {7, 12, 13, 19, 21, 22, 25};
    p->rp.clear();
    for (int tile : kPairTiles) {
      if (rc) break;
      int flip = 0;
      auto launch_group = [&]() -> hipError_t {
        static const int order[NF_DENSE_OPS] = {NF_DENSE_O, NF_DENSE_UG, NF_DENSE_D, NF_DENSE_KQV};
        flip ^= 1;
        for (int o : order) {
          hipError_t e = nf_launch_gemm(x, w[flip], y, res, M, shp[o].N, shp[o].K, shp[o].epi, tile, sg, split);
          if (e != hipSuccess) return e;
        }
        return hipSuccess;
      };
      double g_solo_ms = 0;
      rc = time_ms(ctx, sg, 3, [&] { return launch_group() == hipSuccess ? NF_OK : NF_EHIP; }, &g_solo_ms);
      if (rc) break;
      // kAttnReps attention launches back to back: the pair is measured in a sustained state
      // (a single launch sees clocks that a longer co-run does not keep)
      constexpr int kAttnReps = 5;
      const int n_gemm = std::min(160, (int)ceil(3.0 * kAttnReps * best_long / g_solo_ms) + 2);
      std::vector<hipEvent_t> ev((size_t)n_gemm + 3);
      for (auto& e : ev)
        if (hipEventCreate(&e) != hipSuccess) rc = NF_EHIP;
      hipEvent_t fork = ev[n_gemm], a0 = ev[n_gemm + 1], a1 = ev[n_gemm + 2];
      for (int k = 0; k < n_set && !rc; ++k) {
        (void)hipDeviceSynchronize();
        hipError_t e = hipEventRecord(fork, sg);
        if (e == hipSuccess) e = hipStreamWaitEvent(sa, fork, 0);
        // GEMMs first in issue order; attention joins right behind
        for (int i = 0; i < n_gemm && e == hipSuccess; ++i) {
          e = launch_group();
          if (e == hipSuccess) e = hipEventRecord(ev[i], sg);
          if (i == 0 && e == hipSuccess) {
            e = hipEventRecord(a0, sa);
            for (int rep = 0; rep < kAttnReps && e == hipSuccess; ++rep)
              if (attn_call(1, kAttnWgSettings[k], sa) != NF_OK) e = hipErrorUnknown;
            if (e == hipSuccess) e = hipEventRecord(a1, sa);
          }
        }
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) {
          ctx->last_hip = (int)e;
          rc = NF_EHIP;
          break;
        }
        float t_a0 = 0, t_a1 = 0;
        (void)hipEventElapsedTime(&t_a0, fork, a0);
        (void)hipEventElapsedTime(&t_a1, fork, a1);
        // GEMM work (in units of one GEMM) finished inside the attention window [t_a0, t_a1]
        auto progress_at = [&](float t) {
          float prev = 0.f;
          for (int i = 0; i < n_gemm; ++i) {
            float ti = 0;
            (void)hipEventElapsedTime(&ti, fork, ev[i]);
            if (t <= ti) return (double)i + (double)(t - prev) / std::max(1e-6f, ti - prev);
            prev = ti;
          }
          return (double)n_gemm;
        };
        const double done = progress_at(t_a1) - progress_at(t_a0);
        const double window = std::max(1e-6, (double)(t_a1 - t_a0));
        NfRpRow row;
        row.attn_wgs = kAttnWgSettings[k];
        row.gemm_tile = tile;
        // one GEMM of this tile is worth g_best_ms of the best implementation's time
        row.p_gemm = std::min(1.0, done * g_best_ms / window);
        row.p_attn = std::min(1.0, kAttnReps * best_long / window);
        row.p_attn_solo = std::min(1.0, best_long / t_long_ms[k]);
        row.p_gemm_solo = std::min(1.0, g_best_ms / g_solo_ms);
        p->rp.push_back(row);
      }
      for (auto& e : ev) (void)hipEventDestroy(e);
    }
    // discard dominated pairs: another pair is better for both kernels (Sec. 4.1.1, the
    // greyed-out pairs) - by more than two measurements of one pair differ by (a tenth: how the
    // hardware happens to place the persistent workgroups decides that much), so that a pair within
    // the scatter of its neighbour stays a candidate of the search
    constexpr double kNoise = 1.10;
    std::vector<NfRpRow> keep;
    for (const NfRpRow& r : p->rp) {
      bool dominated = false;
      for (const NfRpRow& q : p->rp)
        if (&q != &r && q.p_gemm >= kNoise * r.p_gemm && q.p_attn >= kNoise * r.p_attn) dominated = true;
      if (!dominated) keep.push_back(r);
    }
    p->rp = keep;
  }
  for (nf_plan* pl : plans) nf_plan_destroy(pl);
  (void)hipDeviceSynchronize();
  if (!rc) p->measured = true;
  return rc;
}

bool same_shape(const nf_model_desc& a, const nf_model_desc& b) {
  return a.hidden == b.hidden && a.n_q_heads == b.n_q_heads && a.n_kv_heads == b.n_kv_heads &&
         a.head_dim == b.head_dim && a.ffn_inner == b.ffn_inner;
}

// The search's knobs: the process-wide ones of nf_tune_set, or those a caller passes with
// nf_plan_search.
struct SearchKnobs {
  int layers, rank, refine, max_parts;
};
SearchKnobs process_knobs() { return SearchKnobs{nf_search_layers(), g_search_rank, g_search_refine, g_search_max_parts}; }

void build_search_input(const nf_model_desc* m, const nf_batch* b, int max_nano, int granule, NfSearchInput* in,
                        const SearchKnobs& knobs = process_knobs()) {
  const int n_reqs = b->n_prefill_reqs + b->n_decode_reqs;
  in->n_tokens = b->n_tokens;
  in->granule = granule;
  in->max_nano = max_nano;
  in->layers = knobs.layers;
  in->rank = knobs.rank;
  in->refine = knobs.refine;
  in->max_parts = knobs.max_parts;
  in->tie_ffn = m->n_experts > 1;
  in->attn_mb_prefix.assign((size_t)b->n_tokens + 1, 0.0);
  in->req_start_of_tok.assign((size_t)b->n_tokens, 0);
  const double tok_mb = 2.0 * m->n_kv_heads * m->head_dim * 2 / 1e6;
  const int T = std::max(1, 16 / (m->n_q_heads / m->n_kv_heads));
  for (int r = 0; r < n_reqs; ++r) {
    const int q0 = b->host_q_indptr[r], q1 = b->host_q_indptr[r + 1];
    for (int t = q0; t < q1; ++t) {
      const double keys = (double)b->host_ctx_len[r] + (t - q0) + 1;
      // the rows of one group (T tokens of a prefill chunk) share one pass over the keys
      const double share = (q1 - q0 > 1) ? 1.0 / T : 1.0;
      in->attn_mb_prefix[t + 1] = in->attn_mb_prefix[t] + keys * tok_mb * share;
      in->req_start_of_tok[t] = q0;
    }
  }
}

const NfProfile* pick_profile(const nf_ctx* ctx, const nf_model_desc* m, int n_tokens, int granule, NfProfile* tmp) {
  if (ctx && ctx->profile && same_shape(ctx->profile->model, *m) && ctx->profile->granule == granule &&
      ctx->profile->max_tokens >= n_tokens)
    return ctx->profile;
  nf_profile_analytic(tmp, m, std::max(n_tokens, granule), granule);
  return tmp;
}

}  // namespace

extern "C" int nf_profile(nf_ctx* ctx, const nf_model_desc* model, int max_tokens, int granule,
                          const char* cache_path) try {
  if (!ctx || max_tokens < 1 || granule < 1) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  NfProfile* p = new (std::nothrow) NfProfile();
  if (!p) return NF_ENOMEM;
  if (cache_path && nf_profile_load(p, cache_path) == NF_OK && same_shape(p->model, *model) &&
      p->granule == granule && p->max_tokens >= max_tokens) {
    nf_profile_free(ctx);
    ctx->profile = p;
    return NF_OK;
  }
  rc = measure(ctx, model, max_tokens, granule, p);
  if (rc) {
    delete p;
    return rc;
  }
  nf_profile_free(ctx);
  ctx->profile = p;
  if (cache_path) return nf_profile_save(*p, cache_path);
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_search_pipeline(const nf_model_desc* model, const nf_batch* batch, const char* profile_path,
                                  int max_nano, int granule, nf_pipeline_desc* out) try {
  if (!out || granule < 1 || max_nano < 0) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, INT64_MAX);
  if (rc) return rc;
  NfProfile prof;
  if (profile_path) {
    rc = nf_profile_load(&prof, profile_path);
    if (rc) return rc;
  } else {
    nf_profile_analytic(&prof, model, std::max(batch->n_tokens, granule), granule);
  }
  NfSearchInput in;
  build_search_input(model, batch, max_nano, granule, &in);
  NfPipeline pl;
  rc = nf_search(prof, in, &pl);
  if (rc) return rc;
  memset(out, 0, sizeof *out);
  out->n_nano = (int32_t)pl.bounds.size() - 1;
  for (size_t i = 0; i < pl.bounds.size() && i < 9; ++i) out->bounds[i] = pl.bounds[i];
  out->overlap = pl.overlap;
  out->attn_wgs = pl.attn_wgs;
  out->gemm_tile = pl.gemm_tile;
  for (int i = 0; i < out->n_nano && i < 8; ++i) {
    out->nano_attn_wgs[i] = pl.nano_attn_wgs.empty() ? pl.attn_wgs : pl.nano_attn_wgs[(size_t)i];
    out->order[i] = pl.order.empty() ? i : pl.order[(size_t)i];
  }
  if (!pl.parts[0].empty())
    for (int k = 0; k < NF_PART_KINDS; ++k) {
      out->parts.n[k] = (int32_t)pl.parts[(size_t)k].size() - 1;
      for (size_t i = 0; i < pl.parts[(size_t)k].size() && i < 9; ++i) out->parts.bounds[k][i] = pl.parts[(size_t)k][i];
    }
  out->est_us = pl.est_us;
  out->est_us_stage1 = pl.est_us_stage1;
  out->est_us_unsplit = pl.est_us_unsplit;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_simulate_pipeline(const nf_model_desc* model, const nf_batch* batch, const char* profile_path,
                                    int n_nano, const int32_t* bounds, int overlap, int rp_row, double* est_us) try {
  if (!est_us || !bounds || n_nano < 1) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, INT64_MAX);
  if (rc) return rc;
  NfProfile prof;
  if (profile_path) {
    rc = nf_profile_load(&prof, profile_path);
    if (rc) return rc;
  } else {
    nf_profile_analytic(&prof, model, std::max(batch->n_tokens, 128), 128);
  }
  if (bounds[0] != 0 || bounds[n_nano] != batch->n_tokens) return NF_EPLAN;
  for (int i = 0; i < n_nano; ++i)
    if (bounds[i + 1] <= bounds[i]) return NF_EPLAN;
  if (rp_row >= (int)prof.rp.size()) return NF_EINVAL;
  NfSearchInput in;
  build_search_input(model, batch, 0, prof.granule, &in);
  *est_us = nf_simulate_per_layer(prof, in, std::vector<int>(bounds, bounds + n_nano + 1), overlap,
                                  rp_row < 0 ? nullptr : &prof.rp[rp_row]);
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_simulate_pipeline_ops(const nf_model_desc* model, const nf_batch* batch, const char* profile_path,
                                        int n_nano, const int32_t* bounds, const int32_t* rp_rows,
                                        const int32_t* order, double* est_us) try {
  if (!est_us || !bounds || !rp_rows || n_nano < 1 || n_nano > 8) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, INT64_MAX);
  if (rc) return rc;
  NfProfile prof;
  if (!profile_path) return NF_EINVAL;  // per-row simulation needs a table
  rc = nf_profile_load(&prof, profile_path);
  if (rc) return rc;
  if (bounds[0] != 0 || bounds[n_nano] != batch->n_tokens) return NF_EPLAN;
  for (int i = 0; i < n_nano; ++i)
    if (bounds[i + 1] <= bounds[i]) return NF_EPLAN;
  std::vector<const NfRpRow*> rows;
  std::vector<int> ord;
  for (int i = 0; i < n_nano; ++i) {
    if (rp_rows[i] < 0 || rp_rows[i] >= (int)prof.rp.size()) return NF_EINVAL;
    rows.push_back(&prof.rp[(size_t)rp_rows[i]]);
    if (order) ord.push_back(order[i]);
  }
  NfSearchInput in;
  build_search_input(model, batch, 0, prof.granule, &in);
  const std::vector<int> b(bounds, bounds + n_nano + 1);
  double t = nf_simulate_ops(prof, in, b, rows, ord, 1);
  if (t >= 0 && in.layers > 1) t = (nf_simulate_ops(prof, in, b, rows, ord, in.layers) - t) / (in.layers - 1);
  if (t < 0) return NF_EPLAN;
  *est_us = t;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

// nf_partitions -> NfParts; false unless every operation has 1..8 nano-operations
static bool parts_from_c(const nf_partitions* c, NfParts* out) {
  for (int k = 0; k < NF_PART_KINDS; ++k) {
    if (c->n[k] < 1 || c->n[k] > NF_MAX_PARTS) return false;
    (*out)[(size_t)k].assign(c->bounds[k], c->bounds[k] + c->n[k] + 1);
  }
  return true;
}

extern "C" int nf_simulate_pipeline_parts(const nf_model_desc* model, const nf_batch* batch, const char* profile_path,
                                          const nf_partitions* parts, int overlap, const int32_t* rp_rows,
                                          double* est_us) try {
  if (!est_us || !parts) return NF_EINVAL;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, INT64_MAX);
  if (rc) return rc;
  NfProfile prof;
  if (profile_path) {
    rc = nf_profile_load(&prof, profile_path);
    if (rc) return rc;
  } else {
    if (rp_rows) return NF_EINVAL;  // rows need a table
    nf_profile_analytic(&prof, model, std::max(batch->n_tokens, 128), 128);
  }
  NfParts p;
  if (!parts_from_c(parts, &p)) return NF_EPLAN;
  std::vector<const NfRpRow*> rows;
  for (int i = 0; rp_rows && i < parts->n[1]; ++i) {
    if (rp_rows[i] < 0 || rp_rows[i] >= (int)prof.rp.size()) return NF_EINVAL;
    rows.push_back(&prof.rp[(size_t)rp_rows[i]]);
  }
  NfSearchInput in;
  build_search_input(model, batch, 0, prof.granule, &in);
  double t = nf_simulate_parts(prof, in, p, overlap, rows, 1);
  if (t >= 0 && in.layers > 1) {
    const double tl = nf_simulate_parts(prof, in, p, overlap, rows, in.layers);
    t = tl < 0 ? tl : (tl - t) / (in.layers - 1);
  }
  if (t < 0) return NF_EPLAN;
  *est_us = t;
  return NF_OK;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

static int plan_search(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch, int max_nano, int granule,
                       const SearchKnobs& knobs, nf_plan** out);

extern "C" int nf_plan_nanobatches(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch, int max_nano,
                                   int granule, nf_plan** out) try {
  return plan_search(ctx, model, batch, max_nano, granule, process_knobs(), out);
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

extern "C" int nf_plan_search(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch,
                              const nf_search_options* opt, nf_plan** out) try {
  if (!opt) return NF_EINVAL;
  if (opt->layers < 1 || opt->layers > 16 || opt->rank < 0 || opt->rank > 64 || opt->refine < 0 || opt->refine > 2 ||
      opt->max_parts < 0 || opt->max_parts > NF_MAX_PARTS)
    return NF_EINVAL;
  return plan_search(ctx, model, batch, opt->max_nano, opt->granule,
                     SearchKnobs{opt->layers, opt->rank, opt->refine, opt->max_parts}, out);
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

static int plan_search(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch, int max_nano, int granule,
                       const SearchKnobs& knobs, nf_plan** out) {
  if (!ctx || !out || granule < 1 || max_nano < 0) return NF_EINVAL;
  *out = nullptr;
  int rc = nf_validate_model(model);
  if (rc) return rc;
  rc = nf_validate_batch(model, batch, INT64_MAX);
  if (rc) return rc;
  NfProfile tmp;
  const NfProfile* prof = pick_profile(ctx, model, batch->n_tokens, granule, &tmp);
  NfSearchInput in;
  build_search_input(model, batch, max_nano, granule, &in, knobs);
  NfPipeline pl;
  rc = nf_search(*prof, in, &pl);
  if (rc) return rc;
  std::vector<int32_t> b32(pl.bounds.begin(), pl.bounds.end());
  const int n_nano = (int)b32.size() - 1;
  if (!pl.parts[0].empty()) {
    nf_partitions c;
    memset(&c, 0, sizeof c);
    for (int k = 0; k < NF_PART_KINDS; ++k) {
      c.n[k] = (int32_t)pl.parts[(size_t)k].size() - 1;
      for (size_t i = 0; i < pl.parts[(size_t)k].size(); ++i) c.bounds[k][i] = pl.parts[(size_t)k][i];
    }
    std::vector<int32_t> wgs((size_t)c.n[1], pl.attn_wgs);
    for (size_t i = 0; i < wgs.size() && i < pl.nano_attn_wgs.size(); ++i) wgs[i] = pl.nano_attn_wgs[i];
    rc = nf_plan_manual_parts(ctx, model, batch, &c, pl.overlap, 0, 0, wgs.data(), nullptr, out);
    if (rc == NF_OK) (*out)->attn_wgs = pl.attn_wgs;
  } else if (pl.nano_attn_wgs.empty() && pl.order.empty()) {
    rc = nf_plan_manual(ctx, model, batch, n_nano, b32.data(), pl.overlap, 0, 0, pl.attn_wgs, out);
  } else {
    std::vector<nf_nano_spec> spec((size_t)n_nano);
    for (int i = 0; i < n_nano; ++i) {
      memset(&spec[(size_t)i], 0, sizeof(nf_nano_spec));
      spec[(size_t)i].attn_wgs = pl.nano_attn_wgs.empty() ? pl.attn_wgs : pl.nano_attn_wgs[(size_t)i];
    }
    for (int k = 0; k < n_nano && !pl.order.empty(); ++k) spec[(size_t)pl.order[(size_t)k]].launch_pos = k;
    rc = nf_plan_manual_ops(ctx, model, batch, n_nano, b32.data(), pl.overlap, 0, 0, spec.data(), out);
    if (rc == NF_OK) (*out)->attn_wgs = pl.attn_wgs;
  }
  if (rc) return rc;
  (*out)->origin = prof->measured ? "search(measured profile)" : "search(analytic profile)";
  (*out)->est_time_us = pl.est_us;
  // Nano-operations that cannot have an attention kernel beside them in a single layer: the first
  // KQV nano-operation (every attention nano-operation waits for it) and everything launched
  // from the O nano-operation that waits for the last attention nano-operation on.  They take the
  // implementation that is fastest alone, not the one of the chosen R -> P pair.
  std::vector<char> runs_alone((*out)->ops.size(), 0);
  if (pl.overlap && knobs.layers <= 1) {
    int last_attn = -1, first_kqv = -1;
    for (size_t i = 0; i < (*out)->ops.size(); ++i) {
      if ((*out)->ops[i].kind == NF_OP_ATTN) last_attn = (int)i;
      if ((*out)->ops[i].kind == NF_OP_KQV && first_kqv < 0) first_kqv = (int)i;
    }
    if (first_kqv >= 0) runs_alone[(size_t)first_kqv] = 1;
    bool tail = false;
    for (size_t i = 0; i < (*out)->ops.size(); ++i) {
      const NfNanoOp& op = (*out)->ops[i];
      if (op.kind == NF_OP_O && std::find(op.deps.begin(), op.deps.end(), last_attn) != op.deps.end()) tail = true;
      if (tail && op.kind != NF_OP_ATTN) runs_alone[i] = 1;
    }
  }
  // implementation map (Sec. 4.1.1): best GEMM tile per (operation, batch size)
  for (NfNanoOp& op : (*out)->ops) {
    const int dense = op.kind == NF_OP_KQV ? NF_DENSE_KQV
                      : op.kind == NF_OP_O ? NF_DENSE_O
                      : op.kind == NF_OP_UG ? NF_DENSE_UG
                      : op.kind == NF_OP_D ? NF_DENSE_D
                                           : -1;
    if (dense < 0 || prof->dense_tile[dense].empty()) continue;
    const int m = op.tok_end - op.tok_begin;
    const int idx = std::min((int)prof->dense_tile[dense].size() - 1, std::max(0, (m + granule - 1) / granule - 1));
    const bool alone = runs_alone[(size_t)(&op - (*out)->ops.data())] != 0;
    op.gemm_tile = (pl.overlap && pl.gemm_tile && !alone) ? pl.gemm_tile : prof->dense_tile[dense][idx];
  }
  return NF_OK;
}
