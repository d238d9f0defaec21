// Auto-search, host part (paper Sec. 4.1.2 - 4.1.3): a discrete-event model of the two-lane
// nano-operation pipeline and the two-stage search over its structure and resource share.
//
// Stage I enumerates the number and the boundaries of the nano-batches (multiples of the
// granule) and ranks the structures by their makespan WITHOUT interference, using the
// interference-free kernel times.  Stage II keeps the best structures and, for each row of
// the R -> P table, recomputes the makespan with the overlapped kernels slowed to p_gemm and
// p_attn; the fastest (structure, row) wins, unless running unsplit is estimated faster.
// The instance has no network operations, so exhaustive enumeration replaces the MILP.
#include "planner.h"

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>

static double interp_table(const std::vector<double>& t, int granule, int m);

double nf_profile_dense_us(const NfProfile& p, int op, int m) { return interp_table(p.dense_us[op], p.granule, m); }

double nf_profile_tile_us(const NfProfile& p, int tile, double p_solo, int op, int m) {
  if (tile >= 1 && tile <= NF_MAX_TILE && !p.tile_us[tile][op].empty())
    return interp_table(p.tile_us[tile][op], p.granule, m);
  return nf_profile_dense_us(p, op, m) / std::max(p_solo, 1e-6);
}

static double interp_table(const std::vector<double>& t, int granule, int m) {
  if (t.empty() || m <= 0) return 0.0;
  const double x = (double)m / granule;  // table index + 1
  if (x <= 1.0) return t[0];               // a partial tile costs a whole one
  const int i = (int)floor(x) - 1;
  if (i + 1 >= (int)t.size()) return t.back() * (x / (double)t.size());
  const double f = x - floor(x);
  return t[i] + f * (t[i + 1] - t[i]);
}

void nf_profile_analytic(NfProfile* p, const nf_model_desc* m, int max_tokens, int granule) {
  p->model = *m;
  p->granule = granule;
  p->max_tokens = max_tokens;
  p->measured = false;
  const double nqkv = (double)(m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
  const double qd = (double)m->n_q_heads * m->head_dim;
  const double NK[NF_DENSE_OPS][2] = {{nqkv, (double)m->hidden},
                                      {(double)m->hidden, qd},
                                      {2.0 * m->ffn_inner, (double)m->hidden},
                                      {(double)m->hidden, (double)m->ffn_inner}};
  const int steps = std::max(1, (max_tokens + granule - 1) / granule);
  for (int o = 0; o < NF_DENSE_OPS; ++o) {
    p->dense_us[o].assign(steps, 0.0);
    p->dense_tile[o].assign(steps, 0);  // nothing measured: leave the implementation to the launcher
    for (int i = 0; i < steps; ++i) {
      const double M = (double)(i + 1) * granule;
      const double flops = 2.0 * M * NK[o][0] * NK[o][1];
      const double bytes = 2.0 * (NK[o][0] * NK[o][1] + M * NK[o][1] + M * NK[o][0]);
      p->dense_us[o][i] = 8.0 + std::max(flops / 0.85e15, bytes / 3.0e12) * 1e6;
    }
  }
  p->attn_fixed_us = 8.0;
  p->attn_us_per_mb = 1.0 / 5.8;
  for (int t = 0; t <= NF_MAX_TILE; ++t)
    for (int o = 0; o < NF_DENSE_OPS; ++o) p->tile_us[t][o].clear();
  p->rp.clear();
}

int nf_profile_save(const NfProfile& p, const char* path) {
  FILE* f = fopen(path, "w");
  if (!f) return NF_EIO;
  const nf_model_desc& m = p.model;
  fprintf(f, "nfprofile 1\n");
  fprintf(f, "model %d %d %d %d %d %d %d\n", m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_inner,
          m.n_experts, m.top_k);
  fprintf(f, "granule %d max_tokens %d measured %d\n", p.granule, p.max_tokens, p.measured ? 1 : 0);
  for (int o = 0; o < NF_DENSE_OPS; ++o)
    for (size_t i = 0; i < p.dense_us[o].size(); ++i)
      fprintf(f, "dense %d %d %.4f %d\n", o, (int)(i + 1) * p.granule, p.dense_us[o][i], p.dense_tile[o][i]);
  for (int t = 1; t <= NF_MAX_TILE; ++t)
    for (int o = 0; o < NF_DENSE_OPS; ++o)
      for (size_t i = 0; i < p.tile_us[t][o].size(); ++i)
        fprintf(f, "tile_us %d %d %d %.4f\n", t, o, (int)(i + 1) * p.granule, p.tile_us[t][o][i]);
  fprintf(f, "misc %.4f %.6f %.4f %.6f %.4f %.6f\n", p.misc_kqv[0], p.misc_kqv[1], p.misc_rest[0], p.misc_rest[1],
          p.misc_attn[0], p.misc_attn[1]);
  fprintf(f, "attn %.6f %.8f\n", p.attn_fixed_us, p.attn_us_per_mb);
  for (const NfRpRow& r : p.rp)
    fprintf(f, "rp %d %.6f %.6f %.6f %d %.6f\n", r.attn_wgs, r.p_gemm, r.p_attn, r.p_attn_solo, r.gemm_tile,
            r.p_gemm_solo);
  return fclose(f) == 0 ? NF_OK : NF_EIO;
}

int nf_profile_load(NfProfile* p, const char* path) {
  FILE* f = fopen(path, "r");
  if (!f) return NF_EIO;
  char line[512];
  int version = 0;
  if (!fgets(line, sizeof line, f) || sscanf(line, "nfprofile %d", &version) != 1 || version != 1) {
    fclose(f);
    return NF_EIO;
  }
  NfProfile q;
  int ok = 1;
  while (fgets(line, sizeof line, f)) {
    int a, b, c, d;
    double x, y;
    nf_model_desc& m = q.model;
    if (sscanf(line, "model %d %d %d %d %d %d %d", &m.hidden, &m.n_q_heads, &m.n_kv_heads, &m.head_dim, &m.ffn_inner,
               &m.n_experts, &m.top_k) == 7) {
      continue;
    } else if (sscanf(line, "granule %d max_tokens %d measured %d", &a, &b, &c) == 3) {
      q.granule = a;
      q.max_tokens = b;
      q.measured = c != 0;
    } else if (sscanf(line, "dense %d %d %lf %d", &a, &b, &x, &d) == 4) {
      if (a < 0 || a >= NF_DENSE_OPS || q.granule <= 0 || b != (int)(q.dense_us[a].size() + 1) * q.granule) {
        ok = 0;
        break;
      }
      q.dense_us[a].push_back(x);
      q.dense_tile[a].push_back(d);
    } else if (sscanf(line, "tile_us %d %d %d %lf", &a, &b, &c, &x) == 4) {
      if (a < 1 || a > NF_MAX_TILE || b < 0 || b >= NF_DENSE_OPS ||
          c != (int)(q.tile_us[a][b].size() + 1) * q.granule) {
        ok = 0;
        break;
      }
      q.tile_us[a][b].push_back(x);
    } else if (!strncmp(line, "misc ", 5)) {
      if (sscanf(line, "misc %lf %lf %lf %lf %lf %lf", &q.misc_kqv[0], &q.misc_kqv[1], &q.misc_rest[0],
                 &q.misc_rest[1], &q.misc_attn[0], &q.misc_attn[1]) != 6) {
        ok = 0;
        break;
      }
    } else if (sscanf(line, "attn %lf %lf", &x, &y) == 2) {
      q.attn_fixed_us = x;
      q.attn_us_per_mb = y;
    } else if (!strncmp(line, "rp ", 3)) {
      NfRpRow r{};
      const int nf = sscanf(line, "rp %d %lf %lf %lf %d %lf", &r.attn_wgs, &r.p_gemm, &r.p_attn, &r.p_attn_solo,
                            &r.gemm_tile, &r.p_gemm_solo);
      if (nf != 4 && nf != 6) {
        ok = 0;
        break;
      }
      if (nf == 4) {
        r.gemm_tile = 0;
        r.p_gemm_solo = 1.0;
      }
      q.rp.push_back(r);
    } else if (line[0] != '#' && line[0] != '\n') {
      ok = 0;
      break;
    }
  }
  fclose(f);
  if (!ok || q.granule <= 0) return NF_EIO;
  for (int o = 0; o < NF_DENSE_OPS; ++o)
    if (q.dense_us[o].empty()) return NF_EIO;
  q.model.page_size = 16;
  *p = q;
  return NF_OK;
}

// ------------------------------------------------------------------ simulation ---

namespace {

struct SimOp {
  int lane;  // 0 GEMM, 1 attention
  double work;  // stand-alone microseconds
  std::vector<int> deps;
};

}  // namespace

static double simulate_impl(const NfProfile& prof, const NfSearchInput& in, const std::vector<int>& bounds, int overlap,
                            const NfRpRow* row, const std::vector<const NfRpRow*>* rows, const std::vector<int>* order,
                            int n_layers) {
  const int n = (int)bounds.size() - 1;
  const int L = std::max(1, n_layers);
  std::vector<double> kqv(n), att(n), rest(n);
  if (rows && !rows->empty()) row = (*rows)[0];  // the GEMM implementation is common to all rows
  // With a table row, every GEMM runs in the row's implementation: its own interference-free
  // time is the work, and its overlapped speed is relative to that implementation alone.
  const bool use_row_tile = overlap && row && row->gemm_tile > 0;
  auto dense = [&](int op, int m) {
    return use_row_tile ? nf_profile_tile_us(prof, row->gemm_tile, row->p_gemm_solo, op, m)
                        : nf_profile_dense_us(prof, op, m);
  };
  for (int i = 0; i < n; ++i) {
    const int m = bounds[i + 1] - bounds[i];
    kqv[i] = dense(NF_DENSE_KQV, m) + prof.misc_kqv[0] + prof.misc_kqv[1] * m;
    rest[i] = dense(NF_DENSE_O, m) + dense(NF_DENSE_UG, m) + dense(NF_DENSE_D, m) + prof.misc_rest[0] +
              prof.misc_rest[1] * m;
    const double mb = in.attn_mb_prefix[bounds[i + 1]] - in.attn_mb_prefix[bounds[i]];
    att[i] = prof.attn_fixed_us + prof.attn_us_per_mb * mb + prof.misc_attn[0] + prof.misc_attn[1] * m;
  }
  if (!overlap) {
    double t = 0;
    for (int i = 0; i < n; ++i) t += kqv[i] + att[i] + rest[i];
    return t * L;
  }
  // launch order of the nano-batches (index order unless given)
  std::vector<int> ord(n);
  for (int k = 0; k < n; ++k) ord[k] = (order && (int)order->size() == n) ? (*order)[k] : k;
  std::vector<int> pos(n, -1);
  for (int k = 0; k < n; ++k) {
    if (ord[k] < 0 || ord[k] >= n || pos[ord[k]] >= 0) return -1.0;
    pos[ord[k]] = k;
  }
  // ops of layer l: KQV_i = 3nl + i, ATTN_i = 3nl + n + i, REST_i (O, Up/Gate, Down) = 3nl + 2n + i.
  // Consecutive layers are pipelined as the executor does it: the KQV nano-operation of a range
  // in layer l + 1 is launched right behind the O/Up/Gate/Down of that range in layer l.
  std::vector<SimOp> ops((size_t)3 * n * L);
  std::vector<int> q[2];
  for (int l = 0; l < L; ++l) {
    const int base = 3 * n * l;
    for (int i = 0; i < n; ++i) {
      ops[base + i] = SimOp{0, kqv[i], {}};
      ops[base + n + i] = SimOp{1, att[i], {}};
      ops[base + 2 * n + i] = SimOp{0, rest[i], {base + n + i}};
      // attention needs the K/V of its own tokens and of the earlier tokens of a prefill
      // request it starts inside of
      const int lo = in.req_start_of_tok.empty() ? bounds[i] : in.req_start_of_tok[bounds[i]];
      for (int j = 0; j <= i; ++j)
        if (bounds[j + 1] > lo) {
          if (pos[j] > pos[i]) return -1.0;  // its KQV would be launched after this attention
          ops[base + n + i].deps.push_back(base + j);
        }
    }
    if (l == 0)
      for (int k = 0; k < n; ++k) q[0].push_back(ord[k]);
    for (int k = 0; k < n; ++k) {
      q[0].push_back(base + 2 * n + ord[k]);
      if (l + 1 < L) q[0].push_back(base + 3 * n + ord[k]);
    }
    for (int k = 0; k < n; ++k) q[1].push_back(base + n + ord[k]);
  }
  std::vector<char> done(ops.size(), 0);
  size_t head[2] = {0, 0};
  double rem[2] = {0, 0};
  bool running[2] = {false, false};
  double t = 0;
  for (;;) {
    for (int l = 0; l < 2; ++l) {
      if (running[l] || head[l] >= q[l].size()) continue;
      const SimOp& o = ops[q[l][head[l]]];
      bool ready = true;
      for (int d : o.deps) ready = ready && done[d];
      if (ready) {
        running[l] = true;
        rem[l] = o.work;
      }
    }
    if (!running[0] && !running[1]) break;  // all done (a valid structure cannot deadlock)
    // the row in force: that of the attention nano-operation at the head of its lane
    const NfRpRow* r = row;
    if (rows && !rows->empty() && head[1] < q[1].size()) r = (*rows)[(size_t)((q[1][head[1]] % (3 * n)) - n)];
    double sp[2] = {1.0, 1.0};
    if (r) {
      // GEMM work is in units of the row's implementation when its table is used
      const double g_solo = use_row_tile ? 1.0 : r->p_gemm_solo;
      if (running[0] && running[1]) {
        sp[0] = use_row_tile ? r->p_gemm / std::max(r->p_gemm_solo, 1e-6) : r->p_gemm;
        sp[1] = r->p_attn;
      } else if (running[1]) {
        sp[1] = r->p_attn_solo;
      } else {
        sp[0] = g_solo;
      }
    }
    double dt = 1e300;
    for (int l = 0; l < 2; ++l)
      if (running[l]) dt = std::min(dt, rem[l] / std::max(sp[l], 1e-6));
    t += dt;
    for (int l = 0; l < 2; ++l) {
      if (!running[l]) continue;
      rem[l] -= dt * std::max(sp[l], 1e-6);
      if (rem[l] <= 1e-9) {
        running[l] = false;
        done[q[l][head[l]]] = 1;
        ++head[l];
      }
    }
  }
  return t;
}

double nf_simulate(const NfProfile& prof, const NfSearchInput& in, const std::vector<int>& bounds, int overlap,
                   const NfRpRow* row, int n_layers) {
  return simulate_impl(prof, in, bounds, overlap, row, nullptr, nullptr, n_layers);
}

double nf_simulate_ops(const NfProfile& prof, const NfSearchInput& in, const std::vector<int>& bounds,
                       const std::vector<const NfRpRow*>& rows, const std::vector<int>& order, int n_layers) {
  if (!rows.empty()) {
    if (rows.size() + 1 != bounds.size()) return -1.0;
    for (const NfRpRow* r : rows)
      if (!r || r->gemm_tile != rows[0]->gemm_tile) return -1.0;
  }
  return simulate_impl(prof, in, bounds, 1, nullptr, &rows, &order, n_layers);
}

// Time per layer of a long run of consecutive layers: the increment between one layer and
// in.layers layers (the ramp-up of the first layer and the drain of the last drop out).
double nf_simulate_per_layer(const NfProfile& prof, const NfSearchInput& in, const std::vector<int>& bounds,
                             int overlap, const NfRpRow* row) {
  if (in.layers <= 1) return nf_simulate(prof, in, bounds, overlap, row, 1);
  const double t1 = nf_simulate(prof, in, bounds, overlap, row, 1);
  const double tl = nf_simulate(prof, in, bounds, overlap, row, in.layers);
  return (tl - t1) / (in.layers - 1);
}

static double simulate_ops_per_layer(const NfProfile& prof, const NfSearchInput& in, const std::vector<int>& bounds,
                                     const std::vector<const NfRpRow*>& rows, const std::vector<int>& order) {
  const double t1 = nf_simulate_ops(prof, in, bounds, rows, order, 1);
  if (t1 < 0 || in.layers <= 1) return t1;
  const double tl = nf_simulate_ops(prof, in, bounds, rows, order, in.layers);
  return (tl - t1) / (in.layers - 1);
}

// ---------------------------------------------------------------------- search ---

namespace {

void enumerate(int n_left, int pos, int n_tokens, int granule, std::vector<int>& cur,
               std::vector<std::vector<int>>& out) {
  if (n_left == 1) {
    cur.push_back(n_tokens);
    out.push_back(cur);
    cur.pop_back();
    return;
  }
  for (int b = pos + granule; b < n_tokens; b += granule) {
    cur.push_back(b);
    enumerate(n_left - 1, b, n_tokens, granule, cur, out);
    cur.pop_back();
  }
}

}  // namespace

int nf_search(const NfProfile& prof, const NfSearchInput& in, NfPipeline* out) {
  if (in.n_tokens < 0 || in.granule <= 0 || (int)in.attn_mb_prefix.size() != in.n_tokens + 1) return NF_EINVAL;
  const std::vector<int> whole = {0, in.n_tokens};
  out->bounds = whole;
  out->overlap = 0;
  out->attn_wgs = 0;
  out->nano_attn_wgs.clear();
  out->order.clear();
  out->est_us_unsplit = in.n_tokens ? nf_simulate_per_layer(prof, in, whole, 0, nullptr) : 0.0;
  out->est_us = out->est_us_stage1 = out->est_us_unsplit;
  const int max_n = in.max_nano > 0 ? std::min(in.max_nano, NF_MAX_NANO) : NF_MAX_NANO;
  if (max_n < 2 || in.n_tokens < 2 * in.granule) return NF_OK;

  // Stage I: structures ranked without interference
  struct Cand {
    std::vector<int> bounds;
    double t1;
  };
  std::vector<Cand> cands;
  for (int n = 2; n <= max_n; ++n) {
    std::vector<std::vector<int>> all;
    std::vector<int> cur = {0};
    enumerate(n, 0, in.n_tokens, in.granule, cur, all);
    for (auto& b : all) cands.push_back(Cand{b, nf_simulate_per_layer(prof, in, b, 1, nullptr)});
  }
  if (cands.empty()) return NF_OK;
  // fewer nano-operations win ties: splitting costs batching efficiency (Sec. 4.1.2)
  std::stable_sort(cands.begin(), cands.end(), [](const Cand& a, const Cand& b) {
    if (fabs(a.t1 - b.t1) > 1e-9) return a.t1 < b.t1;
    return a.bounds.size() < b.bounds.size();
  });
  const size_t keep = std::min<size_t>(cands.size(), 64);

  // Stage II: resource share per structure, with interference.  The best structure is kept
  // per table row; the rows are then ranked by their estimates.  in.rank = 0 asks for the best
  // pipeline (unsplit if nothing beats it); in.rank = r > 0 for the r-th best row's pipeline
  // (r = 1: the best row) whatever its estimate, so that a caller can refine the choice with trial runs.
  const NfRpRow ideal{0, 1.0, 1.0, 1.0, 0, 1.0};
  struct RowBest {
    double t2 = 1e300;
    size_t cand = 0;
    NfRpRow row;
  };
  const size_t n_rows = prof.rp.empty() ? 1 : prof.rp.size();
  std::vector<RowBest> per_row(n_rows);
  for (size_t r = 0; r < n_rows; ++r) {
    per_row[r].row = prof.rp.empty() ? ideal : prof.rp[r];
    for (size_t c = 0; c < keep; ++c) {
      const double t2 = nf_simulate_per_layer(prof, in, cands[c].bounds, 1, &per_row[r].row);
      if (t2 < per_row[r].t2 - 1e-9) {
        per_row[r].t2 = t2;
        per_row[r].cand = c;
      }
    }
  }
  std::stable_sort(per_row.begin(), per_row.end(), [](const RowBest& a, const RowBest& b) { return a.t2 < b.t2; });
  // rank 0: the best row's pipeline if its estimate beats unsplit; rank r > 0: the r-th best
  // row's pipeline (r = 1 is the best row) whatever its estimate
  const size_t rank = (size_t)std::max(0, in.rank);
  const size_t pick = rank > 0 ? rank - 1 : 0;
  if (pick < per_row.size() && (rank > 0 || per_row[0].t2 < out->est_us_unsplit - 1e-9)) {
    const RowBest& b = per_row[pick];
    out->bounds = cands[b.cand].bounds;
    out->overlap = 1;
    out->attn_wgs = b.row.attn_wgs;
    out->gemm_tile = b.row.gemm_tile;
    out->est_us = b.t2;
    out->est_us_stage1 = cands[b.cand].t1;
    // Stage II, second pass (Sec. 4.1.2 - 4.1.3: R is chosen per nano-operation, and the order of the
    // nano-batches belongs to the pipeline): starting from the uniform share, every attention
    // nano-operation in turn tries the other rows measured with the same GEMM implementation, and
    // the launch order tries every permutation the dependencies allow; changes that shorten the
    // estimate are kept until none does.  A few hundred simulations at most.
    if (!prof.rp.empty() && in.refine) {
      const int n = (int)out->bounds.size() - 1;
      std::vector<const NfRpRow*> same_tile;
      const NfRpRow* start = nullptr;
      for (const NfRpRow& r : prof.rp)
        if (r.gemm_tile == b.row.gemm_tile) {
          same_tile.push_back(&r);
          if (r.attn_wgs == b.row.attn_wgs && fabs(r.p_gemm - b.row.p_gemm) < 1e-12) start = &r;
        }
      if (start && n >= 2 && n <= NF_MAX_NANO) {
        std::vector<const NfRpRow*> rows((size_t)n, start);
        std::vector<int> order(n);
        for (int i = 0; i < n; ++i) order[i] = i;
        double best = simulate_ops_per_layer(prof, in, out->bounds, rows, order);
        bool improved = best >= 0;
        for (int pass = 0; pass < 4 && improved; ++pass) {
          improved = false;
          for (int i = 0; i < n; ++i)
            for (const NfRpRow* r : same_tile) {
              if (r == rows[i]) continue;
              const NfRpRow* keep = rows[i];
              rows[i] = r;
              const double t = simulate_ops_per_layer(prof, in, out->bounds, rows, order);
              if (t >= 0 && t < best - 1e-9) {
                best = t;
                improved = true;
              } else {
                rows[i] = keep;
              }
            }
          std::vector<int> perm = order, best_perm = order;
          std::sort(perm.begin(), perm.end());
          do {
            const double t = simulate_ops_per_layer(prof, in, out->bounds, rows, perm);
            if (t >= 0 && t < best - 1e-9) {
              best = t;
              best_perm = perm;
              improved = true;
            }
          } while (std::next_permutation(perm.begin(), perm.end()));
          order = best_perm;
        }
        if (best >= 0 && best < out->est_us - 1e-9) {
          out->est_us = best;
          out->nano_attn_wgs.clear();
          for (const NfRpRow* r : rows) out->nano_attn_wgs.push_back(r->attn_wgs);
          out->order = order;
        }
      }
    }
  }
  return NF_OK;
}
