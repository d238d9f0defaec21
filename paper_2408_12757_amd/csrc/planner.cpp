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
  p->sync_us = 0.0;
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
  fprintf(f, "sync %.4f\n", p.sync_us);
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
    } else if (sscanf(line, "sync %lf", &x) == 1) {
      q.sync_us = x;
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
  std::vector<double> done_at(ops.size(), 0.0);
  size_t head[2] = {0, 0};
  double rem[2] = {0, 0};
  bool running[2] = {false, false};
  double t = 0;
  for (;;) {
    // a nano-operation starts once its dependencies (all on the other lane) are done and the
    // synchronisation latency behind the last of them has passed
    double wake = 1e300;
    for (int l = 0; l < 2; ++l) {
      if (running[l] || head[l] >= q[l].size()) continue;
      const SimOp& o = ops[q[l][head[l]]];
      bool ready = true;
      double at = 0.0;
      for (int d : o.deps) {
        ready = ready && done[d];
        at = std::max(at, done_at[d] + prof.sync_us);
      }
      if (ready && t + 1e-9 >= at) {
        running[l] = true;
        rem[l] = o.work;
      } else if (ready) {
        wake = std::min(wake, at);
      }
    }
    if (!running[0] && !running[1]) {
      if (wake < 1e299) {
        t = wake;
        continue;
      }
      break;  // all done (a valid structure cannot deadlock)
    }
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
    if (wake < 1e299) dt = std::min(dt, wake - t);  // the idle lane's nano-operation joins then
    t += dt;
    for (int l = 0; l < 2; ++l) {
      if (!running[l]) continue;
      rem[l] -= dt * std::max(sp[l], 1e-6);
      if (rem[l] <= 1e-9) {
        running[l] = false;
        done[q[l][head[l]]] = 1;
        done_at[q[l][head[l]]] = t;
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

bool nf_emission_order(const NfParts& parts, std::vector<NfEmitOp>* out) {
  out->clear();
  const int end = parts[0].empty() ? -1 : parts[0].back();
  for (const std::vector<int>& b : parts) {
    if (b.size() < 2 || b.front() != 0 || b.back() != end) return false;
    for (size_t i = 0; i + 1 < b.size(); ++i)
      if (b[i + 1] <= b[i]) return false;
  }
  auto op = [&](int kind, int j) { return NfEmitOp{kind, j, parts[kind][j], parts[kind][j + 1]}; };
  // KQV in range order; an attention nano-operation follows the KQV nano-operation that launches
  // the last of its tokens (its earlier tokens, and the earlier tokens of a request it starts
  // inside of, belong to KQV nano-operations launched before)
  size_t a = 0;
  for (size_t k = 0; k + 1 < parts[0].size(); ++k) {
    out->push_back(op(0, (int)k));
    for (; a + 1 < parts[1].size() && parts[1][a + 1] <= parts[0][k + 1]; ++a) out->push_back(op(1, (int)a));
  }
  // O, Up/Gate, Down: launched[k] = tokens [0, launched[k]) of operation k have been launched
  int launched[NF_PART_KINDS] = {end, end, 0, 0, 0};
  size_t next[NF_PART_KINDS] = {0, 0, 0, 0, 0};
  for (;;) {
    int pick = -1;
    for (int k = 2; k < NF_PART_KINDS; ++k) {
      if (next[k] + 1 >= parts[k].size()) continue;
      const int e = parts[k][next[k] + 1];
      if (launched[k - 1] < e) continue;  // an input row has not been launched yet
      if (pick < 0 || e < parts[pick][next[pick] + 1]) pick = k;
    }
    if (pick < 0) break;
    out->push_back(op(pick, (int)next[pick]));
    launched[pick] = parts[pick][next[pick] + 1];
    ++next[pick];
  }
  return true;
}

// The general form of simulate_impl: one partition per operation, launch order by
// nf_emission_order, O / Up-Gate / Down as nano-operations of their own.  For equal partitions
// it gives simulate_impl's result.
double nf_simulate_parts(const NfProfile& prof, const NfSearchInput& in, const NfParts& parts, int overlap,
                         const std::vector<const NfRpRow*>& rows, int n_layers) {
  std::vector<NfEmitOp> emit;
  if (!nf_emission_order(parts, &emit) || parts[0].back() != in.n_tokens) return -1.0;
  const int L = std::max(1, n_layers);
  const int n_attn = (int)parts[1].size() - 1;
  if (!rows.empty()) {
    if ((int)rows.size() != n_attn) return -1.0;
    for (const NfRpRow* r : rows)
      if (!r || r->gemm_tile != rows[0]->gemm_tile) return -1.0;
  }
  const NfRpRow* row0 = rows.empty() ? nullptr : rows[0];
  const bool use_row_tile = overlap && row0 && row0->gemm_tile > 0;
  auto dense = [&](int op, int m) {
    return use_row_tile ? nf_profile_tile_us(prof, row0->gemm_tile, row0->p_gemm_solo, op, m)
                        : nf_profile_dense_us(prof, op, m);
  };
  auto work_of = [&](const NfEmitOp& e) {
    const int m = e.tok_end - e.tok_begin;
    switch (e.kind) {
      case 0: return dense(NF_DENSE_KQV, m) + prof.misc_kqv[0] + prof.misc_kqv[1] * m;
      case 1:
        return prof.attn_fixed_us +
               prof.attn_us_per_mb * (in.attn_mb_prefix[(size_t)e.tok_end] - in.attn_mb_prefix[(size_t)e.tok_begin]) +
               prof.misc_attn[0] + prof.misc_attn[1] * m;
      case 2: return dense(NF_DENSE_O, m);
      case 3: return dense(NF_DENSE_UG, m) + prof.misc_rest[0] + prof.misc_rest[1] * m;
      default: return dense(NF_DENSE_D, m);
    }
  };
  const size_t per_layer = emit.size();
  if (!overlap) {
    double t = 0;
    for (const NfEmitOp& e : emit) t += work_of(e);
    return t * L;
  }
  // ops of layer l: index l * per_layer + position in `emit`
  struct Op {
    int lane;
    double work;
    int attn_index;  // attention nano-operations: index into rows
    std::vector<int> deps;
  };
  std::vector<Op> ops(per_layer * (size_t)L);
  std::vector<int> q[2];
  for (int l = 0; l < L; ++l) {
    const size_t base = per_layer * (size_t)l;
    for (size_t i = 0; i < per_layer; ++i) {
      const NfEmitOp& e = emit[i];
      Op& o = ops[base + i];
      o.lane = e.kind == 1 ? 1 : 0;
      o.work = work_of(e);
      o.attn_index = e.kind == 1 ? e.index : -1;
      // cross-lane dependencies (same-lane ones are met by the launch order): attention needs the
      // KQV nano-operations of its tokens and of the earlier tokens of a prefill request it starts
      // inside of; O needs the attention nano-operations of its tokens
      if (e.kind == 1 || e.kind == 2) {
        int lo = e.tok_begin;
        if (e.kind == 1 && !in.req_start_of_tok.empty()) lo = in.req_start_of_tok[(size_t)e.tok_begin];
        for (size_t j = 0; j < per_layer; ++j)
          if (emit[j].kind == e.kind - 1 && std::max(lo, emit[j].tok_begin) < std::min(e.tok_end, emit[j].tok_end))
            o.deps.push_back((int)(base + j));
      }
    }
    // lanes: KQV of the first layer up front; later layers' KQV nano-operations right behind the
    // Down nano-operation of the previous layer that completes their tokens
    size_t next_kqv = 0;
    std::vector<size_t> kqv_pos, attn_pos;
    for (size_t i = 0; i < per_layer; ++i)
      if (emit[i].kind == 0)
        kqv_pos.push_back(i);
      else if (emit[i].kind == 1)
        attn_pos.push_back(i);
    if (l == 0)
      for (size_t i : kqv_pos) q[0].push_back((int)i);
    for (size_t i = 0; i < per_layer; ++i) {
      if (emit[i].kind < 2) continue;
      q[0].push_back((int)(base + i));
      if (emit[i].kind == 4 && l + 1 < L)
        for (; next_kqv < kqv_pos.size() && emit[kqv_pos[next_kqv]].tok_end <= emit[i].tok_end; ++next_kqv)
          q[0].push_back((int)(base + per_layer + kqv_pos[next_kqv]));
    }
    for (size_t i : attn_pos) q[1].push_back((int)(base + i));
  }
  std::vector<char> done(ops.size(), 0);
  std::vector<double> done_at(ops.size(), 0.0);
  size_t head[2] = {0, 0};
  double rem[2] = {0, 0};
  bool running[2] = {false, false};
  double t = 0;
  for (;;) {
    double wake = 1e300;  // as in simulate_impl: the synchronisation latency behind a cross-lane dependency
    for (int l = 0; l < 2; ++l) {
      if (running[l] || head[l] >= q[l].size()) continue;
      const Op& o = ops[(size_t)q[l][head[l]]];
      bool ready = true;
      double at = 0.0;
      for (int d : o.deps) {
        ready = ready && done[(size_t)d];
        at = std::max(at, done_at[(size_t)d] + prof.sync_us);
      }
      if (ready && t + 1e-9 >= at) {
        running[l] = true;
        rem[l] = o.work;
      } else if (ready) {
        wake = std::min(wake, at);
      }
    }
    if (!running[0] && !running[1]) {
      if (wake < 1e299) {
        t = wake;
        continue;
      }
      break;
    }
    // the row in force: that of the attention nano-operation at the head of its lane
    const NfRpRow* r = nullptr;
    if (!rows.empty()) r = head[1] < q[1].size() ? rows[(size_t)ops[(size_t)q[1][head[1]]].attn_index] : rows.back();
    double sp[2] = {1.0, 1.0};
    if (r) {
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
    if (wake < 1e299) dt = std::min(dt, wake - t);
    t += dt;
    for (int l = 0; l < 2; ++l) {
      if (!running[l]) continue;
      rem[l] -= dt * std::max(sp[l], 1e-6);
      if (rem[l] <= 1e-9) {
        running[l] = false;
        done[(size_t)q[l][head[l]]] = 1;
        done_at[(size_t)q[l][head[l]]] = t;
        ++head[l];
      }
    }
  }
  for (int l = 0; l < 2; ++l)
    if (head[l] < q[l].size()) return -1.0;  // a nano-operation never became ready
  return t;
}

static double simulate_parts_per_layer(const NfProfile& prof, const NfSearchInput& in, const NfParts& parts,
                                       const std::vector<const NfRpRow*>& rows) {
  const double t1 = nf_simulate_parts(prof, in, parts, 1, rows, 1);
  if (t1 < 0 || in.layers <= 1) return t1;
  const double tl = nf_simulate_parts(prof, in, parts, 1, rows, in.layers);
  return tl < 0 ? tl : (tl - t1) / (in.layers - 1);
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

// Stage II, third pass (Sec. 4.1.2: the number of nano-operations is decided per operation, more
// of them where a bubble is): starting from the common boundaries, every operation's partition
// in turn tries one more boundary (any multiple of the granule) or one fewer, attention
// nano-operations that are split inherit their share and then try the other rows of the same
// GEMM implementation; the single change that shortens the estimate most is kept, until none
// shortens it by a thousandth.  Runs only from the index launch order.
static void refine_partitions(const NfProfile& prof, const NfSearchInput& in, const NfRpRow& picked, NfPipeline* out) {
  const int n = (int)out->bounds.size() - 1;
  for (size_t k = 0; k < out->order.size(); ++k)
    if (out->order[k] != (int)k) return;
  if (n < 2) return;
  const int max_parts = in.max_parts > 0 ? std::min(in.max_parts, NF_MAX_PARTS) : NF_MAX_PARTS;
  std::vector<const NfRpRow*> same_tile, rows;
  if (!prof.rp.empty()) {
    for (const NfRpRow& r : prof.rp)
      if (r.gemm_tile == picked.gemm_tile) same_tile.push_back(&r);
    for (int i = 0; i < n; ++i) {
      const int wgs = out->nano_attn_wgs.empty() ? picked.attn_wgs : out->nano_attn_wgs[(size_t)i];
      const NfRpRow* found = nullptr;
      for (const NfRpRow* r : same_tile)
        if (r->attn_wgs == wgs && (!found || fabs(r->p_gemm - picked.p_gemm) < fabs(found->p_gemm - picked.p_gemm)))
          found = r;
      if (!found) return;
      rows.push_back(found);
    }
  }
  NfParts parts;
  for (auto& b : parts) b = out->bounds;
  double best = simulate_parts_per_layer(prof, in, parts, rows);
  if (best < 0) return;
  bool changed = false;
  for (int pass = 0; pass < 24; ++pass) {
    NfParts best_parts;
    std::vector<const NfRpRow*> best_rows;
    double best_t = best * (1.0 - 1e-3);
    bool found = false;
    auto consider = [&](const NfParts& p, const std::vector<const NfRpRow*>& r) {
      const double t = simulate_parts_per_layer(prof, in, p, r);
      if (t >= 0 && t < best_t) {
        best_t = t;
        best_parts = p;
        best_rows = r;
        found = true;
      }
    };
    // one boundary more or fewer, in one operation or in a group of consecutive operations at once
    // (a bubble behind the first KQV needs KQV and attention split together to close)
    static const int kGroups[][NF_PART_KINDS] = {{1, 0, 0, 0, 0}, {0, 1, 0, 0, 0}, {0, 0, 1, 0, 0}, {0, 0, 0, 1, 0},
                                                 {0, 0, 0, 0, 1}, {1, 1, 0, 0, 0}, {0, 0, 0, 1, 1}, {0, 0, 1, 1, 1},
                                                 {1, 1, 1, 0, 0}, {1, 1, 1, 1, 1}};
    for (const auto& group : kGroups)
      for (int cut = in.granule; cut < in.n_tokens; cut += in.granule)
        for (int add = 0; add < 2; ++add) {
          NfParts p = parts;
          std::vector<const NfRpRow*> r = rows;
          bool any = false, ok = true;
          long split_attn = -1;  // index of the right half of an attention nano-operation split by this move
          for (int k = 0; k < NF_PART_KINDS; ++k) {
            if (!group[k]) continue;
            std::vector<int>& b = p[(size_t)k];
            const auto at = std::lower_bound(b.begin(), b.end(), cut);
            const size_t j = (size_t)(at - b.begin());  // b[j - 1] < cut <= b[j]
            if (add && *at != cut) {
              if ((int)b.size() - 1 >= max_parts) ok = false;
              b.insert(at, cut);
              if (k == 1 && !r.empty()) {
                r.insert(r.begin() + (long)j, r[j - 1]);
                split_attn = (long)j;
              }
              any = true;
            } else if (!add && *at == cut) {
              b.erase(at);
              if (k == 1 && !r.empty()) r.erase(r.begin() + (long)j);
              any = true;
            }
          }
          if (in.tie_ffn && p[3] != p[4]) ok = false;
          if (!any || !ok) continue;
          consider(p, r);
          // the halves of a split attention nano-operation may want different shares (one runs
          // beside GEMMs, the other alone): neither change pays on its own
          for (long half = split_attn - 1; split_attn > 0 && half <= split_attn; ++half)
            for (const NfRpRow* alt : same_tile) {
              if (alt == r[(size_t)half]) continue;
              std::vector<const NfRpRow*> r2 = r;
              r2[(size_t)half] = alt;
              consider(p, r2);
            }
        }
    // another share for one attention nano-operation
    for (size_t i = 0; i < rows.size(); ++i)
      for (const NfRpRow* alt : same_tile) {
        if (alt == rows[i]) continue;
        std::vector<const NfRpRow*> r = rows;
        r[i] = alt;
        consider(parts, r);
      }
    if (!found) break;
    parts = best_parts;
    rows = best_rows;
    best = best_t;
    changed = true;
  }
  if (!changed || best >= out->est_us - 1e-9) return;
  bool uniform = true;
  for (const auto& b : parts) uniform = uniform && b == parts[0];
  out->est_us = best;
  out->bounds = parts[1];
  out->order.clear();
  out->nano_attn_wgs.clear();
  for (const NfRpRow* r : rows) out->nano_attn_wgs.push_back(r->attn_wgs);
  if (!uniform) out->parts = parts;
}

int nf_search(const NfProfile& prof, const NfSearchInput& input, NfPipeline* out) {
  // The time per layer of a run of layers is the increment between one layer and `layers`
  // layers; the pipeline is in its steady state after two or three, so six price a longer run
  // just as well at a fraction of the simulations' cost.
  NfSearchInput in = input;
  in.layers = std::min(input.layers, 6);
  if (in.n_tokens < 0 || in.granule <= 0 || (int)in.attn_mb_prefix.size() != in.n_tokens + 1) return NF_EINVAL;
  const std::vector<int> whole = {0, in.n_tokens};
  out->bounds = whole;
  out->overlap = 0;
  out->attn_wgs = 0;
  out->nano_attn_wgs.clear();
  out->order.clear();
  for (auto& b : out->parts) b.clear();
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
  const size_t keep = std::min<size_t>(cands.size(), 24);

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
  // rank 0: the best row's pipeline, refined, if its estimate beats unsplit; rank r > 0: the r-th
  // best row's pipeline (r = 1 is the best row) whatever its estimate
  const size_t rank = (size_t)std::max(0, in.rank);
  const size_t pick = rank > 0 ? rank - 1 : 0;
  // the refinement passes have gained up to an eighth in the cases seen; a best row that is
  // further than that from unsplit is not worth their time (they run per batch in a serving loop)
  const bool hopeless = rank == 0 && !per_row.empty() && per_row[0].t2 > 1.15 * out->est_us_unsplit;
  // the pipeline of one row, refined; rank 0 refines the three best rows and keeps the best result
  // (the refinement is a local search: the best uniform row is not always its best start)
  auto build = [&](const RowBest& b, NfPipeline* out) {
    out->nano_attn_wgs.clear();
    out->order.clear();
    for (auto& pb : out->parts) pb.clear();
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
    if (in.refine >= 2) refine_partitions(prof, in, b.row, out);
  };
  if (pick < per_row.size() && !hopeless) {
    build(per_row[pick], out);
    for (size_t alt = 1; rank == 0 && in.refine && alt < 3 && alt < per_row.size(); ++alt) {
      NfPipeline other = *out;
      build(per_row[alt], &other);
      if (other.est_us < out->est_us - 1e-9) *out = other;
    }
    if (rank == 0 && out->est_us >= out->est_us_unsplit - 1e-9) {
      // nothing beats running unsplit
      out->bounds = whole;
      out->overlap = 0;
      out->attn_wgs = 0;
      out->gemm_tile = 0;
      out->nano_attn_wgs.clear();
      out->order.clear();
      for (auto& pb : out->parts) pb.clear();
      out->est_us = out->est_us_stage1 = out->est_us_unsplit;
    }
  }
  return NF_OK;
}
