// Auto-search (paper Sec. 4.1): profile tables and the two-stage pipeline search.
// Pure host code; the GPU measurements that fill the tables live in profile.cpp.
#pragma once
#include <stdint.h>

#include <array>
#include <string>
#include <vector>

#include "../../include/nf.h"

constexpr int NF_MAX_TILE = 25;
enum { NF_DENSE_KQV = 0, NF_DENSE_O = 1, NF_DENSE_UG = 2, NF_DENSE_D = 3, NF_DENSE_OPS = 4 };

// One row of the resource-mapping table (Sec. 4.1.1, Table 3) for the memory-bound kernel:
// when decode attention runs with `attn_wgs` persistent workgroups beside a GEMM, the GEMM
// keeps p_gemm of its stand-alone performance (this is R of the GEMM by definition, so the
// attention kernel's share is R = 1 - p_gemm) and attention reaches p_attn of its best
// stand-alone performance.  p_attn_solo is its performance with that workgroup count when
// nothing runs beside it.
struct NfRpRow {
  int attn_wgs;
  double p_gemm, p_attn, p_attn_solo;
  // GEMM implementation (tile shape) of this pair, and the performance of that
  // implementation when it runs alone, relative to the best implementation (<= 1)
  int gemm_tile = 0;
  double p_gemm_solo = 1.0;
};

struct NfProfile {
  nf_model_desc model{};
  int granule = 128;
  int max_tokens = 0;
  bool measured = false;
  // interference-free execution time (microseconds) of dense op `o` at batch size
  // (i + 1) * granule, best over the GEMM tile shapes, and the tile that achieved it
  std::vector<double> dense_us[NF_DENSE_OPS];
  std::vector<int> dense_tile[NF_DENSE_OPS];
  // the same times per implementation (GEMM tile shape 1..NF_MAX_TILE); empty when unknown
  std::vector<double> tile_us[NF_MAX_TILE + 1][NF_DENSE_OPS];
  // the small row-wise kernels, as fixed + per-token microseconds: norm + rotary/append before
  // the KQV GEMM's consumers, norm before Up/Gate, merge after attention
  double misc_kqv[2] = {8.0, 0.02}, misc_rest[2] = {4.0, 0.005}, misc_attn[2] = {4.0, 0.02};
  // a dependency that crosses lanes (an event wait on another stream) lets the waiting kernel
  // start this much later than a kernel that follows its predecessor on one stream (microseconds)
  double sync_us = 0.0;
  // stand-alone attention: fixed cost + cost per byte of K/V read, at the best configuration
  double attn_fixed_us = 5.0;
  double attn_us_per_mb = 1.0 / 5.7;  // 5.7 TB/s
  std::vector<NfRpRow> rp;            // sorted by attn_wgs ascending; last row = "as many as there is work"
};

// Interpolated interference-free time of a dense op on m tokens (0 < m).
double nf_profile_dense_us(const NfProfile& p, int op, int m);
// Same for one implementation; falls back to best / p_solo when that table is missing.
double nf_profile_tile_us(const NfProfile& p, int tile, double p_solo, int op, int m);
// Analytic stand-in used when nothing was measured (no GPU, or nf_profile never called).
void nf_profile_analytic(NfProfile* p, const nf_model_desc* model, int max_tokens, int granule);
int nf_profile_save(const NfProfile& p, const char* path);
int nf_profile_load(NfProfile* p, const char* path);

// Input of the search: per-token-range attention work, in bytes of K/V read.
struct NfSearchInput {
  int n_tokens = 0;
  int granule = 128;
  int max_nano = 0;                  // 0 = search up to NF_MAX_NANO
  int layers = 1;                    // > 1: minimise the time per layer of that many consecutive layers
  int rank = 0;                      // 0: the best pipeline; r > 0: the r-th best table row's pipeline
  int refine = 1;                    // second pass of Stage II: share per attention nano-operation, launch order,
                                     // and the number of nano-operations per operation
  int max_parts = 0;                 // nano-operations per operation in that pass (0 = NF_MAX_PARTS)
  bool tie_ffn = false;              // Up/Gate and Down must share one partition (mixture-of-experts layers)
  std::vector<double> attn_mb_prefix;  // [n_tokens + 1] prefix sums of attention megabytes per token
  std::vector<int> req_start_of_tok;   // [n_tokens] first token of the request that owns token t
};

// The token partition of every operation (Sec. 4.1.2: the number and the sizes of the
// nano-operations are decided per operation): parts[k] holds the boundaries of the nano-operations
// of operation k, in the order KQV, attention, O, Up/Gate, Down.
constexpr int NF_PART_KINDS = 5;
constexpr int NF_MAX_PARTS = 8;
using NfParts = std::array<std::vector<int>, NF_PART_KINDS>;

struct NfPipeline {
  std::vector<int> bounds;   // nano-batch boundaries (of the attention operation when `parts` is set)
  // per-operation partitions; all empty = every operation is split at `bounds`.  With partitions
  // nano_attn_wgs has one entry per attention nano-operation and `order` is empty.
  NfParts parts;
  int overlap = 0;
  // Per nano-batch (Sec. 4.1.1 - 4.1.3: every nano-operation has its own resource share, and the
  // order of the nano-batches is part of the pipeline): the persistent workgroups of its attention
  // nano-operation, and the launch order (order[k] = index of the nano-batch launched k-th).
  // Empty = the uniform share `attn_wgs` / index order.
  std::vector<int> nano_attn_wgs;
  std::vector<int> order;
  int attn_wgs = 0;          // chosen row of the R -> P table (0 = unrestricted)
  int gemm_tile = 0;         // GEMM implementation of the chosen row (0 = per-op best)
  double est_us = 0.0;       // simulated makespan
  double est_us_stage1 = 0.0;  // makespan of the same structure without interference
  double est_us_unsplit = 0.0;
};

constexpr int NF_MAX_NANO = 4;

// Simulated makespan (microseconds) of a pipeline structure.  row = nullptr: no
// interference (Stage I); otherwise overlapped GEMM and attention progress at p_gemm and
// p_attn of their stand-alone speeds and attention alone at p_attn_solo (Stage II).
double nf_simulate(const NfProfile& prof, const NfSearchInput& in, const std::vector<int>& bounds, int overlap,
                   const NfRpRow* row, int n_layers = 1);
// The same with a table row per nano-batch (rows[i] holds while the attention nano-operation of
// nano-batch i runs; all rows must name the same GEMM implementation) and a launch order.  Returns
// a negative value for an order that launches an attention nano-operation before the KQV
// nano-operations it depends on.
double nf_simulate_ops(const NfProfile& prof, const NfSearchInput& in, const std::vector<int>& bounds,
                       const std::vector<const NfRpRow*>& rows, const std::vector<int>& order, int n_layers = 1);
// One nano-operation in launch order: operation kind (index into NfParts), its index within the
// operation's partition, its token range.
struct NfEmitOp {
  int kind, index, tok_begin, tok_end;
};
// Launch order of one layer's nano-operations when every operation has its own partition:
// the KQV nano-operations in range order, each attention nano-operation right behind the KQV
// nano-operation that completes its tokens; then O, Up/Gate and Down nano-operations, always the
// one with the smallest last token among those whose inputs have been launched (ties: O before
// Up/Gate before Down).  For equal partitions this is KQV0 ATTN0 KQV1 ATTN1 .. O0 UG0 D0 O1 UG1 D1 ..
// Returns false for partitions that are not increasing sequences from 0 to one common end.
bool nf_emission_order(const NfParts& parts, std::vector<NfEmitOp>* out);
// Simulated makespan with a partition per operation.  rows: one table row per attention
// nano-operation (all of one GEMM implementation), or empty for no interference.  overlap = 0:
// every nano-operation back to back.  Negative for invalid partitions.
double nf_simulate_parts(const NfProfile& prof, const NfSearchInput& in, const NfParts& parts, int overlap,
                         const std::vector<const NfRpRow*>& rows, int n_layers = 1);
// The objective of the search: the makespan of one layer, or (in.layers > 1) the time per layer
// of a run of consecutive layers pipelined across the layer boundaries.
double nf_simulate_per_layer(const NfProfile& prof, const NfSearchInput& in, const std::vector<int>& bounds,
                             int overlap, const NfRpRow* row);
// Two-stage search.  Returns NF_OK and fills `out`.
int nf_search(const NfProfile& prof, const NfSearchInput& in, NfPipeline* out);
