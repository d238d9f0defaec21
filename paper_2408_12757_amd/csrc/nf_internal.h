// Host-side internals of the library: context, plan, and the helpers shared by
// the planner and the executor.  Nothing here crosses the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <utility>
#include <string>
#include <vector>

#include "../../include/nf.h"
#include "nf_kernels.h"

enum NfOpKind { NF_OP_KQV = 0, NF_OP_ATTN = 1, NF_OP_O = 2, NF_OP_UG = 3, NF_OP_D = 4, NF_OP_KINDS = 5 };
enum NfLane { NF_LANE_GEMM = 0, NF_LANE_ATTN = 1, NF_LANES = 2 };

// One nano-operation (paper Sec. 3.7): a parent operation restricted to the token
// range [tok_begin, tok_end) of the dense batch.
struct NfNanoOp {
  int kind;
  int nano;  // index of the nano-batch the range belongs to
  int tok_begin, tok_end;
  int lane;
  std::vector<int> deps;  // indices of earlier nano-ops this one waits for (other lane only)
  bool record = false;    // some later nano-op on another lane waits for this one
  int gemm_tile = 0;      // GEMM implementation chosen by the profile (0 = default)
  int attn_wgs = 0;       // attention nano-ops: persistent workgroups (its resource share; 0 = automatic, -1 = one per unit)
};

struct NfProfile;  // kernel timing tables (planner input)

struct NfTraceSlot {
  nf_trace_rec rec;
  hipEvent_t start, stop;
};

struct nf_ctx {
  int trace_level = 0;
  std::vector<NfTraceSlot> trace;       // pending records
  std::vector<hipEvent_t> event_pool;   // timing events ready for reuse
  int device = 0;
  int num_cus = 0;
  int last_hip = 0;
  // lane streams keyed by (lane, first CU bit, CU count); count 0 = unmasked stream
  std::map<long, hipStream_t> streams;
  NfProfile* profile = nullptr;
  // simultaneous KV offload (Sec. 4.2.2): device-writable host rows, stride between layers
  void* offload_host = nullptr;
  size_t offload_layer_stride = 0;
  hipStream_t offload_stream = nullptr;
  std::vector<hipEvent_t> offload_events;  // reused from call to call
  // plan = NULL calls of nf_layer_forward: the unsplit plan of the latest such batch (reused
  // while the batch stays the same) and earlier ones whose kernels may still be reading their
  // work lists, each with an event recorded behind its last use
  nf_plan* null_plan = nullptr;
  std::vector<std::pair<nf_plan*, hipEvent_t>> retired_plans;
  // this device's copy of the static attention-partials array (nf_op_attention_static)
  float* static_parts = nullptr;
  size_t static_parts_bytes = 0;
};

struct nf_plan {
  nf_model_desc model;
  int n_tokens = 0, n_reqs = 0, n_prefill_reqs = 0;
  uint64_t batch_sig = 0;
  std::vector<int> bounds;  // nano-batch token boundaries, size n_nano + 1 (the attention operation's when `parts` is set)
  std::vector<int> parts[NF_OP_KINDS];  // a partition per operation (Sec. 4.1.2); all empty = `bounds` for every operation
  std::vector<NfNanoOp> ops;  // launch order
  int overlap = 0;
  int lane_cus[NF_LANES] = {0, 0};        // CU count per lane (0 = whole chip, no mask)
  int lane_cu_first[NF_LANES] = {0, 0};   // first CU bit of the lane's mask
  int attn_wgs = 0;                       // persistent attention workgroups (0 = one per CU, -1 = one per work unit)
  std::vector<int> nano_attn_wgs;         // the same per nano-batch (what the launches use; attn_wgs is the default)
  std::vector<int> nano_order;            // launch order of the nano-batches (empty = index order)
  hipStream_t lane_stream[NF_LANES] = {nullptr, nullptr};
  std::vector<hipEvent_t> events;  // one per nano-op that records
  std::vector<hipEvent_t> events_alt;  // second set: consecutive layers of a multi-layer run alternate
  hipEvent_t ev_fork = nullptr, ev_join[NF_LANES] = {nullptr, nullptr};
  // device work lists
  void* dev_blob = nullptr;
  size_t dev_blob_bytes = 0;
  int device = 0;
  int32_t* d_tok_req = nullptr;
  NfAttnItem* d_items = nullptr;
  NfAttnGroup* d_groups = nullptr;
  std::vector<int> item_off, item_cnt, group_off, group_cnt;  // per nano-batch
  std::vector<long long> item_pages;                          // per nano-batch: KV pages its items read (per kv head)
  int total_parts = 0;
  double est_time_us = 0.0;  // planner's estimate of the pipeline length
  std::string origin;        // "manual" | "search"
};

#define NF_HIP(ctx, call)                         \
  do {                                            \
    hipError_t e__ = (call);                      \
    if (e__ != hipSuccess) {                      \
      if (ctx) (ctx)->last_hip = (int)e__;        \
      return NF_EHIP;                             \
    }                                             \
  } while (0)

int nf_validate_model(const nf_model_desc* m);
int nf_validate_batch(const nf_model_desc* m, const nf_batch* b, int64_t num_pages);
uint64_t nf_batch_signature(const nf_batch* b);
int nf_get_lane_stream(nf_ctx* ctx, int lane, int first_cu, int n_cus, hipStream_t* out);
void nf_profile_free(nf_ctx* ctx);
void nf_set_search_layers(int n);
void nf_set_search_rank(int r);
void nf_set_search_refine(int v);
void nf_set_search_max_parts(int v);
int nf_search_layers();
extern "C" int nf_nano_ops_dependent(int parent_kind, int child_kind, int b0, int e0, int b1, int e1);
extern "C" size_t nf_plan_workspace_bytes(const nf_plan* plan);

// Builds the device work lists, dependencies and events of a plan whose bounds, ops
// order, lanes and CU shares are already filled in.
int nf_plan_finalize(nf_ctx* ctx, nf_plan* p, const nf_batch* batch);
// Default launch order for given nano-batch bounds (used by nf_plan_manual and as the
// search's starting point).
// order (optional, n_nano entries): order[k] = index of the nano-batch launched k-th.
void nf_plan_default_order(nf_plan* p, int overlap, const int* order = nullptr);

size_t nf_align256(size_t v);
