// Host-callable launchers of the HIP kernels and the work-list records shared
// between the planner (host) and the attention kernels (device).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Keys per attention work item (a multiple of 1024: the kernel keeps the ids of 64 pages per
// register).  Part of the numerics contract: a request's keys are always cut at multiples of
// this length, whatever the batch split or CU share.
constexpr int NF_ATTN_CHUNK = 2048;

// One attention work item: the rows of up to 16/G consecutive tokens of one
// request (G = q heads per kv head) against keys [key_begin, key_end) of that
// request.  Token tok0 + j sits at position pos0 + j and may read keys
// 0 .. pos0 + j.  key_begin is a multiple of the page size.
struct NfAttnItem {
  int32_t req;
  int32_t tok0;
  int32_t n_tok;
  int32_t pos0;
  int32_t key_begin;
  int32_t key_end;
  int32_t part;   // slot of the partial result in the workspace; -1: the item covers all keys of
                  // its rows and the kernel writes the final attention output itself
  int32_t pad;
};

// One group of query rows whose partial results (part0 .. part0 + n_parts)
// are merged into the final attention output.
struct NfAttnGroup {
  int32_t tok0;
  int32_t n_tok;
  int32_t part0;
  int32_t n_parts;
};

struct NfAttnShape {
  int32_t n_q_heads, n_kv_heads, head_dim, n_qkv;  // n_qkv = row stride of the qkv buffer
};

static inline size_t nf_attn_part_floats(int head_dim) { return (size_t)16 * head_dim + 32; }

hipError_t nf_launch_rmsnorm(const void* x, const void* g, void* out, int n_tokens, int hidden, float eps,
                             hipStream_t s);
hipError_t nf_launch_rope_append(void* qkv, void* pages, const int32_t* tok_req, const int32_t* q_indptr,
                                 const int32_t* ctx_len, const int32_t* page_indptr, const int32_t* page_ids,
                                 int tok_begin, int tok_end, int n_q_heads, int n_kv_heads, int head_dim,
                                 float rope_theta, int write_k_back, hipStream_t s);
// Copies the (rotated) K and V parts of qkv rows [tok_begin, tok_end) to the same rows of a
// device-writable host buffer of 2 * n_kv_heads * head_dim elements per row.
hipError_t nf_launch_move_pages(void* pool, size_t page_bytes, long num_pages, const int32_t* page_ids, int n,
                                void* staging, int scatter, hipStream_t s);
hipError_t nf_launch_kv_offload(const void* qkv, void* host_rows, int tok_begin, int tok_end, int n_q_heads,
                                int n_kv_heads, int head_dim, hipStream_t s);
// Number of K segments of a dense operation: 1, or 2 for the long-K, narrow-N operations
// (the FFN down projection): K >= 8192, K >= 2 N, N < 8192 (wider outputs give a 1024-row
// nano-batch a tile for every CU anyway), K % 128 == 0, N % 128 == 0, no SwiGLU epilogue.  A two-segment operation computes bf16((sum over the first half of K) + (sum
// over the second half) [+ residual]), each half accumulated from zero in ascending K
// order.  The count depends on the operation's shape alone - never on M, the tile or the
// launch form - so a row's bits do not depend on the nano-batch it is computed in.
int nf_gemm_k_segments(int N, int K, int epilogue);
// Scratch that lets a two-segment operation put its segments on different workgroups:
// 2 x [rows, N] floats, the second block seg_stride floats after the first.  partial may be
// null (then each workgroup sums both segments itself).
struct NfGemmSplit {
  float* partial;
  long long seg_stride;
};
// tile: 0 = automatic, 1..19 = one implementation (see gemm.hip, gemm_dl.hip); all give identical bits
hipError_t nf_launch_gemm(const void* x, const void* w, void* out, const void* residual, int M, int N, int K,
                          int epilogue, int tile, hipStream_t s, NfGemmSplit split = NfGemmSplit{nullptr, 0});
// 0 = automatic, 1 = two-segment operations always as one workgroup per tile, 2 = always as
// two (when scratch is available); a tuning and test switch, the bits are the same
void nf_set_gemm_ksplit(int v);
hipError_t nf_launch_gemm_dl_two_sums(const void* x, const void* w, void* out, const void* residual, int M, int N,
                                      int K, int epilogue, hipStream_t s);
hipError_t nf_launch_gemm_dl_halves(const void* x, const void* w, void* out, const void* residual, int M, int N,
                                    int K, float* partial, long long seg_stride, int variant, hipStream_t s);
// max_workgroups: > 0 = that many persistent workgroups, 0 = automatic, < 0 = one workgroup
// per work unit.  item_pages: KV pages the items read per kv head (the automatic grid depends
// on it: a long, HBM-bound launch does better with fewer workgroups than CUs); 0 = unknown.
// n_cus: compute units of the device the stream belongs to (0 = ask the current device).
hipError_t nf_launch_attention(const void* qkv, const void* pages, const int32_t* page_indptr,
                               const int32_t* page_ids, const NfAttnItem* items, int n_items,
                               const NfAttnShape& shp, float* parts, void* attn_out, int max_workgroups,
                               hipStream_t s, long long item_pages = 0, int n_cus = 0);
// Size of the static device array that holds attention partials for nf_op_attention_static,
// and the device address of that array on `device` (which must be the current device on the
// first call for it; the address is looked up once per device and kept).
constexpr size_t NF_ATTN_STATIC_BYTES = (size_t)64 << 20;
hipError_t nf_attention_static_scratch(int device, float** ptr, size_t* bytes);
hipError_t nf_launch_attention_merge(const float* parts, const NfAttnGroup* groups, int n_groups,
                                     const NfAttnShape& shp, void* attn_out, hipStream_t s);
// Fills a bf16 buffer with pseudo-random, roughly normal values (timing buffers only).
hipError_t nf_launch_fill_random(void* p, size_t n_elems, uint32_t seed, float stddev, hipStream_t s);
void nf_set_attention_variant(int v);
void nf_set_gemm_tile(int v);
void nf_set_grouped_gemm_tile(int v);
// split: scratch for a two-segment operation (nf_gemm_k_segments); with it such an operation
// leaves the fp32 sums of its two K halves in the scratch and does NOT write `out`: the
// consumer adds the halves (nf_launch_moe_combine with the same scratch).
hipError_t nf_launch_grouped_gemm(const void* x, const void* w, void* out, int rows, int N, int K, int epilogue,
                                  const int32_t* expert_offset, const int32_t* row_index, int n_experts,
                                  long long w_stride, hipStream_t s, NfGemmSplit split = NfGemmSplit{nullptr, 0});
hipError_t nf_launch_gemm_dl_grouped_halves(const void* x, const void* w, int rows, int N, int K, float* partial,
                                            long long seg_stride, const int32_t* expert_offset,
                                            const int32_t* row_index, int n_experts, long long w_stride, int variant,
                                            hipStream_t s);
hipError_t nf_launch_gemm_dl_grouped(const void* x, const void* w, void* out, int rows, int N, int K, int epilogue,
                                     const int32_t* expert_offset, const int32_t* row_index, int n_experts,
                                     long long w_stride, int variant, hipStream_t s);
// Embedding / row gather and greedy sampling (token_path.hip)
hipError_t nf_launch_gather_rows(const int32_t* token_ids, const int32_t* from_slot, const int32_t* slot_tokens,
                                 const void* table, int n_rows_table, void* out, int n_rows, int width,
                                 hipStream_t s);
hipError_t nf_launch_argmax(const void* logits, int n_rows, int vocab, const int32_t* out_index, int32_t* out,
                            hipStream_t s);
// Mixture-of-experts helpers (moe.hip)
hipError_t nf_launch_moe_router(const void* h, const void* w_router, int32_t* expert_ids, float* expert_w,
                                int tok_begin, int tok_end, int hidden, int n_experts, int top_k, hipStream_t s);
hipError_t nf_launch_moe_scatter(const int32_t* expert_ids, int tok_begin, int tok_end, int n_experts, int top_k,
                                 int32_t* expert_offset, int32_t* row_token, int32_t* slot_of, hipStream_t s);
// expert_partial (optional): the experts' outputs as the fp32 sums of two K halves, seg_stride
// floats apart (see nf_launch_grouped_gemm); then expert_out is not read and a row's output is
// bf16(half 0 + half 1).
hipError_t nf_launch_moe_combine(const void* y, const void* expert_out, const int32_t* slot_of, const float* expert_w,
                                 void* z, int tok_begin, int tok_end, int hidden, int top_k, hipStream_t s,
                                 const float* expert_partial = nullptr, long long seg_stride = 0);
void nf_set_offload_dma(int v);
hipError_t nf_launch_gemm_dl(const void* x, const void* w, void* out, const void* residual, int M, int N, int K,
                             int epilogue, int variant, hipStream_t s);
