/*
 * nf.h - C ABI of the nano-batched decoder-layer library for MI355X (gfx950).
 *
 * One call of nf_layer_forward() runs one LLaMA-style decoder-layer iteration
 * over a dense batch that mixes the chunk tokens of prefill requests with one
 * token of every decode request (paper Sec. 2.1 for the operation order,
 * Sec. 2.2 for the operation classes, Sec. 3.1 "Batch size" for the dense
 * batch).  The batch may be split into nano-batches whose compute-bound GEMM
 * nano-operations run concurrently with the memory-bound paged decode
 * attention of other nano-batches (Sec. 3.7, Sec. 4.1, Sec. 5).
 *
 * Where this interface departs from the plainest statement of the problem (weights, a
 * paged KV cache, per-request context lengths, the dense batch), on purpose:
 *   - KV page layout: the 16 x head_dim elements of a (page, K|V, kv head) block are stored in
 *     the order the matrix cores consume them (formulas at nf_kv_cache), not token-major.  A
 *     caller with a token-major cache repacks blocks once; appends go through the library.
 *   - Extra arguments: `granule` on nf_profile / nf_plan_nanobatches (the nano-batch size unit
 *     of Sec. 4.1.1, 128 for real models, smaller for toy batches) and `max_context` on
 *     nf_workspace_bytes (the attention partials depend on the longest request).
 *   - Device allocations after nf_ctx_create: a plan's work lists (a few KB per request,
 *     pooled per process and reused), and the scratch of nf_profile and nf_measure_peaks
 *     (freed before they return).  nf_layer_forward / nf_layers_forward / nf_op_* with a
 *     prepared plan allocate nothing.
 *
 * Conventions
 *   - All structs live in HOST memory.  Every pointer inside them, and every
 *     buffer argument, is a DEVICE pointer unless its comment says "host".
 *   - bf16 tensors are row-major with the contraction dimension contiguous.
 *     Accumulation, softmax and row statistics are fp32; indices are int32.
 *   - The caller owns every device buffer it passes (weights, KV pages, batch
 *     arrays, activations, workspace).  The library owns only what its opaque
 *     handles hold (streams, events, the small device-side work lists of a
 *     plan) and releases it in the matching *_destroy call (a plan's work
 *     lists go back to a small per-process pool of device buffers).
 *   - Every function returns NF_OK (0) or a negative nf_status; nothing throws
 *     or aborts across the ABI.  Arguments are validated on the host (using the
 *     host mirrors in nf_batch) before anything is launched.
 *   - Calls are asynchronous with respect to the GPU: they return after
 *     enqueueing.  Work is ordered after everything previously enqueued on the
 *     hipStream_t passed as `hip_stream`, and its results are visible once that
 *     stream drains.  A handle must not be used from two threads at once.
 */
#ifndef NF_H_
#define NF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum nf_status {
  NF_OK = 0,
  NF_EINVAL = -1,     /* null pointer, negative size, unsupported option          */
  NF_ESHAPE = -2,     /* model or batch shape the kernels do not support          */
  NF_EWORKSPACE = -3, /* workspace too small (see nf_workspace_bytes)             */
  NF_EPAGES = -4,     /* page table does not cover a request, or id out of range  */
  NF_EHIP = -5,       /* a HIP call failed; see nf_last_hip_error                 */
  NF_EPLAN = -6,      /* plan does not match the batch, or is malformed           */
  NF_ENOMEM = -7,     /* host allocation failed                                   */
  NF_EIO = -8,        /* profile cache file could not be read or written          */
  NF_ESCRATCH = -9    /* nf_op_attention_static: the plan needs more partial-result
                         space than the library's built-in array holds             */
} nf_status;

/* Model shape of one decoder layer (Sec. 3.1 "Model configuration"). */
typedef struct nf_model_desc {
  int32_t hidden;      /* D_model                                                  */
  int32_t n_q_heads;   /* Hq                                                       */
  int32_t n_kv_heads;  /* Hkv; R_GQA = Hq / Hkv                                    */
  int32_t head_dim;    /* dh: 64 or 128                                            */
  int32_t ffn_inner;   /* I_model                                                  */
  int32_t n_experts;   /* 0 or 1: dense FFN; >1: mixture of experts (Sec. 4.1.4)   */
  int32_t top_k;       /* experts per token (MoE only)                             */
  int32_t page_size;   /* tokens per KV page; must be 16                           */
  float rms_eps;
  float rope_theta;
} nf_model_desc;

/* bf16 weights of one layer. */
typedef struct nf_layer_weights {
  const void *g_attn_norm; /* [D]                                                  */
  const void *w_qkv;       /* [(Hq+2Hkv)*dh, D]  rows: Q heads, K heads, V heads    */
  const void *w_o;         /* [D, Hq*dh]                                           */
  const void *g_ffn_norm;  /* [D]                                                  */
  const void *w_gate_up;   /* [E][2I, D]  gate rows, then up rows                  */
  const void *w_down;      /* [E][D, I]                                            */
  const void *w_router;    /* [E, D], NULL for a dense layer                       */
} nf_layer_weights;

/*
 * Paged KV cache of this layer (Sec. 4.2.2: pages are scattered in device
 * memory).  One page holds page_size = 16 tokens and is bf16 [2][Hkv][16*dh]:
 * pages[p][0][h] is the K block and pages[p][1][h] the V block of kv head h.
 * Inside a block the 16 x dh elements are stored in the order the matrix cores
 * consume them, so that the attention kernel reads every block with wavefront
 * loads of long contiguous runs and no transpose, and a token's own elements
 * stay within few cache lines:
 *   K block: [dh/32][16 tokens][32]          element (t, d) at ((d/32)*16 + t)*32 + d%32
 *   V block: [4][dh/32][16][2][4]            element (t, d) at
 *            ((((t/4)*(dh/32) + d/32)*16 + d%16)*2 + (d/16)%2)*4 + t%4
 * nf_layer_forward WRITES the K/V of the batch's tokens into their slots.
 */
typedef struct nf_kv_cache {
  void *pages;
  int64_t num_pages;
} nf_kv_cache;

/*
 * Dense batch.  Token order: the prefill requests first (the tokens of one
 * request contiguous), then one token per decode request.
 * ctx_len[r] counts the tokens of request r cached BEFORE this iteration; the
 * token with index t of request r sits at position ctx_len[r] + (t - q_indptr[r]).
 * The page list of request r, page_ids[page_indptr[r] .. page_indptr[r+1]),
 * must cover ctx_len[r] + q_len[r] tokens.
 * The host_* arrays are host copies of the same data, used for validation,
 * planning and grid sizing; the device arrays are read by the kernels.
 */
typedef struct nf_batch {
  int32_t n_tokens;
  int32_t n_prefill_reqs;
  int32_t n_decode_reqs;
  const int32_t *q_indptr;         /* [n_reqs + 1]                                 */
  const int32_t *ctx_len;          /* [n_reqs]                                     */
  const int32_t *page_indptr;      /* [n_reqs + 1]                                 */
  const int32_t *page_ids;         /* [page_indptr[n_reqs]]                        */
  const int32_t *host_q_indptr;    /* host                                         */
  const int32_t *host_ctx_len;     /* host                                         */
  const int32_t *host_page_indptr; /* host                                         */
  const int32_t *host_page_ids;    /* host; may be NULL (then page ids are not range-checked) */
} nf_batch;

typedef struct nf_ctx nf_ctx;   /* device, lane streams (with CU masks), events, profile tables */
typedef struct nf_plan nf_plan; /* nano-batch pipeline for one batch + its device work lists      */

/* ---- context ------------------------------------------------------------------------------ */

/* Creates a context on HIP device `device` (makes it current for the calling thread). */
int nf_ctx_create(int device, nf_ctx **out);
void nf_ctx_destroy(nf_ctx *ctx);
/* hipError_t value of the last failed HIP call made through ctx (0 if none). */
int nf_last_hip_error(const nf_ctx *ctx);
/* Static string for a status code. */
const char *nf_strerror(int status);
/* Number of compute units of the context's device. */
int nf_ctx_num_cus(const nf_ctx *ctx);
/* Host-only validation of a model shape and a batch against a pool of num_pages pages:
 * the checks nf_layer_forward performs before launching anything.  Needs no GPU. */
int nf_check_batch(const nf_model_desc *model, const nf_batch *batch, int64_t num_pages);

/*
 * Kernel trace: when enabled, nf_layer_forward brackets kernel launches with timing
 * events on the stream they run on.  level 0 = off, 1 = the attention kernel only,
 * 2 = every kernel.  nf_ctx_read_trace waits for the recorded events, writes up to
 * max_recs records (host array) in launch order, clears the trace and returns the
 * number of records that were pending (or a negative status).
 */
typedef struct nf_trace_rec {
  int32_t kernel;    /* NF_K_* below                                               */
  int32_t op;        /* parent operation: 0 KQV, 1 ATTN, 2 O, 3 UG, 4 D            */
  int32_t nano;      /* nano-batch index                                           */
  int32_t tok_begin, tok_end;
  float start_ms;    /* start relative to the first record of the trace            */
  float ms;          /* duration                                                   */
} nf_trace_rec;
enum { NF_K_RMSNORM = 0, NF_K_GEMM = 1, NF_K_ROPE_APPEND = 2, NF_K_ATTENTION = 3, NF_K_ATTN_MERGE = 4,
       NF_K_MOE_ROUTE = 5, NF_K_MOE_COMBINE = 6 };
int nf_ctx_set_trace(nf_ctx *ctx, int level);
int nf_ctx_read_trace(nf_ctx *ctx, nf_trace_rec *recs, int max_recs);

/*
 * A library-owned stream restricted to n_cus compute units starting at bit first_cu of the
 * device's CU mask (n_cus = 0: unrestricted).  lane (0 or 1) distinguishes streams with the
 * same mask.  Used by the profiler and by tests to run single operations on a CU share;
 * the stream lives until nf_ctx_destroy.  *out receives a hipStream_t.
 */
int nf_ctx_lane_stream(nf_ctx *ctx, int lane, int first_cu, int n_cus, void **out);
/* Same, with an explicit CU mask (host array of `words` 32-bit words, bit i = CU i of the
 * runtime's CU numbering).  Each call creates a new stream owned by ctx. */
int nf_ctx_mask_stream(nf_ctx *ctx, const uint32_t *mask, int words, void **out);

/*
 * Process-wide kernel-variant knobs for tuning runs (Sec. 4.1.1: several implementations
 * per kernel are profiled).  key "attention.variant": 0..7 = pages in flight / occupancy /
 * load-hint trade-off of the attention kernel.  key "gemm.tile": 0 = automatic, 1..25 = force
 * one GEMM implementation (tile shape, LDS feeding scheme, main loop) for every dense
 * operation.  key "search.layers": 1 (default) = the auto-search and nf_simulate_pipeline price
 * one layer on its own; n in 2..16 = they price the time per layer of n consecutive layers
 * pipelined across the layer boundaries, as nf_layers_forward runs them.
 * key "search.rank": 0 (default) = the search returns its best pipeline; r in 1..64 = the best
 * pipeline of the r-th best row of the R -> P table (1 = the best row), whatever its estimate
 * (unsplit when there are fewer rows), so that a caller can refine the model's choice with trial runs.
 * key "search.refine": after the search over (structure, one R -> P row), 1 = the share of every
 * attention nano-operation and the launch order of the nano-batches are refined; 2 (default) = then
 * also the number of nano-operations of every operation (a partition per operation, at most
 * "search.max_parts" = 1..8 nano-operations each, 0 = 8); 0 = one row for all nano-operations, index
 * order, common boundaries.
 * key "gemm.grouped_tile": 0 = automatic, 1 / 7 / 9 / 11 / 12 / 13 / 19 / 21 = force
 * the implementation of the grouped (mixture-of-experts) GEMM.  key "gemm.ksplit": 0 = automatic, 1 / 2 = run a dense operation whose K is
 * summed in two segments (see nf_op_gemm) always with one / with two workgroups per output tile.
 * key "offload.dma": 1 (default) = the simultaneous KV offload copies the rows with a strided
 * device-to-host copy on the copy engines, 0 = with a small kernel that stores to the host buffer.
 * No key ever changes a result bit.  The knobs are process-wide and not thread-safe: they are
 * meant for tuning runs and tests, set while no other thread is inside the library.
 * Returns NF_EINVAL for an unknown key or a value out of range.
 */
int nf_tune_set(const char *key, int value);

/* ---- planning (Sec. 4.1: automated pipeline search) ---------------------------------------- */

/*
 * Measured ceilings of the device, for pricing kernels against what the chip delivers (the
 * measurement section of the paper, Sec. 3.2 / Table 1, uses data-sheet numbers; on a
 * power-limited part the delivered ceilings are lower).  Runs a register-only bf16 MFMA loop
 * on every CU with all-zero operands and with varied operands, and a streaming read of a
 * 4 GiB buffer.  Synchronous on the null stream; allocates and frees 4 GiB of device memory;
 * takes about a second.  Returns NF_EHIP if the device refuses the allocation or a launch.
 */
typedef struct {
  double mfma_bf16_tflops;               /* varied operands: what activation-like data can reach */
  double mfma_bf16_tflops_zero_operands; /* all-zero operands: the clock is not pulled down */
  double hbm_read_gbs;                   /* streaming read, best of three passes */
  int32_t n_cus;
  int32_t reserved;
} nf_peaks;
int nf_measure_peaks(nf_ctx *ctx, nf_peaks *out /* host */);

/*
 * Interference probe (Sec. 4.1.1 profiles how co-running kernels disturb one another): launches
 * n_workgroups (1..4096) single-wavefront workgroups on hip_stream; each follows `iters`
 * dependent loads through a 256 KiB buffer built into the library (it misses the per-CU cache
 * and stays in the L2).  out (DEVICE, 2 * n_workgroups floats): out[2b] = nanoseconds per load
 * seen by workgroup b, out[2b + 1] = the bits of the hardware id register of the compute unit it
 * ran on.  Run alone it gives the L2 hit latency; run beside another kernel it gives what a
 * GEMM's operand loads wait for on a compute unit they share with that kernel's wavefronts (or on
 * a free one).  Asynchronous; allocates nothing.
 */
int nf_probe_load_latency(nf_ctx *ctx, int n_workgroups, int iters, float *out, void *hip_stream);

/*
 * Kernel profiling for the auto-search (Sec. 4.1.1): times every dense
 * operation of `model` alone for batch sizes granule, 2*granule, ... max_tokens
 * with every GEMM tile shape (keeping the best: the kernel -> implementation map),
 * times decode attention alone for every persistent-workgroup count in the search
 * set, and times GEMM || attention pairs to obtain the R -> P resource-mapping
 * table (pairs dominated by more than the scatter of the measurement are dropped), the small
 * row-wise kernels, and how much later a kernel starts when it waits for a kernel of the other
 * lane than when it follows one on its own lane.  Results are kept in ctx and, if cache_path
 * (host string) is not NULL, read from that text file when it matches, else
 * written to it.  Synchronous; allocates and frees its own scratch device memory
 * (weights of one layer plus a few GB of synthetic KV cache).
 */
int nf_profile(nf_ctx *ctx, const nf_model_desc *model, int max_tokens, int granule,
               const char *cache_path);

/*
 * Auto-search (Sec. 4.1.2 - 4.1.3): chooses the number, sizes, order and CU
 * share of the nano-operations for this batch from the profiles held by ctx
 * (built-in analytic estimates if nf_profile was never run).  Uses only the
 * host mirrors of `batch` plus the device arrays' addresses.
 * max_nano = 0 searches; max_nano = 1 yields the unsplit single-stream plan;
 * max_nano = n > 1 bounds the number of nano-batches.
 * granule: nano-batch boundaries are multiples of it (128 is the GEMM-friendly
 * value of Sec. 4.1.1; smaller for tiny batches).
 */
int nf_plan_nanobatches(nf_ctx *ctx, const nf_model_desc *model, const nf_batch *batch,
                        int max_nano, int granule, nf_plan **out);

/*
 * nf_plan_nanobatches with the knobs of the search passed by the caller instead of taken from the
 * process-wide keys of nf_tune_set (two engines in one process do not disturb each other):
 * max_nano, granule as above; layers = 1: the makespan of one layer is minimised, n in 2..16: the
 * time per layer of a run of n consecutive layers pipelined across the layer boundaries (what
 * nf_layers_forward runs); rank, refine, max_parts: keys "search.rank", "search.refine",
 * "search.max_parts".  NF_EINVAL for a value outside its key's range.
 */
typedef struct nf_search_options {
  int32_t max_nano;
  int32_t granule;
  int32_t layers;
  int32_t rank;
  int32_t refine;
  int32_t max_parts;
  int32_t reserved[2];
} nf_search_options;
int nf_plan_search(nf_ctx *ctx, const nf_model_desc *model, const nf_batch *batch,
                   const nf_search_options *options /* host */, nf_plan **out);

/*
 * Host-only forms of the search (no GPU needed; used by CPU tests and offline planning).
 * profile_path: text file written by nf_profile, or NULL for built-in analytic estimates.
 * nf_search_pipeline returns the structure nf_plan_nanobatches would pick from that profile.
 * nf_simulate_pipeline returns the modelled makespan (microseconds) of a given structure:
 * overlap = 0 runs every nano-operation back to back; overlap = 1 runs the GEMM lane and the
 * attention lane concurrently, with rp_row = -1 for no interference (Stage I) or the index
 * of a row of the profile's R -> P table (Stage II: overlapped kernels run at p_gemm and
 * p_attn of their stand-alone speed, so a nano-operation takes D_best / P, Sec. 4.1.3).
 */
/* A token partition per operation (Sec. 4.1.2: the number of nano-operations and their sizes are
 * decided per operation).  Index k: 0 KQV, 1 attention, 2 O, 3 Up/Gate, 4 Down.  Operation k has
 * n[k] nano-operations (1..8) with token boundaries bounds[k][0] = 0 < ... < bounds[k][n[k]] =
 * n_tokens.  Nano-operations depend on each other by the rule of nf_nano_ops_dependent. */
typedef struct nf_partitions {
  int32_t n[5];
  int32_t bounds[5][9];
} nf_partitions;

typedef struct nf_pipeline_desc {
  int32_t n_nano;
  int32_t bounds[9];      /* n_nano + 1 token boundaries                                */
  int32_t overlap;        /* 0 = unsplit / sequential, 1 = two lanes                     */
  int32_t attn_wgs;       /* attention kernel's persistent workgroups (its share R)      */
  int32_t gemm_tile;      /* GEMM implementation of the chosen R -> P pair (0 = per-op best) */
  int32_t reserved;
  int32_t nano_attn_wgs[8]; /* the share per attention nano-operation (Sec. 4.1.1: R per nano-operation) */
  int32_t order[8];       /* launch order: order[k] = index of the nano-batch launched k-th    */
  nf_partitions parts;    /* n[] all zero: every operation is split at `bounds`; otherwise the partition
                             of every operation (then bounds / nano_attn_wgs are the attention
                             operation's, and the order is that of nf_plan_manual_parts)           */
  double est_us;          /* modelled makespan with interference                         */
  double est_us_stage1;   /* same structure without interference                         */
  double est_us_unsplit;  /* the unsplit sequential layer                                */
} nf_pipeline_desc;
int nf_search_pipeline(const nf_model_desc *model, const nf_batch *batch, const char *profile_path,
                       int max_nano, int granule, nf_pipeline_desc *out);
int nf_simulate_pipeline(const nf_model_desc *model, const nf_batch *batch, const char *profile_path,
                         int n_nano, const int32_t *bounds, int overlap, int rp_row, double *est_us);
/* The overlapped pipeline with a table row per nano-batch (rp_rows[i] holds while the attention
 * nano-operation of nano-batch i runs; the rows must share one GEMM implementation) and a launch
 * order (order[k] = nano-batch launched k-th; NULL = index order).  NF_EPLAN for an order that
 * launches an attention nano-operation before a KQV nano-operation it depends on. */
int nf_simulate_pipeline_ops(const nf_model_desc *model, const nf_batch *batch, const char *profile_path,
                             int n_nano, const int32_t *bounds, const int32_t *rp_rows, const int32_t *order,
                             double *est_us);

/* The pipeline with a partition per operation, launched in the order of nf_plan_manual_parts.
 * overlap as in nf_simulate_pipeline; rp_rows: one row index of the profile's R -> P table per
 * attention nano-operation (rows of one GEMM implementation), or NULL for no interference
 * (profile_path may then be NULL too).  NF_EPLAN for invalid partitions. */
int nf_simulate_pipeline_parts(const nf_model_desc *model, const nf_batch *batch, const char *profile_path,
                               const nf_partitions *parts, int overlap, const int32_t *rp_rows, double *est_us);

/* Dependency rule of Sec. 4.1.2: 1 iff the parent operations are dependent (kinds: 0 KQV,
 * 1 ATTN, 2 O, 3 UG, 4 D; KQV -> ATTN -> O -> UG -> D) and the token ranges [b0,e0) and
 * [b1,e1) intersect.  Host only. */
int nf_nano_ops_dependent(int parent_kind, int child_kind, int b0, int e0, int b1, int e1);

/*
 * Explicit pipeline structure (tests and the ablation of Sec. 6.4):
 * n_nano nano-batches with token boundaries bounds[0..n_nano] (host; bounds[0]
 * = 0, bounds[n_nano] = n_tokens, strictly increasing).
 * overlap = 0: every nano-operation on the caller's stream, in order
 *              (nano-batching only).
 * overlap = 1: GEMM nano-operations on one lane (stream), attention
 *              nano-operations on a second lane.  attn_cus / gemm_cus give the
 *              number of compute units each lane's stream is restricted to
 *              (0 = unrestricted).  The attention lane takes the first attn_cus
 *              bits of the CU mask; the GEMM lane the gemm_cus bits after them
 *              when attn_cus + gemm_cus fits the device, else the first gemm_cus.
 * attn_wgs   : number of persistent workgroups (4 wavefronts each) the attention kernel is
 *              launched with; 0 = one per compute unit (the stand-alone optimum), -1 = one per
 *              work unit.  This is the resource share R of the
 *              memory-bound kernel (Sec. 4.1.1): fewer workgroups leave more of every
 *              compute unit to the GEMMs running beside it.  It never changes results.
 */
int nf_plan_manual(nf_ctx *ctx, const nf_model_desc *model, const nf_batch *batch, int n_nano,
                   const int32_t *bounds, int overlap, int attn_cus, int gemm_cus, int attn_wgs,
                   nf_plan **out);

/*
 * nf_plan_manual with a resource share and kernel implementation per nano-operation
 * (Sec. 4.1.1 - 4.1.3: every nano-operation has its own R and its own kernel choice).
 * spec[i] (host array of n_nano entries) belongs to nano-batch i: attn_wgs as in
 * nf_plan_manual for its attention nano-operation, gemm_tile[k] = the GEMM implementation
 * (key "gemm.tile" of nf_tune_set; 0 = automatic) of its KQV, O, Up/Gate and Down
 * nano-operations (k = 0..3).  Neither changes a result bit.
 */
typedef struct nf_nano_spec {
  int32_t attn_wgs;
  int32_t gemm_tile[4];
  int32_t launch_pos;   /* position of this nano-batch in the launch order (a permutation of
                           0..n_nano-1; all zero = index order).  NF_EPLAN if an attention
                           nano-operation would be launched before a KQV it depends on. */
  int32_t reserved[2];
} nf_nano_spec;
int nf_plan_manual_ops(nf_ctx *ctx, const nf_model_desc *model, const nf_batch *batch, int n_nano,
                       const int32_t *bounds, int overlap, int attn_cus, int gemm_cus,
                       const nf_nano_spec *spec, nf_plan **out);

/*
 * Explicit pipeline structure with a partition per operation (Sec. 4.1.2; Fig. 6 shows such
 * pipelines: the operations near a bubble are split into more nano-operations than the others).
 * Launch order of a layer: the KQV nano-operations in range order, each attention nano-operation
 * right behind the KQV nano-operation that launches the last of its tokens; then the O, Up/Gate
 * and Down nano-operations, always the one with the smallest last token among those whose input
 * rows have all been launched (ties: O, then Up/Gate, then Down).  Equal partitions give the order
 * of nf_plan_manual.  overlap, attn_cus, gemm_cus as in nf_plan_manual.
 * attn_wgs : host array, one entry per attention nano-operation (NULL = 0 for all).
 * gemm_tile: host array of 4 (KQV, O, Up/Gate, Down; NULL = automatic).
 * Mixture-of-experts layers need equal Up/Gate and Down partitions (NF_EPLAN otherwise): the rows
 * of a Down nano-operation are the (token, expert) rows its Up/Gate nano-operation grouped.
 * Results do not depend on the partitions by a single bit.
 */
int nf_plan_manual_parts(nf_ctx *ctx, const nf_model_desc *model, const nf_batch *batch,
                         const nf_partitions *parts, int overlap, int attn_cus, int gemm_cus,
                         const int32_t *attn_wgs, const int32_t *gemm_tile, nf_plan **out);

/* Writes a JSON description of the plan into buf (host); returns the number of
 * bytes needed (excluding the terminator), or a negative status. */
int nf_plan_describe(const nf_plan *plan, char *buf, size_t buf_len);
/* Frees the plan.  The work enqueued with it must have completed: its device work lists go
 * back to a small per-process pool (no device-wide wait) and may be rewritten by the next plan. */
void nf_plan_destroy(nf_plan *plan);

/* ---- the layer ------------------------------------------------------------------------------ */

/* Upper bound of the device workspace nf_layer_forward needs for any batch of up to
 * max_tokens tokens whose requests hold at most max_context tokens (0 on a bad model). */
size_t nf_workspace_bytes(const nf_model_desc *model, int max_tokens, int max_context);
/* Exact workspace requirement of nf_layer_forward with this plan. */
size_t nf_plan_workspace_bytes(const nf_plan *plan);
/* Where nf_layer_forward keeps an intermediate inside the caller's workspace, for
 * inspection after a call: name = "h", "qkv", "attn", "y", "f", "moe.expert_ids"
 * (int32 [B, top_k]), "moe.expert_w" (float [B, top_k]), "moe.slot_of". */
int nf_workspace_region(const nf_plan *plan, const char *name, size_t *offset, size_t *bytes);

/*
 * One decoder-layer iteration (Sec. 2.1):
 *   h = RMSNorm(x); [Q|K|V] = h W_qkv^T; rotary embedding on Q, K; K, V appended
 *   to the pages; attention of every token over its request's cached tokens,
 *   the earlier tokens of its chunk and itself; y = x + attn W_o^T;
 *   z = y + FFN(RMSNorm(y)) with FFN = SwiGLU (dense) or top-k routed experts.
 * plan = NULL runs unsplit on hip_stream with a plan the context builds and keeps: it is
 * reused while the batch stays the same; after a change the old one is freed by a later
 * call, once an event recorded behind its last use has passed.  The call does not wait for
 * hip_stream (building the plan for a new batch copies its small work lists to the device
 * with a synchronous copy, like nf_plan_manual).
 * x_in  : bf16 [n_tokens, D]; must not alias x_out.
 * x_out : bf16 [n_tokens, D].
 * Mutates the KV pages and x_out.  Returns NF_EWORKSPACE / NF_EPAGES /
 * NF_ESHAPE / NF_EPLAN before launching anything when arguments are inconsistent.
 */
int nf_layer_forward(nf_ctx *ctx, const nf_model_desc *model, const nf_layer_weights *weights,
                     nf_kv_cache *kv, const nf_batch *batch, const nf_plan *plan,
                     const void *x_in, void *x_out, void *workspace, size_t workspace_bytes,
                     void *hip_stream);

/*
 * n_layers consecutive decoder layers on one dense batch (Sec. 2.1: a layer's output is the
 * next layer's input), with one plan.  weights[l] and kv[l] (host arrays of n_layers
 * structs) belong to layer l; the pools must be pairwise distinct (NF_EINVAL otherwise) and
 * each must satisfy the batch's page table.  With an overlapped plan the nano-operations
 * are pipelined across the layer boundary as in the paper's pipelines (Sec. 4.1.4): the KQV
 * nano-operation of a token range in layer l + 1 is issued behind the Down nano-operation
 * of that range in layer l, so its attention runs beside the remaining GEMMs of layer l.
 * Results are bit-identical to n_layers calls of nf_layer_forward.  plan must not be NULL.
 * workspace: at least nf_layers_workspace_bytes(plan, n_layers) bytes (the plan's workspace
 * plus two intermediate activations).  Errors as nf_layer_forward.
 */
size_t nf_layers_workspace_bytes(const nf_plan *plan, int n_layers);
int nf_layers_forward(nf_ctx *ctx, const nf_model_desc *model, int n_layers,
                      const nf_layer_weights *weights /* host [n_layers] */,
                      nf_kv_cache *kv /* host [n_layers] */, const nf_batch *batch, const nf_plan *plan,
                      const void *x_in, void *x_out, void *workspace, size_t workspace_bytes,
                      void *hip_stream);

/* ---- single operations (kernel-level parity tests and profiling) ---------------------------- */

/* RMSNorm rows ("other operations", Sec. 2.2): out[t] = x[t] * rsqrt(mean(x[t]^2) + eps) * g. */
int nf_op_rmsnorm(const void *x, const void *g, void *out, int n_tokens, int hidden, float eps,
                  void *hip_stream);

/* Dense operation (Sec. 2.2): out[M, N] = epilogue(x[M, K] w[N, K]^T).
 *   NF_EPI_NONE    : plain bf16 store
 *   NF_EPI_RESIDUAL: out = residual[M, N] + product
 *   NF_EPI_SWIGLU  : w is [2*N, K] (gate rows then up rows); out[M, N] = silu(gate) * up
 * Requires K % 64 == 0 and N % 64 == 0.
 * The product is accumulated in fp32 in ascending K order.  Operations with a long K and few
 * output columns - K >= 8192, K >= 2 N, N < 8192, K % 128 == 0, N % 128 == 0, no SwiGLU epilogue; the FFN
 * down projection - instead add the fp32 sums of the two halves of K, so that nano-batches
 * with few rows can spread an output tile over two workgroups; the rule looks at the shape
 * only, never at M, hence a row has the same bits in every nano-batch (inside the layer entry
 * points too). */
enum { NF_EPI_NONE = 0, NF_EPI_RESIDUAL = 1, NF_EPI_SWIGLU = 2 };
int nf_op_gemm(const void *x, const void *w, void *out, const void *residual, int M, int N, int K,
               int epilogue, void *hip_stream);
/* Number of K segments (1 or 2) the library sums a dense operation of this shape in - the rule
 * stated above, part of the numerics contract.  Host only; 0 for arguments nf_op_gemm rejects. */
int nf_gemm_segments(int N, int K, int epilogue);

/* Rotary embedding of the Q and K heads of qkv[n_tokens, (Hq+2Hkv)*dh] (Q rotated
 * in place) and append of K, V into the pages, for tokens [tok_begin, tok_end). */
int nf_op_rope_append(nf_ctx *ctx, const nf_model_desc *model, nf_kv_cache *kv, const nf_batch *batch,
                      const nf_plan *plan, void *qkv, int tok_begin, int tok_end, void *hip_stream);

/* Attention (decode and prefill rows) of tokens [tok_begin, tok_end) of the
 * plan's batch: reads rotated Q from qkv and K, V from the pages; writes
 * attn_out[n_tokens, Hq*dh].  tok_begin/tok_end must be nano-batch boundaries
 * of the plan. */
int nf_op_attention(nf_ctx *ctx, const nf_model_desc *model, const nf_kv_cache *kv,
                    const nf_batch *batch, const nf_plan *plan, const void *qkv, void *attn_out,
                    void *workspace, size_t workspace_bytes, int nano_index, void *hip_stream);

/*
 * nf_op_attention for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and same result bits as nf_op_attention, but the partial results of
 * rows whose keys span several 2048-key chunks live in an array built into the library
 * (nf_attention_static_bytes() = 64 MiB per device, held from library load to process exit)
 * instead of a caller workspace.  The call itself allocates and frees nothing (the plan was
 * built beforehand).  A plan that needs more than the array holds -
 *   plan partial slots * n_kv_heads * (16 * head_dim + 32) * 4 bytes; the LLaMA-3-8B layer at
 *   dense batch 2048 with lognormal contexts up to 8192 needs 53 MiB -
 * is rejected with NF_ESCRATCH before anything is launched.  Nothing in the array has to start
 * at zero (every slot a merge reads was written by the attention kernel of the same call).
 * All calls on one device share the array: two calls whose kernels may overlap in time on one
 * GPU (different streams, or different threads) race and must be serialised by the caller.
 */
size_t nf_attention_static_bytes(void);
int nf_op_attention_static(nf_ctx *ctx, const nf_model_desc *model, const nf_kv_cache *kv,
                           const nf_batch *batch, const nf_plan *plan, const void *qkv, void *attn_out,
                           int nano_index, void *hip_stream);

/* ---- the ends of the iteration (Sec. 2.1: tokens enter through the embedding and leave through
 * the LM head and sampling; Sec. 2.2 counts them among the "other operations") ------------- */

/* out[t, :] = table[id(t), :] for t < n_rows, rows of `width` bf16 (width % 8 == 0), where
 * id(t) = slot_tokens[from_slot[t]] if from_slot is given and from_slot[t] >= 0, else
 * token_ids[t].  The indirection lets a decode token be the token the previous iteration
 * sampled for its request without a trip to the host.  Ids outside [0, table_rows) are
 * clamped.  With table = an activation matrix and token_ids = row numbers this is a row
 * gather (the rows that need logits).  All pointers are device pointers. */
int nf_op_embedding(const int32_t *token_ids, const int32_t *from_slot, const int32_t *slot_tokens,
                    const void *table, int table_rows, void *out, int n_rows, int width, void *hip_stream);

/* Greedy sampling: out[out_index ? out_index[r] : r] = index of the largest of the `vocab`
 * bf16 logits of row r (vocab % 8 == 0), the lowest index among equal values.  The LM head
 * itself is nf_op_rmsnorm followed by nf_op_gemm on the gathered rows. */
int nf_op_argmax(const void *logits, int n_rows, int vocab, const int32_t *out_index, int32_t *out,
                 void *hip_stream);

/*
 * Simultaneous KV offload (Sec. 4.2.2 "Simultaneous offloading"): while it is switched on,
 * every layer iteration copies the K row (after the rotary embedding) and the V row of every
 * token of the batch, as they come out of KQV generation, to host memory, so that the host
 * holds the same K/V as the cache.  The copy is enqueued on a stream of the library behind the
 * nano-batch's attention launch (a strided device-to-host copy on the copy engines, or a small
 * kernel: key "offload.dma" of nf_tune_set) and runs beside the attention and FFN operations;
 * the call's work on hip_stream is complete only after the copies.
 * host_rows: HOST memory the device can write (pinned, e.g. hipHostMalloc), 16-byte aligned;
 *   layer l of a call writes row t (2 * n_kv_heads * head_dim bf16: K heads, then V heads) of
 *   token t at host_rows + l * layer_stride_bytes + t * row bytes (l = 0 for nf_layer_forward).
 *   A batch whose rows do not fit layer_stride_bytes is rejected with NF_EINVAL.
 * host_rows = NULL switches the offload off.
 */
int nf_ctx_set_kv_offload(nf_ctx *ctx, void *host_rows /* host */, size_t layer_stride_bytes);

/*
 * KV loading and scattering (Sec. 4.2.2; also the swap-out and reload of Sec. 4.2.1): the cache
 * of a request crosses the bus as one contiguous copy, and on the device its pages are gathered
 * from, or scattered to, the places the page allocator gave them.
 * scatter = 0: staging page i = pool page page_ids[i];  scatter = 1: pool page page_ids[i] =
 * staging page i, for i < n_pages.  pool (num_pages pages of page_bytes bytes: the pages of
 * nf_kv_cache), staging (n_pages contiguous pages) and page_ids are DEVICE pointers;
 * page_bytes % 16 == 0 (NF_ESHAPE).  Ids outside [0, num_pages) are skipped.  Ids must be
 * distinct when scattering.  Enqueues one kernel on hip_stream; the copy between staging and
 * host memory is the caller's.
 */
int nf_op_move_pages(void *pool, size_t page_bytes, int64_t num_pages, const int32_t *page_ids, int n_pages,
                     void *staging, int scatter, void *hip_stream);

/* ---- continuous batching (Sec. 4.2.1 "Request scheduling"), host only ---------------------- */

/*
 * Forms the dense batch of every iteration the way the paper's runtime does: unfinished
 * decode requests first (one token each), then prefill chunks cut at token granularity so
 * that the batch holds exactly dense_batch tokens whenever enough prompt tokens are
 * waiting; new requests are admitted only while the predicted peak of the page pool (every
 * resident request running to the average output length) stays within the pool; if the
 * pool still runs out, a decode request is swapped out (its pages are to be copied to the
 * host by the caller) and brought back later without recomputation.  The scheduler owns
 * the request states and the page allocator (page ids are shared by all layers' pools);
 * it never touches the GPU.  End-of-sequence is the caller's news: nf_sched_complete(k)
 * tells the scheduler that the outputs of iteration k are known, which lets the caller
 * form iteration k + 1 before iteration k has finished (asynchronous scheduling: a
 * request then decodes at most one token past its end).  The synthetic stand-in for
 * "the model emitted EOS" is the request's output_len.
 */
typedef struct nf_sched nf_sched;
typedef struct {
  int32_t dense_batch;     /* tokens per iteration */
  int32_t page_size;       /* tokens per page */
  int64_t num_pages;       /* pages in (each layer's) pool */
  int32_t max_requests;    /* most requests resident at once */
  int32_t max_chunk;       /* longest prefill chunk of one request per iteration; 0 = no limit */
  int32_t reserve_pages;   /* pages the memory prediction keeps free */
  float avg_decode_len;    /* prior of the average output length (weight: 16 requests) */
} nf_sched_config;

/* One formed batch.  All arrays are host memory owned by the scheduler and stay valid
 * until the next nf_sched_next_batch / nf_sched_destroy.  The first four arrays have the
 * meaning and order of nf_batch (prefill entries first, then decode entries). */
typedef struct {
  int64_t iteration;
  int32_t n_tokens, n_prefill_reqs, n_decode_reqs;
  const int32_t *q_indptr, *ctx_len, *page_indptr, *page_ids;
  const int64_t *request_ids;      /* [n_reqs] */
  /* requests swapped out before this iteration runs: copy pages
   * swap_out_pages[swap_out_indptr[i] .. swap_out_indptr[i+1]) of every layer to the host
   * (they are reused from this iteration on) */
  int32_t n_swap_out;
  const int64_t *swap_out_req;
  const int32_t *swap_out_indptr, *swap_out_pages;
  /* requests brought back: copy their saved pages, in order, into these page ids */
  int32_t n_swap_in;
  const int64_t *swap_in_req;
  const int32_t *swap_in_indptr, *swap_in_pages;
  /* swapped-out requests that turned out to be finished: their host copies can be dropped */
  int32_t n_released;
  const int64_t *released_req;
  /* requests retired (their last token seen) since the previous batch was formed */
  int32_t n_finished;
  const int64_t *finished_req;
} nf_sched_batch;

typedef struct {
  int64_t iterations_formed, iterations_completed;
  int64_t submitted, finished, waiting, resident, swapped;
  int64_t prefill_tokens, decode_tokens, wasted_decode_tokens; /* scheduled so far; wasted = past EOS */
  int64_t swap_outs, swap_ins;
  int64_t free_pages;
  double avg_decode_len;
} nf_sched_stats;

int nf_sched_create(const nf_sched_config *cfg, nf_sched **out);
void nf_sched_destroy(nf_sched *s);
/* Queues a request of prompt_len >= 1 prompt tokens that ends with its output_len-th
 * (>= 1) generated token.  NF_EPAGES if it could never fit the pool. */
int nf_sched_submit(nf_sched *s, int32_t prompt_len, int32_t output_len, int64_t *request_id);
/* Forms the next iteration's batch (n_tokens may be below dense_batch, or 0, when work or
 * memory is short). */
int nf_sched_next_batch(nf_sched *s, nf_sched_batch *out);
/* The outputs of iteration `iteration` are known; iterations complete in order
 * (NF_EINVAL otherwise).  Retires the requests that emitted their last token. */
int nf_sched_complete(nf_sched *s, int64_t iteration);
int nf_sched_get_stats(const nf_sched *s, nf_sched_stats *out);

#ifdef __cplusplus
}
#endif
#endif /* NF_H_ */
