// Paged attention (paper Sec. 2.2 "Attention operations"): for every query row,
// softmax(q . K^T / sqrt(dh)) . V over the keys of its request, read from the paged KV
// cache.  Decode rows (one token per request) make this the memory-bound operation of
// the layer: the kernel's job is to stream the K and V blocks from HBM once per kv head.
//
// Work decomposition.  One wavefront handles one work item x one kv head: up to 16 query
// rows that share the kv head (the G = Hq/Hkv q heads of up to 16/G consecutive tokens of
// one request) against a contiguous key range of at most a fixed chunk length.  It keeps
// running softmax statistics (max, sum) and an unnormalised output per row.  Rows whose
// keys fit one chunk are normalised and written directly; for longer rows the result of
// every chunk is written as a partial result and a second kernel merges the partials of a
// row group in chunk order.  The chunking depends only on the request's length, never on
// the batch split or on the number of compute units, so results do not depend on
// nano-batching.
//
// Matrix-core mapping (all wave64, 16 query rows padded with zeros):
//   S^T[16 keys x 16 rows]  = K_page[16 x dh] . Q^T[dh x 16]   v_mfma_f32_16x16x32_bf16, dh/32 steps
//   O^T[dh x 16 rows]      += V_page^T[dh x 16 keys] . P^T      v_mfma_f32_16x16x16_bf16, dh/16 blocks
// The K and V blocks of a page are stored in MFMA operand order, so every wavefront load
// lands straight in operand registers: K as [dh/32][16 keys][32] (a wavefront load is 1 KiB
// of contiguous memory: 16 keys x 64 bytes), V as [4 key groups][dh/32][16 dims][2 blocks]
// [4 keys] (a wavefront load is four runs of 256 bytes).  Measured: the four-run V load
// streams as fast as a contiguous one, while a row-major K block (sixteen 64-byte runs per
// load) is 22 % slower.  Both orders keep the pieces a single token writes close together
// (4 and 8 cache lines per head instead of 16 and 32 with the key index innermost in K and
// the key group innermost in V): the append of the batch's tokens is a scatter of partial
// cache lines, and it costs in its own kernel and again when this kernel reads the pages
// while the partial lines are written back.  The accumulator
// layout of S^T (lane = row, 4 consecutive keys) is exactly the B-operand layout the second
// product needs, so P never leaves registers.
#include <math.h>

#include <algorithm>

#include "nf_device.h"
#include "nf_kernels.h"

namespace {

template <int DH>
struct PageRegs {
  bf16x8 k[DH / 32];
  s16x4 v[DH / 16];
};

// Issues the loads of one page.  `page_base` is wave-uniform, so the loads take the
// scalar-base + 32-bit lane offset form.  K step s (dimensions 32s .. 32s+31 of all 16 keys)
// is lanes x 16 bytes at s * 1024; V pair q (blocks 2q, 2q+1) is lanes x 16 bytes at
// q * 256 inside each key group's run.
template <int DH, bool NT = false>
__device__ __forceinline__ void load_page(PageRegs<DH>& r, const char* __restrict__ page_base, uint32_t v_block_off,
                                          uint32_t koff, uint32_t voff) {
  const char* vb = page_base + v_block_off;
#pragma unroll
  for (int s = 0; s < DH / 32; ++s) {
    const bf16x8* p = reinterpret_cast<const bf16x8*>(page_base + koff + s * 1024);
    r.k[s] = NT ? __builtin_nontemporal_load(p) : *p;  // NT: streaming hint, the cache is read once
  }
#pragma unroll
  for (int q = 0; q < DH / 32; ++q) {
    const bf16x8* p = reinterpret_cast<const bf16x8*>(vb + voff + q * 256);
    const bf16x8 t = NT ? __builtin_nontemporal_load(p) : *p;
    r.v[2 * q] = __builtin_bit_cast(s16x4, (bf16x4){t[0], t[1], t[2], t[3]});
    r.v[2 * q + 1] = __builtin_bit_cast(s16x4, (bf16x4){t[4], t[5], t[6], t[7]});
  }
}

template <int DH>
struct AttnState {
  f32x4 o[DH / 16];
  float m_run, l_run;
};

// One page (16 keys) of online softmax.  p = page index within the request.
template <int DH>
__device__ __forceinline__ void attend_page(AttnState<DH>& st, PageRegs<DH>& pg, const bf16x8 (&qf)[DH / 32], int p,
                                            int g, int lim, int key_end, float scale_log2) {
  // scores S^T: lane (row c, g) gets keys 16p + 4g + i
  f32x4 sc4 = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < DH / 32; ++s) sc4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pg.k[s], qf[s], sc4, 0, 0, 0);
  const int key0 = p * 16 + 4 * g;
  float sc[4];
  float pm = -INFINITY;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    sc[i] = (key0 + i <= lim) ? sc4[i] * scale_log2 : -INFINITY;
    pm = fmaxf(pm, sc[i]);
  }
  pm = fmaxf(pm, __shfl_xor(pm, 16, 64));
  pm = fmaxf(pm, __shfl_xor(pm, 32, 64));
  const float m_new = fmaxf(st.m_run, pm);
  const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(st.m_run - m_use);
  float pr[4];
  float ps = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    pr[i] = __builtin_amdgcn_exp2f(sc[i] - m_use);
    ps += pr[i];
  }
  st.l_run = st.l_run * alpha + ps;
  st.m_run = m_new;
  bf16x4 pb = {(__bf16)pr[0], (__bf16)pr[1], (__bf16)pr[2], (__bf16)pr[3]};
  const s16x4 pf = __builtin_bit_cast(s16x4, pb);
  // a page that reaches past the chunk's last key: clear V beyond it so that
  // 0 * (uninitialised slot) cannot produce NaN
  if (p * 16 + 16 > key_end) {
#pragma unroll
    for (int b = 0; b < DH / 16; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (key0 + i >= key_end) pg.v[b][i] = 0;
  }
  // the running maximum moves on few pages only: skip the rescale when no lane needs it
  if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
    for (int b = 0; b < DH / 16; ++b) st.o[b] *= alpha;
  }
#pragma unroll
  for (int b = 0; b < DH / 16; ++b)
    st.o[b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pg.v[b], pf, st.o[b], 0, 0, 0);
}

template <int DH, int NBUF, int WAVES_PER_SIMD, bool NT = false>
__global__ __launch_bounds__(256, WAVES_PER_SIMD) void attention_kernel(const bf16_t* __restrict__ qkv,
                                                        const bf16_t* __restrict__ pages,
                                                        const int32_t* __restrict__ page_indptr,
                                                        const int32_t* __restrict__ page_ids,
                                                        const NfAttnItem* __restrict__ items, int n_work,
                                                        int head_groups, int Hq, int Hkv, int n_qkv,
                                                        float scale_log2, float* __restrict__ parts,
                                                        bf16_t* __restrict__ out) {
  constexpr int NIDS = NF_ATTN_CHUNK / 1024;  // page-id registers: 64 pages of 16 keys each
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int G = Hq / Hkv;
  const int c = lane & 15, g = lane >> 4;
  const int stride = gridDim.x;

  // Descriptor of work unit `w` (clamped past the end: such a unit is fetched but never run).
  auto item_of = [&](int w) { return items[(w < n_work ? w : n_work - 1) / head_groups]; };
  // Operands that do not depend on the page data: the Q^T fragments (lane (row c, k-group g)
  // holds Q[row c][(4s+g)*8 .. +8] for step s; rows past the item's are zero) and the physical
  // ids of the item's pages.  The chunk spans at most 64 * NIDS pages: lane i keeps the ids of
  // pages p_begin + i, p_begin + 64 + i, ..., so the id of any page is one cross-lane read away
  // and no page load waits on the page table.
  auto load_operands = [&](const NfAttnItem& it, int list_base, int w, bf16x8 (&qf)[DH / 32], int (&ids)[NIDS]) {
    int kvh = (w % head_groups) * 4 + wave;
    kvh = kvh < Hkv ? kvh : Hkv - 1;
    const int n_rows = it.n_tok * G;
    const int j = c / G, hg = c - j * G;
    const bf16_t* qrow = qkv + (size_t)(it.tok0 + (c < n_rows ? j : 0)) * n_qkv + (size_t)(kvh * G + hg) * DH;
#pragma unroll
    for (int s = 0; s < DH / 32; ++s) {
      qf[s] = *reinterpret_cast<const bf16x8*>(qrow + (4 * s + g) * 8);
      if (c >= n_rows) {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[s][e] = (__bf16)0.0f;
      }
    }
    const int p_begin = it.key_begin >> 4;
    const int n_pages = ((it.key_end + 15) >> 4) - p_begin;
#pragma unroll
    for (int k = 0; k < NIDS; ++k)
      ids[k] = lane + 64 * k < n_pages ? page_ids[list_base + p_begin + 64 * k + lane] : 0;
  };

  // Persistent workgroups: the list is sorted longest first and is dealt out in rounds of
  // gridDim.x units, forwards in even rounds and backwards in odd ones, so that the workgroup
  // that drew the longest unit of one round draws the shortest of the next and all workgroups
  // end up with nearly the same number of pages (dealing every round forwards leaves the first
  // workgroup with a few per cent more than the last).  There are no workgroup barriers: the
  // four wavefronts (four kv heads of one item) run independently.
  //
  // The chain descriptor -> page-list base -> page ids / Q -> first page costs three memory
  // round trips before a unit streams its first byte, and a wavefront runs tens of units.
  // It is therefore software-pipelined over units: while unit k streams, the operands of
  // unit k + 1 and the descriptor and page-list base of unit k + 2 are fetched.
  auto unit_at = [&](int r) { return r * stride + ((r & 1) ? stride - 1 - (int)blockIdx.x : (int)blockIdx.x); };
  int round = 0;
  int work = unit_at(0);
  NfAttnItem it = item_of(work);
  int list_base = page_indptr[it.req];
  NfAttnItem it1 = item_of(unit_at(1));
  int list_base1 = page_indptr[it1.req];
  bf16x8 qf[DH / 32];
  int ids[NIDS];
  load_operands(it, list_base, work, qf, ids);

  const size_t blk_bytes = (size_t)16 * DH * 2;
  const size_t page_bytes = 2 * (size_t)Hkv * blk_bytes;
  const uint32_t v_block_off = (uint32_t)((size_t)Hkv * blk_bytes);
  const uint32_t koff = (uint32_t)((c * 4 + g) * 16);      // K: [dh/32][16 keys][32]; step s at s * 1024, key c, dims 8g..
  const uint32_t voff = (uint32_t)(g * DH * 8 + c * 16);  // V: [4 g][dh/32][16 c][2][4 keys]

  // The ring of page registers lives across units: while the last pages of a unit are
  // multiplied, its free slots already receive the first pages of the next unit (`pre` of
  // them), so the memory pipeline does not drain and refill at every unit boundary (that cost
  // 6 - 8 us per unit).  A unit occupies a whole number of turns of the ring - an odd page
  // count leaves a slot position unused - which keeps the slot of every page a compile-time
  // index.
  PageRegs<DH> buf[NBUF];
  int pre = 0;
  auto page_id = [&](const int (&id)[NIDS], int i) {
    int v = __builtin_amdgcn_readlane(id[0], i & 63);
#pragma unroll
    for (int k = 1; k < NIDS; ++k)
      if ((i >> 6) == k) v = __builtin_amdgcn_readlane(id[k], i & 63);
    return v;
  };

  for (;;) {
    const int kvh = (work % head_groups) * 4 + wave;
    const int work1 = unit_at(round + 1);
    bf16x8 qf1[DH / 32];
    int ids1[NIDS];
    load_operands(it1, list_base1, work1, qf1, ids1);
    const NfAttnItem it2 = item_of(unit_at(round + 2));
    int list_base2 = 0;

    // only the last round can be short: there a workgroup's unit may lie past the end
    if (work < n_work && kvh < Hkv) {
      const int n_rows = it.n_tok * G;
      // last key this lane's row may read (rows past n_rows read nothing)
      const int lim = c < n_rows ? it.pos0 + c / G : -1;
      AttnState<DH> st;
#pragma unroll
      for (int b = 0; b < DH / 16; ++b) st.o[b] = (f32x4){0.f, 0.f, 0.f, 0.f};
      st.m_run = -INFINITY;
      st.l_run = 0.f;
      const int p_begin = it.key_begin >> 4;
      const int n_pages = ((it.key_end + 15) >> 4) - p_begin;
      const char* head_base = reinterpret_cast<const char*>(pages) + (size_t)kvh * blk_bytes;
      // the next unit of this wavefront, if it has one: its page ids are in ids1 by now
      const int kvh1 = (work1 % head_groups) * 4 + wave;
      const int np1 = (work1 < n_work && kvh1 < Hkv) ? ((it1.key_end + 15) >> 4) - (it1.key_begin >> 4) : 0;
      const char* head_base1 = reinterpret_cast<const char*>(pages) + (size_t)(kvh1 < Hkv ? kvh1 : 0) * blk_bytes;
      // The ids of the next unit's first pages come through the scalar cache: a cross-lane read
      // of ids1 here would have to wait for that vector load, and with it (loads return in
      // order, the number issued since is not known at compile time) for every page in flight.
      int nid[NBUF];
#pragma unroll
      for (int j = 0; j < NBUF; ++j) nid[j] = j < np1 ? page_ids[list_base1 + (it1.key_begin >> 4) + j] : 0;
#define NF_PAGE_BASE(i) (head_base + (size_t)(uint32_t)page_id(ids, (i)) * page_bytes)
#define NF_NEXT_PAGE_BASE(j) (head_base1 + (size_t)(uint32_t)nid[j] * page_bytes)
      // NBUF pages in flight per wavefront: a ring of register buffers, refilled as soon as a
      // page has been consumed; the first `pre` pages were loaded during the previous unit.
      // (Loads return in order, and because a page's loads are conditional the generated code
      // waits for everything in flight once per turn of the ring.  A variant with a fixed
      // number of loads per step - a dummy page for a slot with nothing to fetch - gets exact
      // waits from the compiler, but measured slower for every ring depth and grid size but
      // one; more slots serve a small grid better.)
#pragma unroll
      for (int j = 0; j < NBUF; ++j)
        if (j >= pre && j < n_pages) load_page<DH, NT>(buf[j], NF_PAGE_BASE(j), v_block_off, koff, voff);
      const int padded = (n_pages + NBUF - 1) / NBUF * NBUF;
      int pre_next = 0;
      for (int i = 0; i < n_pages; i += NBUF) {
#pragma unroll
        for (int j = 0; j < NBUF; ++j) {
          const int q = i + j, t = q + NBUF;  // this slot's page, and the stream position it is refilled for
          // where the slot's next page comes from is decided first, so that there is one load
          // site per slot (two sites in two branches cost 10 % at small grids: the generated
          // waits get more conservative with every site)
          const char* base = reinterpret_cast<const char*>(pages);
          bool has_page = true;
          if (t < n_pages) {
            base = NF_PAGE_BASE(t);
          } else if (t >= padded && t - padded < np1) {
            base = NF_NEXT_PAGE_BASE(j);  // t - padded == j
            ++pre_next;
          } else {
            has_page = false;
          }
          if (q < n_pages) attend_page<DH>(st, buf[j], qf, p_begin + q, g, lim, it.key_end, scale_log2);
          if (has_page) load_page<DH, NT>(buf[j], base, v_block_off, koff, voff);
        }
        if (i == 0) list_base2 = page_indptr[it2.req];  // its descriptor has arrived by now
      }
      pre = pre_next;
#undef NF_PAGE_BASE
#undef NF_NEXT_PAGE_BASE

      float l_run = st.l_run;
      l_run += __shfl_xor(l_run, 16, 64);
      l_run += __shfl_xor(l_run, 32, 64);
      if (it.part < 0) {
        // the only chunk of its rows: normalise and write the attention output directly
        if (c < n_rows) {
          const int tok = it.tok0 + c / G, hq = kvh * G + (c % G);
          bf16_t* orow = out + ((size_t)tok * Hq + hq) * DH + 4 * g;
#pragma unroll
          for (int b = 0; b < DH / 16; ++b) {
            u16x4 v;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = f2bf(st.o[b][i] / l_run);
            *reinterpret_cast<u16x4*>(orow + b * 16) = v;
          }
        }
      } else {
        // partial result: [16 rows][DH] floats, then m[16], l[16]
        float* part = parts + ((size_t)it.part * Hkv + kvh) * (16 * DH + 32);
        if (c < n_rows) {
#pragma unroll
          for (int b = 0; b < DH / 16; ++b) *reinterpret_cast<f32x4*>(part + c * DH + b * 16 + 4 * g) = st.o[b];
          if (g == 0) {
            part[16 * DH + c] = st.m_run;
            part[16 * DH + 16 + c] = l_run;
          }
        }
      }
    } else {
      list_base2 = page_indptr[it2.req];
      pre = 0;
    }

    ++round;
    if (round * stride >= n_work) break;
    work = work1;
    it = it1;
    list_base = list_base1;
#pragma unroll
    for (int s = 0; s < DH / 32; ++s) qf[s] = qf1[s];
#pragma unroll
    for (int k = 0; k < NIDS; ++k) ids[k] = ids1[k];
    it1 = it2;
    list_base1 = list_base2;
  }
}

// Merge the partial results of one row group in chunk order and write bf16 output.
// grid (n_groups, Hkv), block (DH, 4): thread (d, y) owns output dimension d of the rows
// y, y + 4, ... (the rows are independent chains of dependent loads: four run side by side).
template <int DH>
__global__ __launch_bounds__(DH * 4) void attention_merge_kernel(const float* __restrict__ parts,
                                                             const NfAttnGroup* __restrict__ groups, int Hq, int Hkv,
                                                             bf16_t* __restrict__ out) {
  const NfAttnGroup gr = groups[blockIdx.x];
  const int kvh = blockIdx.y;
  const int G = Hq / Hkv;
  const int d = threadIdx.x;
  const int n_rows = gr.n_tok * G;
  const size_t stride = (size_t)Hkv * (16 * DH + 32);
  const float* base = parts + ((size_t)gr.part0 * Hkv + kvh) * (16 * DH + 32);
  for (int r = threadIdx.y; r < n_rows; r += 4) {
    float M = -INFINITY;
    for (int j = 0; j < gr.n_parts; ++j) M = fmaxf(M, base[j * stride + 16 * DH + r]);
    float L = 0.f, acc = 0.f;
    for (int j = 0; j < gr.n_parts; ++j) {
      const float* pj = base + j * stride;
      const float mj = pj[16 * DH + r];
      const float w = (mj == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mj - M);
      L += pj[16 * DH + 16 + r] * w;
      acc += pj[r * DH + d] * w;
    }
    const int tok = gr.tok0 + r / G, hq = kvh * G + (r % G);
    out[((size_t)tok * Hq + hq) * DH + d] = f2bf(acc / L);
  }
}

}  // namespace

// Kernel variant: pages in flight per wavefront (more pages = more bytes in flight per
// wavefront but fewer resident wavefronts).  With the default (5: two pages) the launcher
// switches to four pages for small grids, where each wavefront has to stream more.
static int g_attn_variant = 5;
void nf_set_attention_variant(int v) { g_attn_variant = v; }


template <int DH>
static hipError_t launch_attention_dh(int variant, dim3 grid, hipStream_t s, const bf16_t* qkv, const bf16_t* pages,
                                      const int32_t* page_indptr, const int32_t* page_ids, const NfAttnItem* items,
                                      int n_work, int head_groups, const NfAttnShape& shp, float scale_log2,
                                      float* parts, bf16_t* out) {
#define NF_ATTN_LAUNCH(NB, W, NT)                                                                                  \
  attention_kernel<DH, NB, W, NT><<<grid, dim3(256), 0, s>>>(qkv, pages, page_indptr, page_ids, items, n_work,          \
                                                         head_groups, shp.n_q_heads, shp.n_kv_heads, shp.n_qkv,     \
                                                         scale_log2, parts, out)
  switch (variant) {
    case 0: NF_ATTN_LAUNCH(2, 3, false); break;
    case 1: NF_ATTN_LAUNCH(3, 2, false); break;
    case 2: NF_ATTN_LAUNCH(4, 2, false); break;
    case 3: NF_ATTN_LAUNCH(5, 2, false); break;
    case 4: NF_ATTN_LAUNCH(3, 2, true); break;
    case 5: NF_ATTN_LAUNCH(2, 3, true); break;
    case 6: NF_ATTN_LAUNCH(4, 2, true); break;
    case 7: NF_ATTN_LAUNCH(5, 2, true); break;
    default: return hipErrorInvalidValue;
  }
#undef NF_ATTN_LAUNCH
  return hipGetLastError();
}

hipError_t nf_launch_attention(const void* qkv, const void* pages, const int32_t* page_indptr,
                               const int32_t* page_ids, const NfAttnItem* items, int n_items,
                               const NfAttnShape& shp, float* parts, void* attn_out, int max_workgroups,
                               hipStream_t s, long long item_pages, int n_cus) {
  if (n_items <= 0) return hipSuccess;
  const int head_groups = (shp.n_kv_heads + 3) / 4;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)shp.head_dim);
  const int n_work = n_items * head_groups;
  // Default: one persistent workgroup per compute unit; for a launch long enough to be bound
  // by HBM (more than 1024 pages per workgroup) only 11/16 of that (176 of 256).  Measured on
  // MI355X at the 8B layer's dense batch of 2048 with 2.5 M cached tokens: 1.50 ms against
  // 1.54 with a workgroup on every CU and 1.55 with 160 - enough bytes in flight to saturate
  // HBM, fewer requesters queueing in front of it - while the short launches of the iteration
  // loop (0.6 M cached tokens, many prefill rows) lose 2 % of the layer with 176.  More
  // workgroups than CUs lose much more (320 on 256 CUs: 25 %).
  if (n_cus <= 0) {  // no context at hand: the device that is current now
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      n_cus = prop.multiProcessorCount;
    if (n_cus <= 0) n_cus = 256;
  }
  const bool hbm_bound = item_pages * head_groups >= 1024LL * n_cus;
  const int automatic = hbm_bound ? std::max(8, n_cus * 11 / 16 / 8 * 8) : n_cus;
  int wgs = max_workgroups > 0 ? max_workgroups : (max_workgroups < 0 ? n_work : automatic);
  if (wgs > n_work) wgs = n_work;
  const dim3 grid((unsigned)wgs);
  // measured: at 5/8 of the CUs and below, four pages in flight per wavefront beat two (128
  // workgroups: 1.72 against 1.83 ms)
  const int variant = (g_attn_variant == 5 && max_workgroups >= 0 && 8 * wgs <= 5 * n_cus) ? 6 : g_attn_variant;

  if (shp.head_dim == 128)
    return launch_attention_dh<128>(variant, grid, s, (const bf16_t*)qkv, (const bf16_t*)pages, page_indptr,
                                    page_ids, items, n_work, head_groups, shp, scale_log2, parts, (bf16_t*)attn_out);
  if (shp.head_dim == 64)
    return launch_attention_dh<64>(variant, grid, s, (const bf16_t*)qkv, (const bf16_t*)pages, page_indptr,
                                   page_ids, items, n_work, head_groups, shp, scale_log2, parts, (bf16_t*)attn_out);
  return hipErrorInvalidValue;
}

hipError_t nf_launch_attention_merge(const float* parts, const NfAttnGroup* groups, int n_groups,
                                     const NfAttnShape& shp, void* attn_out, hipStream_t s) {
  if (n_groups <= 0) return hipSuccess;
  const dim3 grid(n_groups, shp.n_kv_heads);
  if (shp.head_dim == 128) {
    attention_merge_kernel<128><<<grid, dim3(128, 4), 0, s>>>(parts, groups, shp.n_q_heads, shp.n_kv_heads,
                                                           (bf16_t*)attn_out);
  } else if (shp.head_dim == 64) {
    attention_merge_kernel<64><<<grid, dim3(64, 4), 0, s>>>(parts, groups, shp.n_q_heads, shp.n_kv_heads,
                                                         (bf16_t*)attn_out);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---- partial results in a static device array (for callers that cannot allocate) ----------
//
// nf_op_attention_static keeps the partial results of multi-chunk rows here instead of in a
// caller-provided workspace.  Every device the library runs on holds its own copy of the array
// (at its own address) until the process ends.  Host code never uses the array's name as an
// address: nf_attention_static_scratch() asks the runtime for the device address once per
// device, with that device current, and hands that pointer to the kernels.
static __device__ __align__(256) unsigned char scratch[NF_ATTN_STATIC_BYTES];

hipError_t nf_attention_static_scratch(int device, float** ptr, size_t* bytes) {
  constexpr int kMaxDevices = 64;
  static float* per_device[kMaxDevices] = {};
  if (!ptr || !bytes || device < 0 || device >= kMaxDevices) return hipErrorInvalidValue;
  if (!per_device[device]) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return e;
    if (cur != device) return hipErrorInvalidDevice;   // the caller makes the device current first
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    per_device[device] = (float*)p;
  }
  *ptr = per_device[device];
  *bytes = NF_ATTN_STATIC_BYTES;
  return hipSuccess;
}
