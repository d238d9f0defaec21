// Paged attention (paper Sec. 2.2 "Attention operations"): for every query row,
// softmax(q . K^T / sqrt(dh)) . V over the keys of its request, read from the paged KV
// cache.  Decode rows (one token per request) make this the memory-bound operation of
// the layer: the kernel's job is to stream the K and V blocks from HBM once per kv head.
//
// Work decomposition.  One wavefront handles one work item x one kv head: up to 16 query
// rows that share the kv head (the G = Hq/Hkv q heads of up to 16/G consecutive tokens of
// one request) against a contiguous key range of at most a fixed chunk length.  It keeps
// running softmax statistics (max, sum) and an unnormalised output per row and writes
// them as a partial result; a second kernel merges the partials of a row group in chunk
// order.  The chunking depends only on the request's length, never on the batch split or
// on the number of compute units, so results do not depend on nano-batching.
//
// Matrix-core mapping (all wave64, 16 query rows padded with zeros):
//   S^T[16 keys x 16 rows]  = K_page[16 x dh] . Q^T[dh x 16]   v_mfma_f32_16x16x32_bf16, dh/32 steps
//   O^T[dh x 16 rows]      += V_page^T[dh x 16 keys] . P^T      v_mfma_f32_16x16x16_bf16, dh/16 blocks
// The K block of a page is token-major, so a lane reads 16 contiguous bytes of one key;
// the V block is dimension-major, so a lane reads 8 contiguous bytes (4 keys of one
// dimension) - both straight from global memory into MFMA operand registers.  The
// accumulator layout of S^T (lane = row, 4 consecutive keys) is exactly the B-operand
// layout the second product needs, so P never leaves registers.
#include <math.h>

#include "nf_device.h"
#include "nf_kernels.h"

namespace {

template <int DH>
struct PageRegs {
  bf16x8 k[DH / 32];
  s16x4 v[DH / 16];
};

template <int DH>
__device__ __forceinline__ void load_page(PageRegs<DH>& r, const bf16_t* __restrict__ pages, int page_id, int Hkv,
                                          int kvh, int lane) {
  const int c = lane & 15, g = lane >> 4;
  const bf16_t* kb = pages + (((size_t)page_id * 2 + 0) * Hkv + kvh) * (16 * DH);
  const bf16_t* vb = pages + (((size_t)page_id * 2 + 1) * Hkv + kvh) * (16 * DH);
#pragma unroll
  for (int s = 0; s < DH / 32; ++s)
    r.k[s] = *reinterpret_cast<const bf16x8*>(kb + c * DH + (4 * s + g) * 8);
#pragma unroll
  for (int b = 0; b < DH / 16; ++b)
    r.v[b] = *reinterpret_cast<const s16x4*>(vb + (b * 16 + c) * 16 + 4 * g);
}

template <int DH>
__global__ __launch_bounds__(256) void attention_kernel(const bf16_t* __restrict__ qkv,
                                                        const bf16_t* __restrict__ pages,
                                                        const int32_t* __restrict__ page_indptr,
                                                        const int32_t* __restrict__ page_ids,
                                                        const NfAttnItem* __restrict__ items, int head_groups,
                                                        int Hq, int Hkv, int n_qkv, float scale_log2,
                                                        float* __restrict__ parts) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int item_idx = blockIdx.x / head_groups;
  const int kvh = (blockIdx.x % head_groups) * 4 + wave;
  if (kvh >= Hkv) return;  // no workgroup barriers in this kernel
  const NfAttnItem it = items[item_idx];
  const int G = Hq / Hkv;
  const int c = lane & 15, g = lane >> 4;
  const int n_rows = it.n_tok * G;

  // Q^T operand: lane (row c, k-group g) holds Q[row c][(4s+g)*8 .. +8] for step s
  bf16x8 qf[DH / 32];
  {
    const int j = c / G, hg = c - j * G;
    const bf16_t* qrow = qkv + (size_t)(it.tok0 + j) * n_qkv + (size_t)(kvh * G + hg) * DH;
#pragma unroll
    for (int s = 0; s < DH / 32; ++s) {
      if (c < n_rows) {
        qf[s] = *reinterpret_cast<const bf16x8*>(qrow + (4 * s + g) * 8);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[s][e] = (__bf16)0.0f;
      }
    }
  }
  // last key this lane's row may read (rows past n_rows read nothing)
  const int lim = c < n_rows ? it.pos0 + c / G : -1;

  f32x4 o[DH / 16];
#pragma unroll
  for (int b = 0; b < DH / 16; ++b) o[b] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  const int32_t* plist = page_ids + page_indptr[it.req];
  const int p_begin = it.key_begin >> 4;
  const int p_end = (it.key_end + 15) >> 4;

  PageRegs<DH> cur, nxt;
  load_page<DH>(cur, pages, plist[p_begin], Hkv, kvh, lane);
  for (int p = p_begin; p < p_end; ++p) {
    if (p + 1 < p_end) load_page<DH>(nxt, pages, plist[p + 1], Hkv, kvh, lane);

    // scores S^T: lane (row c, g) gets keys 16p + 4g + i
    f32x4 st = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < DH / 32; ++s) st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.k[s], qf[s], st, 0, 0, 0);
    const int key0 = p * 16 + 4 * g;
    float sc[4];
    float pm = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sc[i] = (key0 + i <= lim) ? st[i] * scale_log2 : -INFINITY;
      pm = fmaxf(pm, sc[i]);
    }
    pm = fmaxf(pm, __shfl_xor(pm, 16, 64));
    pm = fmaxf(pm, __shfl_xor(pm, 32, 64));
    const float m_new = fmaxf(m_run, pm);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    float pr[4];
    float ps = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pr[i] = __builtin_amdgcn_exp2f(sc[i] - m_use);
      ps += pr[i];
    }
    l_run = l_run * alpha + ps;
    m_run = m_new;
    bf16x4 pb = {(__bf16)pr[0], (__bf16)pr[1], (__bf16)pr[2], (__bf16)pr[3]};
    const s16x4 pf = __builtin_bit_cast(s16x4, pb);

    // a page that reaches past the chunk's last key: clear V beyond it so that
    // 0 * (uninitialised slot) cannot produce NaN
    if (p * 16 + 16 > it.key_end) {
#pragma unroll
      for (int b = 0; b < DH / 16; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (key0 + i >= it.key_end) cur.v[b][i] = 0;
    }
#pragma unroll
    for (int b = 0; b < DH / 16; ++b) {
      o[b] *= alpha;
      o[b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(cur.v[b], pf, o[b], 0, 0, 0);
    }
    cur = nxt;
  }

  // partial result: [16 rows][DH] floats, then m[16], l[16]
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  float* part = parts + ((size_t)it.part * Hkv + kvh) * (16 * DH + 32);
  if (c < n_rows) {
#pragma unroll
    for (int b = 0; b < DH / 16; ++b) *reinterpret_cast<f32x4*>(part + c * DH + b * 16 + 4 * g) = o[b];
    if (g == 0) {
      part[16 * DH + c] = m_run;
      part[16 * DH + 16 + c] = l_run;
    }
  }
}

// Merge the partial results of one row group in chunk order and write bf16 output.
// grid (n_groups, Hkv), DH threads: thread d owns output dimension d of every row.
template <int DH>
__global__ __launch_bounds__(DH) void attention_merge_kernel(const float* __restrict__ parts,
                                                             const NfAttnGroup* __restrict__ groups, int Hq, int Hkv,
                                                             bf16_t* __restrict__ out) {
  const NfAttnGroup gr = groups[blockIdx.x];
  const int kvh = blockIdx.y;
  const int G = Hq / Hkv;
  const int d = threadIdx.x;
  const int n_rows = gr.n_tok * G;
  const size_t stride = (size_t)Hkv * (16 * DH + 32);
  const float* base = parts + ((size_t)gr.part0 * Hkv + kvh) * (16 * DH + 32);
  for (int r = 0; r < n_rows; ++r) {
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

hipError_t nf_launch_attention(const void* qkv, const void* pages, const int32_t* page_indptr,
                               const int32_t* page_ids, const NfAttnItem* items, int n_items,
                               const NfAttnShape& shp, float* parts, hipStream_t s) {
  if (n_items <= 0) return hipSuccess;
  const int head_groups = (shp.n_kv_heads + 3) / 4;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)shp.head_dim);
  const dim3 grid((unsigned)n_items * head_groups), block(256);
  if (shp.head_dim == 128) {
    attention_kernel<128><<<grid, block, 0, s>>>((const bf16_t*)qkv, (const bf16_t*)pages, page_indptr, page_ids,
                                                 items, head_groups, shp.n_q_heads, shp.n_kv_heads, shp.n_qkv,
                                                 scale_log2, parts);
  } else if (shp.head_dim == 64) {
    attention_kernel<64><<<grid, block, 0, s>>>((const bf16_t*)qkv, (const bf16_t*)pages, page_indptr, page_ids,
                                                items, head_groups, shp.n_q_heads, shp.n_kv_heads, shp.n_qkv,
                                                scale_log2, parts);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t nf_launch_attention_merge(const float* parts, const NfAttnGroup* groups, int n_groups,
                                     const NfAttnShape& shp, void* attn_out, hipStream_t s) {
  if (n_groups <= 0) return hipSuccess;
  const dim3 grid(n_groups, shp.n_kv_heads);
  if (shp.head_dim == 128) {
    attention_merge_kernel<128><<<grid, dim3(128), 0, s>>>(parts, groups, shp.n_q_heads, shp.n_kv_heads,
                                                           (bf16_t*)attn_out);
  } else if (shp.head_dim == 64) {
    attention_merge_kernel<64><<<grid, dim3(64), 0, s>>>(parts, groups, shp.n_q_heads, shp.n_kv_heads,
                                                         (bf16_t*)attn_out);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
