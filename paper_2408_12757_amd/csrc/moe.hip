// Mixture-of-experts feed-forward stage (paper Sec. 4.1.4: the FFN is a grouped GEMM and
// there is an additional gate routing operation): router + top-k, the stable counting
// sort that groups (token, expert) rows by expert, and the weighted combine.
#include <math.h>

#include "nf_device.h"
#include "nf_kernels.h"

namespace {

constexpr int MAX_E = 64;
constexpr int MAX_K = 4;

// One wavefront per token: logits[e] = h[t] . w_router[e] in fp32; the top_k largest logits
// (ties to the lower expert index); softmax over the selected logits.
__global__ __launch_bounds__(256) void moe_router_kernel(const bf16_t* __restrict__ h, const bf16_t* __restrict__ wr,
                                                         int32_t* __restrict__ ids, float* __restrict__ wts,
                                                         int tok_begin, int tok_end, int D, int E, int K) {
  const int lane = threadIdx.x & 63;
  const int t = tok_begin + blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= tok_end) return;
  const bf16_t* hr = h + (size_t)t * D;
  float sel_v[MAX_K];
  int sel_i[MAX_K];
#pragma unroll
  for (int k = 0; k < MAX_K; ++k) {
    sel_v[k] = -INFINITY;
    sel_i[k] = 0x7fffffff;
  }
  for (int e = 0; e < E; ++e) {
    const bf16_t* w = wr + (size_t)e * D;
    float acc = 0.f;
    for (int v = lane; v < (D >> 3); v += 64) {
      const u32x4 a = *reinterpret_cast<const u32x4*>(hr + v * 8);
      const u32x4 b = *reinterpret_cast<const u32x4*>(w + v * 8);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc += __uint_as_float(a[i] << 16) * __uint_as_float(b[i] << 16);
        acc += __uint_as_float(a[i] & 0xffff0000u) * __uint_as_float(b[i] & 0xffff0000u);
      }
    }
    const float logit = wave_sum(acc);  // identical in every lane
    // insert into the sorted selection (descending logit, ascending index on ties)
    float v = logit;
    int idx = e;
#pragma unroll
    for (int k = 0; k < MAX_K; ++k) {
      if (k < K && (v > sel_v[k] || (v == sel_v[k] && idx < sel_i[k]))) {
        const float tv = sel_v[k];
        const int ti = sel_i[k];
        sel_v[k] = v;
        sel_i[k] = idx;
        v = tv;
        idx = ti;
      }
    }
  }
  if (lane == 0) {
    float p[MAX_K], sum = 0.f;
#pragma unroll
    for (int k = 0; k < MAX_K; ++k) {
      p[k] = k < K ? expf(sel_v[k] - sel_v[0]) : 0.f;
      sum += p[k];
    }
#pragma unroll
    for (int k = 0; k < MAX_K; ++k) {
      if (k < K) {
        ids[(size_t)t * K + k] = sel_i[k];
        wts[(size_t)t * K + k] = p[k] / sum;
      }
    }
  }
}

// Stable counting sort of the rows (t, k), t in [tok_begin, tok_end), by expert.  One
// workgroup; row r = (t - tok_begin) * K + k.  Outputs (all relative to the global row
// space, rows of this range start at tok_begin * K):
//   expert_offset[e]  first sorted row of expert e (expert_offset[E] = end)
//   row_token[pos]    token whose activations row `pos` multiplies
//   slot_of[t*K + k]  sorted position of row (t, k)
__global__ __launch_bounds__(1024) void moe_scatter_kernel(const int32_t* __restrict__ ids, int tok_begin, int tok_end,
                                                           int E, int K, int32_t* __restrict__ expert_offset,
                                                           int32_t* __restrict__ row_token,
                                                           int32_t* __restrict__ slot_of) {
  __shared__ int scan[1024];
  __shared__ int base_e;
  const int n_rows = (tok_end - tok_begin) * K;
  const int row0 = tok_begin * K;
  const int tid = threadIdx.x;
  const int per = (n_rows + 1023) / 1024;  // consecutive rows per thread keeps the sort stable
  const int lo = tid * per, hi = min(n_rows, lo + per);
  if (tid == 0) base_e = row0;
  __syncthreads();
  for (int e = 0; e < E; ++e) {
    int cnt = 0;
    for (int r = lo; r < hi; ++r) cnt += (ids[row0 + r] == e);
    scan[tid] = cnt;
    __syncthreads();
    // inclusive Hillis-Steele scan over the 1024 per-thread counts
    for (int off = 1; off < 1024; off <<= 1) {
      const int v = tid >= off ? scan[tid - off] : 0;
      __syncthreads();
      scan[tid] += v;
      __syncthreads();
    }
    const int base = base_e;
    int pos = base + scan[tid] - cnt;
    for (int r = lo; r < hi; ++r) {
      if (ids[row0 + r] == e) {
        row_token[pos] = tok_begin + r / K;
        slot_of[row0 + r] = pos;
        ++pos;
      }
    }
    const int total = scan[1023];
    __syncthreads();
    if (tid == 0) {
      expert_offset[e] = base;
      base_e = base + total;
      if (e == E - 1) expert_offset[E] = base + total;
    }
    __syncthreads();
  }
}

// z[t] = y[t] + sum_k w[t,k] * expert_out[slot_of[t,k]], summed in k order (fp32).
// PARTIAL: an expert's output row is given as the fp32 sums of the two halves of its down
// projection's K (p0, p1) and is bf16(p0 + p1) - the value a two-segment dense operation stores.
template <bool PARTIAL>
__global__ __launch_bounds__(256) void moe_combine_kernel(const bf16_t* __restrict__ y, const bf16_t* __restrict__ eo,
                                                          const float* __restrict__ p0, const float* __restrict__ p1,
                                                          const int32_t* __restrict__ slot_of,
                                                          const float* __restrict__ wts, bf16_t* __restrict__ z,
                                                          int tok_begin, int D, int K) {
  const int t = tok_begin + blockIdx.x;
  for (int v = threadIdx.x; v < (D >> 3); v += 256) {
    const u32x4 yy = *reinterpret_cast<const u32x4*>(y + (size_t)t * D + v * 8);
    float acc[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[2 * i] = __uint_as_float(yy[i] << 16);
      acc[2 * i + 1] = __uint_as_float(yy[i] & 0xffff0000u);
    }
    for (int k = 0; k < K; ++k) {
      const float w = wts[(size_t)t * K + k];
      const size_t row = (size_t)slot_of[(size_t)t * K + k] * D + v * 8;
      if (PARTIAL) {
        const f32x4 a0 = *reinterpret_cast<const f32x4*>(p0 + row), a1 = *reinterpret_cast<const f32x4*>(p0 + row + 4);
        const f32x4 b0 = *reinterpret_cast<const f32x4*>(p1 + row), b1 = *reinterpret_cast<const f32x4*>(p1 + row + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[i] += w * bf2f(f2bf(a0[i] + b0[i]));
          acc[4 + i] += w * bf2f(f2bf(a1[i] + b1[i]));
        }
      } else {
        const u32x4 ee = *reinterpret_cast<const u32x4*>(eo + row);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[2 * i] += w * __uint_as_float(ee[i] << 16);
          acc[2 * i + 1] += w * __uint_as_float(ee[i] & 0xffff0000u);
        }
      }
    }
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = pack_bf2(acc[2 * i], acc[2 * i + 1]);
    *reinterpret_cast<u32x4*>(z + (size_t)t * D + v * 8) = o;
  }
}

}  // namespace

hipError_t nf_launch_moe_router(const void* h, const void* w_router, int32_t* expert_ids, float* expert_w,
                                int tok_begin, int tok_end, int hidden, int n_experts, int top_k, hipStream_t s) {
  const int n = tok_end - tok_begin;
  if (n <= 0) return hipSuccess;
  if (n_experts > MAX_E || top_k > MAX_K) return hipErrorInvalidValue;
  moe_router_kernel<<<dim3((n + 3) / 4), dim3(256), 0, s>>>((const bf16_t*)h, (const bf16_t*)w_router, expert_ids,
                                                           expert_w, tok_begin, tok_end, hidden, n_experts, top_k);
  return hipGetLastError();
}

hipError_t nf_launch_moe_scatter(const int32_t* expert_ids, int tok_begin, int tok_end, int n_experts, int top_k,
                                 int32_t* expert_offset, int32_t* row_token, int32_t* slot_of, hipStream_t s) {
  if (tok_end <= tok_begin) return hipSuccess;
  moe_scatter_kernel<<<dim3(1), dim3(1024), 0, s>>>(expert_ids, tok_begin, tok_end, n_experts, top_k, expert_offset,
                                                   row_token, slot_of);
  return hipGetLastError();
}

hipError_t nf_launch_moe_combine(const void* y, const void* expert_out, const int32_t* slot_of, const float* expert_w,
                                 void* z, int tok_begin, int tok_end, int hidden, int top_k, hipStream_t s,
                                 const float* expert_partial, long long seg_stride) {
  if (tok_end <= tok_begin) return hipSuccess;
  if (expert_partial)
    moe_combine_kernel<true><<<dim3(tok_end - tok_begin), dim3(256), 0, s>>>(
        (const bf16_t*)y, nullptr, expert_partial, expert_partial + seg_stride, slot_of, expert_w, (bf16_t*)z,
        tok_begin, hidden, top_k);
  else
    moe_combine_kernel<false><<<dim3(tok_end - tok_begin), dim3(256), 0, s>>>(
        (const bf16_t*)y, (const bf16_t*)expert_out, nullptr, nullptr, slot_of, expert_w, (bf16_t*)z, tok_begin,
        hidden, top_k);
  return hipGetLastError();
}
