// The ends of the iteration loop around the decoder layers (paper Sec. 2.1 / Fig. 1: tokens
// enter through an embedding and leave through the LM head and sampling; Sec. 2.2 lists these
// among the "other operations"): embedding / row gather, and greedy sampling (argmax).
#include <math.h>

#include "nf_device.h"
#include "nf_kernels.h"

namespace {

// out[t] = table[id(t)] with id(t) = slot_tokens[from_slot[t]] when from_slot[t] >= 0 (a decode
// token: the token the previous iteration sampled for that request, still on the device) and
// token_ids[t] otherwise.  Ids outside the table are clamped.  One workgroup per row.
__global__ __launch_bounds__(256) void gather_rows_kernel(const int32_t* __restrict__ token_ids,
                                                          const int32_t* __restrict__ from_slot,
                                                          const int32_t* __restrict__ slot_tokens,
                                                          const bf16_t* __restrict__ table, int n_rows_table,
                                                          bf16_t* __restrict__ out, int width) {
  const int t = blockIdx.x;
  int id = token_ids[t];
  if (from_slot && from_slot[t] >= 0) id = slot_tokens[from_slot[t]];
  id = id < 0 ? 0 : (id >= n_rows_table ? n_rows_table - 1 : id);
  const u32x4* src = reinterpret_cast<const u32x4*>(table + (size_t)id * width);
  u32x4* dst = reinterpret_cast<u32x4*>(out + (size_t)t * width);
  for (int c = threadIdx.x; c < width / 8; c += 256) dst[c] = src[c];
}

// Greedy sampling: index of the largest logit of each row, the lowest index among equal ones.
// One workgroup per row; out[out_index ? out_index[r] : r] = argmax.
__global__ __launch_bounds__(256) void argmax_kernel(const bf16_t* __restrict__ logits, int vocab,
                                                     const int32_t* __restrict__ out_index,
                                                     int32_t* __restrict__ out) {
  const int r = blockIdx.x;
  const bf16_t* row = logits + (size_t)r * vocab;
  float best = -INFINITY;
  int best_i = 0x7fffffff;
  for (int c = threadIdx.x; c < vocab / 8; c += 256) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(row + c * 8);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = __uint_as_float(v[e] << 16), hi = __uint_as_float(v[e] & 0xffff0000u);
      const int i = c * 8 + 2 * e;
      if (lo > best) {  // indices grow within a thread: ">" keeps the first of equal values
        best = lo;
        best_i = i;
      }
      if (hi > best) {
        best = hi;
        best_i = i + 1;
      }
    }
  }
  if (best_i == 0x7fffffff) best_i = 0;  // a row of NaN or -inf only
  __shared__ float sv[256];
  __shared__ int si[256];
  sv[threadIdx.x] = best;
  si[threadIdx.x] = best_i;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      const float ov = sv[threadIdx.x + s];
      const int oi = si[threadIdx.x + s];
      if (ov > sv[threadIdx.x] || (ov == sv[threadIdx.x] && oi < si[threadIdx.x])) {
        sv[threadIdx.x] = ov;
        si[threadIdx.x] = oi;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) out[out_index ? out_index[r] : r] = si[0];
}

}  // namespace

hipError_t nf_launch_gather_rows(const int32_t* token_ids, const int32_t* from_slot, const int32_t* slot_tokens,
                                 const void* table, int n_rows_table, void* out, int n_rows, int width,
                                 hipStream_t s) {
  if (n_rows <= 0) return hipSuccess;
  gather_rows_kernel<<<dim3(n_rows), dim3(256), 0, s>>>(token_ids, from_slot, slot_tokens, (const bf16_t*)table,
                                                        n_rows_table, (bf16_t*)out, width);
  return hipGetLastError();
}

hipError_t nf_launch_argmax(const void* logits, int n_rows, int vocab, const int32_t* out_index, int32_t* out,
                            hipStream_t s) {
  if (n_rows <= 0) return hipSuccess;
  argmax_kernel<<<dim3(n_rows), dim3(256), 0, s>>>((const bf16_t*)logits, vocab, out_index, out);
  return hipGetLastError();
}
