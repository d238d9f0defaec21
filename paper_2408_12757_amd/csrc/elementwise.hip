// Row-wise "other operations" of the decoder layer (paper Sec. 2.2): RMSNorm,
// and rotary position embedding fused with the KV-cache append (Sec. 2.1: Key
// and Value are concatenated into the existing KV cache).
#include "nf_device.h"
#include "nf_kernels.h"

// ---------------------------------------------------------------- RMSNorm ---
// One workgroup per token row.  fp32 statistics; out = (x * rstd) * g.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ g,
                                                      bf16_t* __restrict__ out, int hidden, float eps) {
  const int row = blockIdx.x;
  const bf16_t* xr = x + (size_t)row * hidden;
  bf16_t* orow = out + (size_t)row * hidden;
  __shared__ float red[4];
  float ss = 0.f;
  const int nvec = hidden >> 3;
  for (int v = threadIdx.x; v < nvec; v += 256) {
    u32x4 p = *reinterpret_cast<const u32x4*>(xr + v * 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float a = __uint_as_float(p[i] << 16), b = __uint_as_float(p[i] & 0xffff0000u);
      ss += a * a;
      ss += b * b;
    }
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = (red[0] + red[1]) + (red[2] + red[3]);
  const float rstd = rsqrtf(tot / (float)hidden + eps);
  for (int v = threadIdx.x; v < nvec; v += 256) {
    u32x4 p = *reinterpret_cast<const u32x4*>(xr + v * 8);
    u32x4 gg = *reinterpret_cast<const u32x4*>(g + v * 8);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float a = __uint_as_float(p[i] << 16), b = __uint_as_float(p[i] & 0xffff0000u);
      float ga = __uint_as_float(gg[i] << 16), gb = __uint_as_float(gg[i] & 0xffff0000u);
      o[i] = pack_bf2(a * rstd * ga, b * rstd * gb);
    }
    *reinterpret_cast<u32x4*>(orow + v * 8) = o;
  }
}

hipError_t nf_launch_rmsnorm(const void* x, const void* g, void* out, int n_tokens, int hidden, float eps,
                             hipStream_t s) {
  if (n_tokens <= 0) return hipSuccess;
  rmsnorm_kernel<<<dim3(n_tokens), dim3(256), 0, s>>>((const bf16_t*)x, (const bf16_t*)g, (bf16_t*)out, hidden, eps);
  return hipGetLastError();
}

// ------------------------------------------------- rotary embedding + append ---
// One workgroup per token.  The pair (i, i + dh/2) of every Q and K head is
// rotated by pos * theta^(-2i/dh); the angle is formed in double so that large
// positions lose no accuracy.  Q is rotated in place in the qkv buffer; K and V go to
// their page slot in the operand-ordered block layouts.
__global__ __launch_bounds__(256) void rope_append_kernel(bf16_t* __restrict__ qkv, bf16_t* __restrict__ pages,
                                                          const int32_t* __restrict__ tok_req,
                                                          const int32_t* __restrict__ q_indptr,
                                                          const int32_t* __restrict__ ctx_len,
                                                          const int32_t* __restrict__ page_indptr,
                                                          const int32_t* __restrict__ page_ids, int tok_begin,
                                                          int Hq, int Hkv, int dh, float theta) {
  const int t = tok_begin + blockIdx.x;
  const int r = tok_req[t];
  const int pos = ctx_len[r] + (t - q_indptr[r]);
  const int page = page_ids[page_indptr[r] + (pos >> 4)];
  const int slot = pos & 15;
  const int half = dh >> 1;
  __shared__ float cs[64], sn[64];
  if ((int)threadIdx.x < half) {
    const double freq = exp2(-2.0 * (double)threadIdx.x / (double)dh * log2((double)theta));
    double sv, cv;
    sincos((double)pos * freq, &sv, &cv);
    cs[threadIdx.x] = (float)cv;
    sn[threadIdx.x] = (float)sv;
  }
  __syncthreads();
  bf16_t* row = qkv + (size_t)t * ((Hq + 2 * Hkv) * dh);
  bf16_t* kpage = pages + ((size_t)page * 2 + 0) * Hkv * 16 * dh;
  bf16_t* vpage = pages + ((size_t)page * 2 + 1) * Hkv * 16 * dh;
  const int n_pairs = (Hq + Hkv) * half;
  for (int p = threadIdx.x; p < n_pairs; p += 256) {
    const int h = p / half, i = p - h * half;
    bf16_t* hv = row + h * dh;
    const float a = bf2f(hv[i]), b = bf2f(hv[i + half]);
    const float c = cs[i], s = sn[i];
    const bf16_t ra = f2bf(a * c - b * s), rb = f2bf(a * s + b * c);
    if (h < Hq) {
      hv[i] = ra;
      hv[i + half] = rb;
    } else {
      // K block [dh/8][16 keys][8]
      bf16_t* kb = kpage + (size_t)(h - Hq) * 16 * dh;
      const int j = i + half;
      kb[((i >> 3) * 16 + slot) * 8 + (i & 7)] = ra;
      kb[((j >> 3) * 16 + slot) * 8 + (j & 7)] = rb;
    }
  }
  const bf16_t* vrow = row + (Hq + Hkv) * dh;
  for (int e = threadIdx.x; e < Hkv * dh; e += 256) {
    const int h = e / dh, d = e - h * dh;
    // V block [dh/32][16 c][4 g][2][4 keys]: dimension d = (2*quad + hb)*16 + c, key = 4*g + j
    const int b = d >> 4, c = d & 15;
    const int off = ((((b >> 1) * 16 + c) * 4 + (slot >> 2)) * 2 + (b & 1)) * 4 + (slot & 3);
    vpage[(size_t)h * 16 * dh + off] = vrow[e];
  }
}

hipError_t nf_launch_rope_append(void* qkv, void* pages, const int32_t* tok_req, const int32_t* q_indptr,
                                 const int32_t* ctx_len, const int32_t* page_indptr, const int32_t* page_ids,
                                 int tok_begin, int tok_end, int n_q_heads, int n_kv_heads, int head_dim,
                                 float rope_theta, hipStream_t s) {
  if (tok_end <= tok_begin) return hipSuccess;
  rope_append_kernel<<<dim3(tok_end - tok_begin), dim3(256), 0, s>>>(
      (bf16_t*)qkv, (bf16_t*)pages, tok_req, q_indptr, ctx_len, page_indptr, page_ids, tok_begin, n_q_heads,
      n_kv_heads, head_dim, rope_theta);
  return hipGetLastError();
}

namespace {

// Pseudo-random bf16 values, roughly normal with the given standard deviation: the sum of
// the four bytes of a hashed counter.  Only for timing buffers: dense kernels on this chip
// run measurably slower on varied data than on constant data, so profiling inputs must
// look like activations and weights.
__global__ __launch_bounds__(256) void fill_random_kernel(bf16_t* __restrict__ p, size_t n, uint32_t seed,
                                                          float stddev) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    uint32_t h = (uint32_t)i * 0x9E3779B9u + (uint32_t)(i >> 32) + seed;
    h ^= h >> 16;
    h *= 0x7FEB352Du;
    h ^= h >> 15;
    h *= 0x846CA68Bu;
    h ^= h >> 16;
    const int sum = (int)(h & 255) + (int)((h >> 8) & 255) + (int)((h >> 16) & 255) + (int)(h >> 24);
    p[i] = f2bf((float)(sum - 510) * (1.0f / 147.8f) * stddev);
  }
}

}  // namespace

hipError_t nf_launch_fill_random(void* p, size_t n_elems, uint32_t seed, float stddev, hipStream_t s) {
  if (n_elems == 0) return hipSuccess;
  const size_t want = (n_elems + 255) / 256;
  fill_random_kernel<<<dim3((unsigned)(want < 4096 ? want : 4096)), dim3(256), 0, s>>>((bf16_t*)p, n_elems, seed,
                                                                                        stddev);
  return hipGetLastError();
}
