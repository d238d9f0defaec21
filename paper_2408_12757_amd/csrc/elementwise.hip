// Row-wise "other operations" of the decoder layer (paper Sec. 2.2): RMSNorm,
// and rotary position embedding fused with the KV-cache append (Sec. 2.1: Key
// and Value are concatenated into the existing KV cache).
#include <algorithm>

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
// rotated by pos * theta^(-2i/dh).  The frequencies come from the host in double; the
// angle is formed and reduced to [-pi, pi] in double (a product, a rounding and two fused
// multiply-adds against a two-term 2 pi), so large positions lose no accuracy, and only the
// reduced angle goes through the single-precision sine and cosine.  Q is rotated in place
// in the qkv buffer; K and V go to their page slot in the operand-ordered block layouts.
struct RopeFreq {
  double f[64];  // theta^(-2i/dh), i < dh/2 <= 64
};

__global__ __launch_bounds__(256) void rope_append_kernel(bf16_t* __restrict__ qkv, bf16_t* __restrict__ pages,
                                                          const int32_t* __restrict__ tok_req,
                                                          const int32_t* __restrict__ q_indptr,
                                                          const int32_t* __restrict__ ctx_len,
                                                          const int32_t* __restrict__ page_indptr,
                                                          const int32_t* __restrict__ page_ids, int tok_begin,
                                                          int Hq, int Hkv, int dh, RopeFreq freq,
                                                          int write_k_back) {
  const int t = tok_begin + blockIdx.x;
  const int r = tok_req[t];
  const int pos = ctx_len[r] + (t - q_indptr[r]);
  const bool lone = q_indptr[r + 1] - q_indptr[r] == 1;
  const int page = page_ids[page_indptr[r] + (pos >> 4)];
  const int slot = pos & 15;
  const int half = dh >> 1;
  __shared__ float cs[64], sn[64];
  if ((int)threadIdx.x < half) {
    const double angle = (double)pos * freq.f[threadIdx.x];
    const double turns = rint(angle * 0.15915494309189535);  // 1 / (2 pi)
    double red = fma(-turns, 6.283185307179586, angle);
    red = fma(-turns, 2.4492935982947064e-16, red);  // 2 pi - (double)(2 pi)
    float sv, cv;
    sincosf((float)red, &sv, &cv);
    cs[threadIdx.x] = cv;
    sn[threadIdx.x] = sv;
  }
  __syncthreads();
  bf16_t* row = qkv + (size_t)t * ((Hq + 2 * Hkv) * dh);
  bf16_t* kpage = pages + ((size_t)page * 2 + 0) * Hkv * 16 * dh;
  bf16_t* vpage = pages + ((size_t)page * 2 + 1) * Hkv * 16 * dh;
  // one unit = 8 consecutive dimensions i of a head and their partners i + dh/2: 16-byte
  // loads and stores (8 dimensions are also contiguous in the K block)
  const int octets = half >> 3;
  const int n_units = (Hq + Hkv) * octets;
  for (int u = threadIdx.x; u < n_units; u += 256) {
    const int h = u / octets, o = u - h * octets;
    bf16_t* hv = row + h * dh;
    const u32x4 av = *reinterpret_cast<const u32x4*>(hv + 8 * o);
    const u32x4 bv = *reinterpret_cast<const u32x4*>(hv + half + 8 * o);
    u32x4 ra, rb;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a0 = __uint_as_float(av[e] << 16), a1 = __uint_as_float(av[e] & 0xffff0000u);
      const float b0 = __uint_as_float(bv[e] << 16), b1 = __uint_as_float(bv[e] & 0xffff0000u);
      const float c0 = cs[8 * o + 2 * e], s0 = sn[8 * o + 2 * e];
      const float c1 = cs[8 * o + 2 * e + 1], s1 = sn[8 * o + 2 * e + 1];
      ra[e] = pack_bf2(a0 * c0 - b0 * s0, a1 * c1 - b1 * s1);
      rb[e] = pack_bf2(a0 * s0 + b0 * c0, a1 * s1 + b1 * c1);
    }
    if (h < Hq) {
      *reinterpret_cast<u32x4*>(hv + 8 * o) = ra;
      *reinterpret_cast<u32x4*>(hv + half + 8 * o) = rb;
    } else {
      // K block [dh/32][16 keys][32]: dimensions 8o .. 8o+7 are octet o, their partners octet o + dh/16.
      // The page stores of a request's only token (a decode request) are non-temporal: they are
      // partial cache lines that nothing completes, and written back lazily they cost the
      // attention kernel that follows more than they cost here (measured at the 8B layer: 25 us
      // of the layer).  The tokens of a prefill chunk fill lines together and keep plain stores.
      bf16_t* kb = kpage + (size_t)(h - Hq) * 16 * dh;
      const int o2 = octets + o;
      u32x4* ka = reinterpret_cast<u32x4*>(kb + ((o >> 2) * 16 + slot) * 32 + (o & 3) * 8);
      u32x4* kc = reinterpret_cast<u32x4*>(kb + ((o2 >> 2) * 16 + slot) * 32 + (o2 & 3) * 8);
      if (lone) {
        __builtin_nontemporal_store(ra, ka);
        __builtin_nontemporal_store(rb, kc);
      } else {
        *ka = ra;
        *kc = rb;
      }
      if (write_k_back) {  // the offload copy takes the rotated K from the qkv row
        *reinterpret_cast<u32x4*>(hv + 8 * o) = ra;
        *reinterpret_cast<u32x4*>(hv + half + 8 * o) = rb;
      }
    }
  }
  const bf16_t* vrow = row + (Hq + Hkv) * dh;
  for (int e8 = threadIdx.x; e8 < Hkv * dh / 8; e8 += 256) {
    const int e0 = e8 * 8;
    const int h = e0 / dh, d0 = e0 - h * dh;
    const u32x4 vv = *reinterpret_cast<const u32x4*>(vrow + e0);
    // V block [4 g][dh/32][16 c][2][4 keys]: dimension d = (2*quad + hb)*16 + c, key = 4*g + j
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int d = d0 + k;
      const int b = d >> 4, c = d & 15;
      const int off = ((((slot >> 2) * (dh >> 5) + (b >> 1)) * 16 + c) * 2 + (b & 1)) * 4 + (slot & 3);
      const bf16_t val = (bf16_t)((k & 1) ? (vv[k >> 1] >> 16) : (vv[k >> 1] & 0xffffu));
      if (lone)
        __builtin_nontemporal_store(val, &vpage[(size_t)h * 16 * dh + off]);
      else
        vpage[(size_t)h * 16 * dh + off] = val;
    }
  }
}

hipError_t nf_launch_rope_append(void* qkv, void* pages, const int32_t* tok_req, const int32_t* q_indptr,
                                 const int32_t* ctx_len, const int32_t* page_indptr, const int32_t* page_ids,
                                 int tok_begin, int tok_end, int n_q_heads, int n_kv_heads, int head_dim,
                                 float rope_theta, int write_k_back, hipStream_t s) {
  if (tok_end <= tok_begin) return hipSuccess;
  if (head_dim > 128 || head_dim % 16) return hipErrorInvalidValue;
  RopeFreq freq;
  for (int i = 0; i < 64; ++i)
    freq.f[i] = i < head_dim / 2 ? pow((double)rope_theta, -2.0 * (double)i / (double)head_dim) : 0.0;
  rope_append_kernel<<<dim3(tok_end - tok_begin), dim3(256), 0, s>>>(
      (bf16_t*)qkv, (bf16_t*)pages, tok_req, q_indptr, ctx_len, page_indptr, page_ids, tok_begin, n_q_heads,
      n_kv_heads, head_dim, freq, write_k_back);
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

namespace {

// Moves whole KV pages between their scattered places in a pool and a contiguous buffer
// (Sec. 4.2.2, loading and scattering: a request's cache crosses the bus as one contiguous
// copy; on the device its pages are gathered from / scattered to wherever the allocator put
// them).  One 16-byte element per thread and step; ids outside the pool are skipped.
__global__ __launch_bounds__(256) void move_pages_kernel(char* __restrict__ pool, const int32_t* __restrict__ ids,
                                                         int n, long chunks_per_page, long num_pages,
                                                         char* __restrict__ staging, int scatter) {
  const long total = (long)n * chunks_per_page;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
    const long id = ids[i / chunks_per_page];
    if (id < 0 || id >= num_pages) continue;
    u32x4* in_pool = reinterpret_cast<u32x4*>(pool) + id * chunks_per_page + i % chunks_per_page;
    u32x4* in_line = reinterpret_cast<u32x4*>(staging) + i;
    if (scatter)
      *in_pool = *in_line;
    else
      *in_line = *in_pool;
  }
}

// Copies the K and V part of the qkv rows of tokens [tok_begin, tok_begin + n_tok) to rows
// tok_begin.. of a host buffer the device can write (Sec. 4.2.2: the fresh K/V vectors are
// contiguous right after KQV generation and leave the GPU through a copy the GPU itself
// issues).  One 16-byte store per thread.
__global__ __launch_bounds__(256) void kv_offload_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ host,
                                                         int tok_begin, int n_tok, int n_qkv, int kv_first,
                                                         int row_elems) {
  const int chunks = row_elems / 8;
  const long total = (long)n_tok * chunks;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
    const int t = tok_begin + (int)(i / chunks), c = (int)(i % chunks);
    const u32x4 v = *reinterpret_cast<const u32x4*>(qkv + (size_t)t * n_qkv + kv_first + c * 8);
    *reinterpret_cast<u32x4*>(host + (size_t)t * row_elems + c * 8) = v;
  }
}

}  // namespace

// How the offload rows leave the GPU.  Measured on the 8B layer (8 MB per layer): the copy
// kernel below, although bound by the host link and limited to 64 workgroups, slows the dense
// kernel it runs beside by 120 us (the O projection: 198 instead of 78 us; its waves stall the
// memory pipeline of the CUs they sit on) - 5.6 % of the layer; a strided copy on the copy
// engines costs 0.3 - 1 %.
static int g_offload_dma = 1;
void nf_set_offload_dma(int v) { g_offload_dma = v; }

hipError_t nf_launch_kv_offload(const void* qkv, void* host_rows, int tok_begin, int tok_end, int n_q_heads,
                                int n_kv_heads, int head_dim, hipStream_t s) {
  if (tok_end <= tok_begin) return hipSuccess;
  const int row_elems = 2 * n_kv_heads * head_dim;
  const int n_qkv = (n_q_heads + 2 * n_kv_heads) * head_dim;
  if (g_offload_dma) {
    // a strided copy on the copy engines: rows of row_elems elements, n_qkv apart in the qkv buffer
    const char* src = (const char*)qkv + ((size_t)tok_begin * n_qkv + (size_t)n_q_heads * head_dim) * 2;
    char* dst = (char*)host_rows + (size_t)tok_begin * row_elems * 2;
    return hipMemcpy2DAsync(dst, (size_t)row_elems * 2, src, (size_t)n_qkv * 2, (size_t)row_elems * 2,
                            (size_t)(tok_end - tok_begin), hipMemcpyDeviceToHost, s);
  }
  const long total = (long)(tok_end - tok_begin) * (row_elems / 8);
  // a small grid on purpose: the copy is bound by the host link, not by the GPU
  const int blocks = (int)std::min<long>(64, (total + 255) / 256);
  kv_offload_kernel<<<dim3(blocks), dim3(256), 0, s>>>((const bf16_t*)qkv, (bf16_t*)host_rows, tok_begin,
                                                       tok_end - tok_begin, n_qkv, n_q_heads * head_dim, row_elems);
  return hipGetLastError();
}

hipError_t nf_launch_move_pages(void* pool, size_t page_bytes, long num_pages, const int32_t* page_ids, int n,
                                void* staging, int scatter, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const long chunks = (long)(page_bytes / 16);
  const long total = (long)n * chunks;
  const int blocks = (int)std::min<long>(4096, (total + 255) / 256);
  move_pages_kernel<<<dim3(blocks), dim3(256), 0, s>>>((char*)pool, page_ids, n, chunks, num_pages, (char*)staging,
                                                       scatter);
  return hipGetLastError();
}
