// Measured ceilings of the device the library runs on, for pricing the kernels against
// what the chip delivers rather than against its data sheet: a register-only bf16 MFMA
// loop (all-zero and varied operands: the second is the power-limited rate activation-like
// data allows) and a streaming read of a buffer far larger than the caches.
#include <algorithm>
#include <new>

#include "nf_device.h"
#include "nf_internal.h"

namespace {

__device__ __forceinline__ uint32_t mix32(uint32_t h) {
  h ^= h >> 16;
  h *= 0x7FEB352Du;
  h ^= h >> 15;
  h *= 0x846CA68Bu;
  h ^= h >> 16;
  return h;
}

// 8 wavefronts per CU, each issuing independent 32x32x16 MFMAs from registers.
// varied = 0: all-zero operands; 1: 8 operand pairs of pseudo-random bf16 values near 1.
__global__ __launch_bounds__(256) void mfma_loop_kernel(float* __restrict__ out, int iters, int varied) {
  bf16x8 fa[8], fb[8];
  const uint32_t id = blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    u32x4 a, b;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t ha = mix32(id * 64 + i * 8 + e), hb = mix32(id * 64 + i * 8 + e + 4);
      a[e] = varied ? ((ha & 0x807f807fu) | 0x3f003f00u | ((ha >> 3) & 0x00800080u)) : 0u;
      b[e] = varied ? ((hb & 0x807f807fu) | 0x3c003c00u | ((hb >> 3) & 0x00800080u)) : 0u;
    }
    fa[i] = __builtin_bit_cast(bf16x8, a);
    fb[i] = __builtin_bit_cast(bf16x8, b);
  }
  f32x16 acc0 = {0}, acc1 = {0}, acc2 = {0}, acc3 = {0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[i], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i + 1], fb[i], acc1, 0, 0, 0);
      acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[i + 1], acc2, 0, 0, 0);
      acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i + 1], fb[i + 1], acc3, 0, 0, 0);
    }
  }
  const float r = acc0[0] + acc1[1] + acc2[2] + acc3[3];
  if (r == 1.2345f) out[threadIdx.x] = r;  // keeps the loop alive; never true in practice
}

// Persistent workgroups stream the buffer once with 16-byte loads, 8 KiB per wavefront step.
__global__ __launch_bounds__(256) void stream_read_kernel(const char* __restrict__ buf, size_t n_steps,
                                                          uint32_t* __restrict__ out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t n_waves = (size_t)gridDim.x * 4;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t step = (size_t)blockIdx.x * 4 + wave; step < n_steps; step += n_waves) {
    const char* p = buf + step * 8192 + lane * 16;
    u32x4 r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + j * 1024));
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= r[j];
  }
  if (acc[0] == 0x1234567u) out[threadIdx.x] = acc[1];  // never true for the zero-filled buffer
}

}  // namespace

extern "C" int nf_measure_peaks(nf_ctx* ctx, nf_peaks* out) try {
  if (!ctx || !out) return NF_EINVAL;
  NF_HIP(ctx, hipSetDevice(ctx->device));
  hipDeviceProp_t prop;
  NF_HIP(ctx, hipGetDeviceProperties(&prop, ctx->device));
  const int n_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  const size_t bytes = (size_t)4 << 30;  // 4 GiB: sixteen times the last-level cache
  char* buf = nullptr;
  float* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = NF_OK;
  auto fail = [&](hipError_t e) {
    if (e != hipSuccess && rc == NF_OK) {
      ctx->last_hip = (int)e;
      rc = NF_EHIP;
    }
    return e != hipSuccess;
  };
  if (!fail(hipMalloc(&buf, bytes)) && !fail(hipMalloc(&sink, 4096)) && !fail(hipMemset(buf, 0, bytes)) &&
      !fail(hipEventCreate(&e0)) && !fail(hipEventCreate(&e1))) {
    float ms = 0.f;
    // ---- matrix cores: zero operands, then varied operands ----
    const int iters = 100000;  // 16 MFMAs of 32768 flop per iteration and wavefront
    const dim3 grid_m(n_cus * 2), block(256);
    double tf[2] = {0, 0};
    for (int varied = 0; varied < 2 && rc == NF_OK; ++varied) {
      mfma_loop_kernel<<<grid_m, block>>>(sink, 1000, varied);
      fail(hipGetLastError());
      fail(hipDeviceSynchronize());
      fail(hipEventRecord(e0, nullptr));
      mfma_loop_kernel<<<grid_m, block>>>(sink, iters, varied);
      fail(hipGetLastError());
      fail(hipEventRecord(e1, nullptr));
      fail(hipEventSynchronize(e1));
      fail(hipEventElapsedTime(&ms, e0, e1));
      tf[varied] = (double)grid_m.x * 4 * iters * 16 * 32768.0 / ((double)ms * 1e-3) / 1e12;
    }
    out->mfma_bf16_tflops_zero_operands = tf[0];
    out->mfma_bf16_tflops = tf[1];
    // ---- HBM: best of three streaming reads ----
    double best = 0;
    for (int rep = 0; rep < 4 && rc == NF_OK; ++rep) {
      fail(hipEventRecord(e0, nullptr));
      stream_read_kernel<<<dim3(n_cus * 2), block>>>(buf, bytes / 8192, (uint32_t*)sink);
      fail(hipGetLastError());
      fail(hipEventRecord(e1, nullptr));
      fail(hipEventSynchronize(e1));
      fail(hipEventElapsedTime(&ms, e0, e1));
      if (rep > 0 && ms > 0) best = std::max(best, (double)bytes / ((double)ms * 1e-3) / 1e9);
    }
    out->hbm_read_gbs = best;
    out->n_cus = n_cus;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (buf) (void)hipFree(buf);
  if (sink) (void)hipFree(sink);
  return rc;
} catch (const std::bad_alloc&) {
  return NF_ENOMEM;
} catch (...) {
  return NF_EINVAL;
}

// ---- interference probe: latency of cache-resident loads (Sec. 4.1.1 profiles how kernels
// disturb one another; this measures what a GEMM's operand loads wait for while another kernel
// streams from HBM) ------------------------------------------------------------------------
namespace {

constexpr uint32_t kChaseLines = 2048;  // 256 KiB of 128-byte lines: misses the 32 KiB L1, fits any L2
static __device__ __align__(256) uint32_t chase_buf[kChaseLines * 32];

// Every word of line i holds the word index of the line that follows i in one cycle through
// all lines (an odd multiplier modulo a power of two walks every line before it repeats).
__global__ void chase_init_kernel(uint32_t* __restrict__ buf) {
  const uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= kChaseLines * 32) return;
  const uint32_t line = w / 32;
  buf[w] = ((line * 1229u + 977u) & (kChaseLines - 1)) * 32u;
}

// One wavefront per workgroup; lane 0 follows the chain with device-scope loads (they bypass
// the per-CU cache), everything else idles.  out[2b] = nanoseconds per load of workgroup b,
// out[2b + 1] = the hardware id register of the CU it ran on.
__global__ __launch_bounds__(64) void chase_kernel(const uint32_t* __restrict__ buf, int iters,
                                                   float* __restrict__ out) {
  uint32_t idx = ((blockIdx.x * 131u + 7u) & (kChaseLines - 1)) * 32u;
  for (int i = 0; i < 64; ++i) idx = __hip_atomic_load(buf + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned long long t0 = wall_clock64();
  if (threadIdx.x == 0)
    for (int i = 0; i < iters; ++i) idx = __hip_atomic_load(buf + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned long long t1 = wall_clock64();
  if (threadIdx.x == 0) {
    uint32_t hw;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    // wall_clock64 ticks at 100 MHz; idx enters the result so that the chain cannot be dropped
    out[2 * blockIdx.x] = (float)(t1 - t0) * 10.0f / (float)iters + (idx == 0xffffffffu ? 1.0f : 0.0f);
    out[2 * blockIdx.x + 1] = __uint_as_float(hw);
  }
}

}  // namespace

extern "C" int nf_probe_load_latency(nf_ctx* ctx, int n_workgroups, int iters, float* out, void* hip_stream) {
  if (!ctx || !out || n_workgroups < 1 || n_workgroups > 4096 || iters < 1 || iters > (1 << 24)) return NF_EINVAL;
  constexpr int kMaxDevices = 64;
  static uint32_t* per_device[kMaxDevices] = {};
  if (ctx->device < 0 || ctx->device >= kMaxDevices) return NF_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  if (!per_device[ctx->device]) {
    NF_HIP(ctx, hipSetDevice(ctx->device));
    void* p = nullptr;
    NF_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(chase_buf)));
    chase_init_kernel<<<dim3(kChaseLines * 32 / 256), dim3(256), 0, s>>>((uint32_t*)p);
    NF_HIP(ctx, hipGetLastError());
    per_device[ctx->device] = (uint32_t*)p;
  }
  chase_kernel<<<dim3(n_workgroups), dim3(64), 0, s>>>(per_device[ctx->device], iters, out);
  NF_HIP(ctx, hipGetLastError());
  return NF_OK;
}
