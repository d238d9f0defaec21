// Dense operations with direct global -> LDS loads (global_load_lds_dwordx4 on gfx950).
//
// Same contract and the same arithmetic as gemm.hip (v_mfma_f32_32x32x16_bf16, K walked in
// steps of 64 in ascending order, transposed product, shared epilogues), hence the same
// output bits.  What differs is how the x and w tiles reach LDS: each wavefront instruction
// moves 64 x 16 bytes from global memory straight into 1 KiB of LDS (the destination is
// wave-uniform base + 16 * lane), so no VGPR holds data in flight, there is no ds_write
// burst before the barrier, and an LDS ring of STAGES tiles keeps STAGES - 1 K-steps of
// loads in flight.
//
// LDS layout: a tile row is 128 contiguous bytes (8 chunks of 16 bytes), rows are not padded
// (a wavefront instruction fills 8 whole rows); bank conflicts are avoided by storing global
// chunk c of row r in slot c ^ ((r >> 1) & 7) - the lane picks its global address accordingly -
// and reading fragments through the same XOR.  A 16-byte fragment read is served 16 lanes
// (16 consecutive rows, one chunk) at a time from 256 bytes of banks: two adjacent rows fill
// the two halves of that window, so the slot must vary with r >> 1.  Measured: 179 B/clk/CU
// against 119 with the XOR taken from r & 7 (two-way conflicts) and 172 with rows padded to
// 144 bytes.
#include <algorithm>
#include <utility>

#include "gemm_common.h"
#include "nf_kernels.h"

namespace {

using namespace nfgemm;

typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  if (N == 0)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// LDS fragment read the compiler does not see as a memory access: it then adds no wait of
// its own for the LDS-DMA loads still in flight into OTHER stages of the ring (it cannot
// tell the stages apart and would wait for all of them).  Completion is awaited explicitly.
__device__ __forceinline__ bf16x8 lds_read_frag(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return __builtin_bit_cast(bf16x8, v);
}

template <int OFFSET>
__device__ __forceinline__ bf16x8 lds_read_frag_at(uint32_t addr) {
  static_assert(OFFSET >= 0 && OFFSET < 65536, "immediate offset of a DS instruction");
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET) : "memory");
  return __builtin_bit_cast(bf16x8, v);
}
// dst[i] = the fragment at addr + BASE + i * STRIDE (immediate offsets: no address arithmetic)
template <int BASE, int STRIDE, int N, int... I>
__device__ __forceinline__ void lds_read_frags(bf16x8 (&dst)[N], uint32_t addr, std::integer_sequence<int, I...>) {
  ((dst[I] = lds_read_frag_at<BASE + I * STRIDE>(addr)), ...);
}
template <int OFFSET>
__device__ __forceinline__ void lds_write_at(uint32_t addr, const u32x4& v) {
  static_assert(OFFSET >= 0 && OFFSET < 65536, "immediate offset of a DS instruction");
  asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(OFFSET) : "memory");
}

// Waits until at most N LDS operations of this wavefront are outstanding; the fragments are
// passed through so that their uses are ordered after the wait.
template <int N, int TN, int TM>
__device__ __forceinline__ void wait_frags(bf16x8 (&fw)[TN], bf16x8 (&fx)[TM]) {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
#pragma unroll
  for (int i = 0; i < TN; ++i) asm volatile("" : "+v"(fw[i]));
#pragma unroll
  for (int j = 0; j < TM; ++j) asm volatile("" : "+v"(fx[j]));
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int STAGES, bool GROUPED, bool PIPE = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_dl_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, bf16_t* __restrict__ Y, const bf16_t* __restrict__ R,
    int M, int N, int K, int tiles_m, int tiles_n, GroupedArgs grp, KRange kr) {
  constexpr int NW = WAVES_M * WAVES_N;              // wavefronts per workgroup
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wavefront tile
  constexpr int TM = WM / 32, TN = WN / 32;          // 32x32 MFMA tiles per wavefront
  constexpr int ROWS = BM + BN;                      // tile rows per stage: x rows, then w rows
  constexpr int LOADS = ROWS / 8 / NW;               // wavefront load instructions per stage
  constexpr int STAGE_BYTES = ROWS * 128;
  static_assert(ROWS % (8 * NW) == 0, "rows must split evenly over the wavefronts");
  static_assert(STAGES >= 2 && STAGES <= 4, "LDS ring depth");
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  int m0, n0;
  size_t w_off;
  if (!locate_tile<BM, BN, GROUPED>(tiles_m, tiles_n, grp, m0, n0, M, w_off)) return;  // before any barrier
  const size_t k_begin = (size_t)blockIdx.y * K;  // this workgroup's K segment
  X += k_begin;
  W += w_off + k_begin;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  // Loader: instruction i of this wavefront fills LDS rows (i*NW + wave)*8 .. +8 of the stage;
  // this lane supplies row +lane/8, slot lane%8, i.e. global chunk (lane%8) ^ ((row >> 1) & 7).
  const bf16_t* src[LOADS];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int row = (i * NW + wave) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    if (row < BM) {
      int gm = m0 + row;
      gm = gm < M ? gm : M - 1;  // rows past M are computed on a copy of the last row and never stored
      if (GROUPED && grp.row_index) gm = grp.row_index[gm];
      src[i] = X + (size_t)gm * kr.ldk + chunk * 8;
    } else {
      src[i] = W + (size_t)weight_row<EPI>(row - BM, n0, N) * kr.ldk + chunk * 8;
    }
  }
  auto issue_stage = [&](int stage, int kt) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(src[i] + (size_t)kt * BK),
                                       (lptr_t)(lds + stage * STAGE_BYTES + (i * NW + wave) * 1024), 16, 0, 0);
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = K / BK;
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < KT) issue_stage(s, s);

  // fragment addressing: row = wave tile base + i*32 + (lane & 31); the k-chunk of slice kk is
  // 2*kk + (lane >> 5), found in slot chunk ^ ((row >> 1) & 7); wave tile bases are multiples of 32
  const int frag_row = lane & 31, swz = (lane >> 1) & 7, g = lane >> 5;
  const int x_off = (wm * WM + frag_row) * 128;
  const int w_off_lds = (BM + wn * WN + frag_row) * 128;

  int stage = 0;
  if (PIPE) {
    // Explicitly scheduled loop: bare barrier, explicit waits, fragments of K-slice kk + 1 read
    // from LDS while the MFMAs of slice kk issue.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lptr_t)lds;
    for (int kt = 0; kt < KT; ++kt) {
      if (kt + STAGES - 2 < KT)
        wait_vmcnt<(STAGES - 2) * LOADS>();
      else
        wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      if (kt + STAGES - 1 < KT) {
        int fill = stage + STAGES - 1;
        if (fill >= STAGES) fill -= STAGES;
        issue_stage(fill, kt + STAGES - 1);
      }
      const uint32_t base = lds_base + stage * STAGE_BYTES;
      bf16x8 fw[2][TN], fx[2][TM];
      {
        const uint32_t slot = ((uint32_t)(g ^ swz)) * 16;
#pragma unroll
        for (int i = 0; i < TN; ++i) fw[0][i] = lds_read_frag(base + w_off_lds + i * 32 * 128 + slot);
#pragma unroll
        for (int j = 0; j < TM; ++j) fx[0][j] = lds_read_frag(base + x_off + j * 32 * 128 + slot);
      }
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        const int cb = kk & 1, nb = cb ^ 1;
        if (kk + 1 < BK / 16) {
          const uint32_t slot = ((uint32_t)((2 * (kk + 1) + g) ^ swz)) * 16;
#pragma unroll
          for (int i = 0; i < TN; ++i) fw[nb][i] = lds_read_frag(base + w_off_lds + i * 32 * 128 + slot);
#pragma unroll
          for (int j = 0; j < TM; ++j) fx[nb][j] = lds_read_frag(base + x_off + j * 32 * 128 + slot);
          wait_frags<TN + TM, TN, TM>(fw[cb], fx[cb]);  // slice kk has arrived; kk + 1 may be in flight
        } else {
          wait_frags<0, TN, TM>(fw[cb], fx[cb]);
        }
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int j = 0; j < TM; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[cb][i], fx[cb][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);  // keep this slice's MFMAs in front of the next slice's waits
      }
      if (++stage == STAGES) stage = 0;
    }
  } else {
  for (int kt = 0; kt < KT; ++kt) {
    // tile kt has landed once at most (STAGES - 2) younger stages of loads are outstanding
    if (kt + STAGES - 2 < KT)
      wait_vmcnt<(STAGES - 2) * LOADS>();
    else
      wait_vmcnt<0>();
    __syncthreads();  // every wavefront's part of tile kt is in LDS; stage (kt - 1) % STAGES is free
    if (kt + STAGES - 1 < KT) {
      int fill = stage + STAGES - 1;
      if (fill >= STAGES) fill -= STAGES;
      issue_stage(fill, kt + STAGES - 1);
    }
    const char* base = lds + stage * STAGE_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int slot = ((2 * kk + g) ^ swz) * 16;
      bf16x8 fw[TN], fx[TM];
#pragma unroll
      for (int i = 0; i < TN; ++i) fw[i] = *reinterpret_cast<const bf16x8*>(base + w_off_lds + i * 32 * 128 + slot);
#pragma unroll
      for (int j = 0; j < TM; ++j) fx[j] = *reinterpret_cast<const bf16x8*>(base + x_off + j * 32 * 128 + slot);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fx[j], acc[i][j], 0, 0, 0);
    }
    if (++stage == STAGES) stage = 0;
  }

  }

  store_tile<EPI, TM, TN, WM, WN>(acc, Y, R, M, N, m0, n0, wm, wn, lane,
                                  kr.partial + (size_t)blockIdx.y * (size_t)kr.seg_stride);
}

// Second main loop: K-step BKT of 32 or 64, an LDS ring of up to 5 stages, and the stage
// barrier moved in front of the last K-slice's MFMAs: a wavefront finishes its LDS reads of
// stage k, waits for its own loads of stage k + 1, meets the others at the barrier, issues
// the fragment reads of stage k + 1 and only then the MFMAs of the last slice of stage k, so
// the matrix pipe has work queued while the barrier and the first fragment reads complete.
// With BKT = 32 a tile row is 64 bytes (4 chunks): 16 lanes read 16 consecutive rows, four
// rows fill the 256-byte bank window, so the slot XOR comes from (row >> 2) & 3.
//
// SEG2: the workgroup sums the two halves of K separately (two accumulator sets) and adds
// the two sums at the end - the arithmetic of a two-segment operation (nf_gemm_k_segments)
// without any scratch memory.
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int STAGES, bool GROUPED, int BKT, bool SEG2 = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_dl2_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, bf16_t* __restrict__ Y, const bf16_t* __restrict__ R,
    int M, int N, int K, int tiles_m, int tiles_n, GroupedArgs grp, KRange kr) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int ROWS = BM + BN;
  constexpr int RB = BKT * 2;     // bytes per tile row
  constexpr int CPR = RB / 16;    // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;   // rows filled by one wavefront load instruction
  constexpr int LOADS = ROWS / RPI / NW;
  constexpr int STAGE_BYTES = ROWS * RB;
  constexpr int SLICES = BKT / 16;
  static_assert(BKT == 32 || BKT == 64, "K-step");
  static_assert(ROWS % (RPI * NW) == 0, "rows must split evenly over the wavefronts");
  static_assert(STAGES >= 2 && STAGES <= 6, "LDS ring depth");
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  int m0, n0;
  size_t w_off;
  if (!locate_tile<BM, BN, GROUPED>(tiles_m, tiles_n, grp, m0, n0, M, w_off)) return;  // before any barrier
  const size_t k_begin = (size_t)blockIdx.y * K;  // this workgroup's K segment
  X += k_begin;
  W += w_off + k_begin;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  auto slot_xor = [](int row) { return CPR == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3); };

  const bf16_t* src[LOADS];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int row = (i * NW + wave) * RPI + lane / CPR;
    const int chunk = (lane % CPR) ^ slot_xor(row);
    if (row < BM) {
      int gm = m0 + row;
      gm = gm < M ? gm : M - 1;  // rows past M are computed on a copy of the last row and never stored
      if (GROUPED && grp.row_index) gm = grp.row_index[gm];
      src[i] = X + (size_t)gm * kr.ldk + chunk * 8;
    } else {
      src[i] = W + (size_t)weight_row<EPI>(row - BM, n0, N) * kr.ldk + chunk * 8;
    }
  }
  auto issue_stage = [&](int stage, int kt) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(src[i] + (size_t)kt * BKT),
                                       (lptr_t)(lds + stage * STAGE_BYTES + (i * NW + wave) * 1024), 16, 0, 0);
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = K / BKT;
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < KT) issue_stage(s, s);

  const int frag_row = lane & 31, g = lane >> 5;
  const uint32_t sx = (uint32_t)slot_xor(frag_row);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lptr_t)lds;
  const uint32_t x_off = (uint32_t)((wm * WM + frag_row) * RB);
  const uint32_t w_off_lds = (uint32_t)((BM + wn * WN + frag_row) * RB);
  bf16x8 fw[2][TN], fx[2][TM];
  auto read_slice = [&](uint32_t base, int kk, bf16x8 (&dw)[TN], bf16x8 (&dx)[TM]) {
    const uint32_t slot = (((uint32_t)(2 * kk + g)) ^ sx) * 16;
#pragma unroll
    for (int i = 0; i < TN; ++i) dw[i] = lds_read_frag(base + w_off_lds + i * 32 * RB + slot);
#pragma unroll
    for (int j = 0; j < TM; ++j) dx[j] = lds_read_frag(base + x_off + j * 32 * RB + slot);
  };

  if (KT >= STAGES - 1)
    wait_vmcnt<(STAGES - 2) * LOADS>();
  else
    wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  read_slice(lds_base, 0, fw[0], fx[0]);

  int stage = 0;
  auto k_step = [&](int kt) {
    // every wavefront has passed the barrier that ended stage kt - 1: its buffer is free
    if (kt + STAGES - 1 < KT) {
      int fill = stage + STAGES - 1;
      if (fill >= STAGES) fill -= STAGES;
      issue_stage(fill, kt + STAGES - 1);
    }
    const uint32_t base = lds_base + stage * STAGE_BYTES;
    int next = stage + 1;
    if (next == STAGES) next = 0;
#pragma unroll
    for (int kk = 0; kk < SLICES; ++kk) {
      const int cb = kk & 1, nb = cb ^ 1;
      if (kk + 1 < SLICES) {
        read_slice(base, kk + 1, fw[nb], fx[nb]);
        wait_frags<TN + TM, TN, TM>(fw[cb], fx[cb]);  // slice kk has arrived; kk + 1 may be in flight
      } else {
        wait_frags<0, TN, TM>(fw[cb], fx[cb]);  // this wavefront's last reads of the stage are done
        if (kt + 1 < KT) {
          if (kt + STAGES - 1 < KT)
            wait_vmcnt<(STAGES - 2) * LOADS>();  // stage kt + 1 has landed; younger stages stay in flight
          else
            wait_vmcnt<0>();
          __builtin_amdgcn_s_barrier();
          read_slice(lds_base + next * STAGE_BYTES, 0, fw[nb], fx[nb]);
        }
      }
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[cb][i], fx[cb][j], acc[i][j], 0, 0, 0);
      // keep this slice's MFMAs in front of the next slice's waits
      __builtin_amdgcn_sched_barrier(0);
    }
    stage = next;
  };

  // SEG2: the loop runs in two parts (the load pipeline runs through); the sums of the first
  // half of K are set aside between them - every MFMA of a K-step is issued inside its step
  f32x16 acc_lo[SEG2 ? TN : 1][SEG2 ? TM : 1];
  const int kt_first = SEG2 ? (KT >> 1) : KT;
  for (int kt = 0; kt < kt_first; ++kt) k_step(kt);
  if (SEG2) {
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j) {
        acc_lo[SEG2 ? i : 0][SEG2 ? j : 0] = acc[i][j];
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
      }
    for (int kt = kt_first; kt < KT; ++kt) k_step(kt);
  }

  if (SEG2) {
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j) acc[i][j] = acc_lo[SEG2 ? i : 0][SEG2 ? j : 0] + acc[i][j];
  }
  store_tile<EPI, TM, TN, WM, WN>(acc, Y, R, M, N, m0, n0, wm, wn, lane,
                                  kr.partial + (size_t)blockIdx.y * (size_t)kr.seg_stride);
}

// Epilogue of the four-wavefront loop for bf16 outputs: the accumulator layout gives a lane 4
// consecutive columns of one row, so direct stores are 8-byte pieces of 32 different rows
// per instruction (measured: 13 us per 256x256 tile, 11 % of the Up/Gate GEMM).  Here each
// wavefront passes its share through its own LDS region (rows padded by 16 bytes) and stores
// whole rows: 16 bytes per lane, 256 contiguous bytes per row.  The residual is brought in
// the same way (coalesced loads into the region, read back in accumulator layout) and added
// in fp32 before the single rounding, exactly as in store_tile.  No workgroup barrier: the
// region is private to the wavefront, and nobody reads the tile stages after the main loop.
template <int EPI, int TM, int TN, int WM, int WN>
__device__ __forceinline__ void store_tile_rows(const f32x16 (&acc)[TN][TM], bf16_t* __restrict__ Y,
                                                const bf16_t* __restrict__ R, int M, int N, int m0, int n0, int wm,
                                                int wn, int lane, uint32_t region) {
  constexpr int WO = EPI == EPI_SWIGLU ? WN / 2 : WN;  // output columns of this wavefront
  constexpr int ROWB = WO * 2 + 16;                     // bytes per LDS row
  constexpr int CPR = WO / 8, RPI = 64 / CPR;           // 16-byte chunks per row, rows per wavefront instruction
  constexpr int PASSES = (WM + RPI - 1) / RPI;          // (96-column shares: 12 chunks, 5 rows, 4 lanes idle)
  const int col0 = EPI == EPI_SWIGLU ? (n0 >> 1) + wn * WO : n0 + wn * WO;
  const int row_lo = m0 + wm * WM;
  const int rr = lane / CPR, kc = lane % CPR;
  const bool lane_on = rr < RPI;
  if (EPI == EPI_RESIDUAL) {
#pragma unroll
    for (int t = 0; t < PASSES; ++t) {
      const int row = t * RPI + rr;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (lane_on && row < WM) {
        if (row_lo + row < M) v = *reinterpret_cast<const u32x4*>(R + (size_t)(row_lo + row) * N + col0 + kc * 8);
        asm volatile("ds_write_b128 %0, %1" ::"v"(region + (uint32_t)(row * ROWB + kc * 16)), "v"(v) : "memory");
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  const uint32_t mine = region + (uint32_t)((lane & 31) * ROWB + (lane >> 5) * 8);
#pragma unroll
  for (int j = 0; j < TM; ++j) {
#pragma unroll
    for (int i = 0; i < (EPI == EPI_SWIGLU ? TN / 2 : TN); ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t addr = mine + (uint32_t)(j * 32 * ROWB + (i * 32 + q * 8) * 2);
        float o[4];
        if (EPI == EPI_SWIGLU) {
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = silu_f(acc[2 * i][j][q * 4 + e]) * acc[2 * i + 1][j][q * 4 + e];
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = acc[i][j][q * 4 + e];
        }
        if (EPI == EPI_RESIDUAL) {
          u32x2 r;
          asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(addr) : "memory");
          o[0] += __uint_as_float(r[0] << 16);
          o[1] += __uint_as_float(r[0] & 0xffff0000u);
          o[2] += __uint_as_float(r[1] << 16);
          o[3] += __uint_as_float(r[1] & 0xffff0000u);
        }
        const u32x2 pk = {pack_bf2(o[0], o[1]), pack_bf2(o[2], o[3])};
        asm volatile("ds_write_b64 %0, %1" ::"v"(addr), "v"(pk) : "memory");
      }
    }
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int t = 0; t < PASSES; ++t) {
    const int row = t * RPI + rr;
    if (lane_on && row < WM) {
      u32x4 v;
      asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(region + (uint32_t)(row * ROWB + kc * 16)) : "memory");
      if (row_lo + row < M) *reinterpret_cast<u32x4*>(Y + (size_t)(row_lo + row) * N + col0 + kc * 8) = v;
    }
  }
}

// Fourth main loop: four wavefronts (one per SIMD), each with a 128x128 share of a 256x256
// tile (256 accumulator registers, the whole register file of its SIMD).  A 128x128
// wavefront tile reads a third less from LDS per flop than the 128x64 tiles of the
// eight-wavefront loops above, whose LDS instructions fill the LDS queues (measured:
// SQ_WAIT_INST_LDS 17 % of the wavefront cycles, the LDS data FIFO full when the tiles are
// written from registers).  The tiles come by direct global -> LDS loads of whole 128-byte
// lines (K-step 64; with 64-byte rows the texture path is busy 1.7x as long for the same
// bytes), two LDS stages of x rows and three of w rows (160 KiB with 256x256 tiles, all the
// LDS of a CU), rows and slot XOR as in the loops at the top of this file.
// One workgroup barrier per K-step, between its second and third K-slice: by then a wavefront
// has all four slices' fragments of K-step k in registers (four fragment buffers) and its
// part of K-step k + 1 has landed; behind the barrier it requests the first two slices of
// K-step k + 1 and issues the loads of the x rows of K-step k + 2 and of the w rows of K-step
// k + 3 - into the stages K-step k has just left - one by one between the MFMAs of slices 2
// and 3.  The w rows so have two K-steps to arrive (measured against two stages of both on one
// device: 2-2.5 % on Up/Gate and KQV, 5 % on O, 6 % on the 70B KQV).  TM = 4: 256x256 tiles; TM = 2: 128x256
// tiles with 64x128 shares (for shapes whose 256x256 tiles leave CUs idle, and for the
// remainder of a launch beyond its last whole round of tiles).  TN = 3: 192 columns with
// 96-column shares (N = 6144, the 8B layer's KQV: 8 x 32 = 256 tiles of 256x192 at 2048 rows,
// of 128x192 at 1024 rows, one per CU, where 256 columns give 192 tiles; not for SwiGLU, whose
// epilogue pairs 32-column groups).  Same MFMA and K order as
// the other loops, hence the same output bits.  Requires K % 128 == 0 and 64 * TN | N.
// XS = 3 (128x256 tiles only): three stages of x rows as well, so that the x rows are requested
// two K-steps ahead like the w rows.  Alone it changes little; on a CU shared with wavefronts
// that stream from HBM, where a cache hit waits about a microsecond behind their misses (the
// per-CU memory path returns in order), a K-step of lead is not enough and two are.
template <int EPI, bool GROUPED = false, int TM = 4, int TN = 4, int XS = 2>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_w4_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, bf16_t* __restrict__ Y, const bf16_t* __restrict__ R,
    int M, int N, int K, int tiles_m, int tiles_n, GroupedArgs grp, KRange kr) {
  constexpr int WM = 32 * TM, BM = 2 * WM, BN = 64 * TN, NW = 4, WN = 32 * TN;
  static_assert(TM == 4 || TM == 2, "256x256 tiles, or 128x256 tiles with 64x128 wavefront shares");
  static_assert(TN == 4 || (TN == 3 && EPI != EPI_SWIGLU), "or 192 columns with 96-column shares");
  constexpr int BKT = 64, RB = 128, CPR = 8, RPI = 8;
  constexpr int ROWS = BM + BN;
  constexpr int LOADS = ROWS / RPI / NW;  // per K-step: BM / 32 of x, then 8 of w
  constexpr int XLOADS = BM / RPI / NW, WLOADS = BN / RPI / NW;
  // LDS: two stages of x rows, then three stages of w rows (a third stage of both would not fit)
  static_assert(XS == 2 || (XS == 3 && TM == 2), "a third stage of x rows fits beside 128-row tiles only");
  constexpr int XSTAGE = BM * RB, WSTAGE = BN * RB, WBASE = XS * XSTAGE;
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  int m0, n0;
  size_t w_off;
  if (!locate_tile<BM, BN, GROUPED>(tiles_m, tiles_n, grp, m0, n0, M, w_off)) return;  // before any barrier
  n0 += kr.n_first * BN;
  const size_t k_begin = (size_t)blockIdx.y * K;  // this workgroup's K segment
  X += k_begin;
  W += w_off + k_begin;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;

  // Loader: instruction i of this wavefront fills LDS rows (i*4 + wave)*8 .. +8 of a stage
  // (i < BM / 32: rows of x, else rows of w); this lane supplies row +lane/8, slot lane%8, i.e. global
  // chunk (lane%8) ^ ((row >> 1) & 7).
  const bf16_t* src[LOADS];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int row = (i * NW + wave) * RPI + lane / CPR;
    const int chunk = (lane % CPR) ^ ((row >> 1) & 7);
    if (row < BM) {
      int gm = m0 + row;
      gm = gm < M ? gm : M - 1;  // rows past M are computed on a copy of the last row and never stored
      if (GROUPED && grp.row_index) gm = grp.row_index[gm];
      src[i] = X + (size_t)gm * kr.ldk + chunk * 8;
    } else {
      src[i] = W + (size_t)weight_row<EPI>(row - BM, n0, N) * kr.ldk + chunk * 8;
    }
  }
  // load I of the K-step its pointer stands at: an x load into x stage xs, a w load to byte
  // offset wf of the w region
  auto load_one = [&](const int I, const uint32_t xf, const uint32_t wf) __attribute__((always_inline)) {
    // weight rows are used by the few tiles of one tile column and then never again: loaded
    // non-temporal they do not push the x rows, which every tile column re-reads, out of the
    // L2 (measured: 2-3 % on Up/Gate; non-temporal x rows or both: no gain; with 128x256 tiles,
    // where twice as many tiles share a weight row, it costs 15 %, so those load normally)
    if (I < XLOADS)
      __builtin_amdgcn_global_load_lds((gptr_t)src[I], (lptr_t)(lds + xf + (I * NW + wave) * 1024), 16, 0, 0);
    else if (TM != 4)
      __builtin_amdgcn_global_load_lds((gptr_t)src[I],
                                       (lptr_t)(lds + WBASE + wf + ((I - XLOADS) * NW + wave) * 1024), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((gptr_t)src[I],
                                       (lptr_t)(lds + WBASE + wf + ((I - XLOADS) * NW + wave) * 1024), 16, 0, 2);
    src[I] += BKT;
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = K / BKT;  // even
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lptr_t)lds;
  const int frag_row = lane & 31, g = lane >> 5;
  const uint32_t swz = (uint32_t)((frag_row >> 1) & 7);
  uint32_t x_addr[4], w_addr[4];  // fragment addresses of the four K-slices in stage 0 of their regions
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const uint32_t slot = (((uint32_t)(2 * kk + g)) ^ swz) * 16;
    x_addr[kk] = lds_base + (uint32_t)((wm * WM + frag_row) * RB) + slot;
    w_addr[kk] = lds_base + (uint32_t)(WBASE + (wn * WN + frag_row) * RB) + slot;
  }
  bf16x8 fw[4][TN], fx[4][TM];  // one fragment buffer per K-slice
  using seq_w = std::make_integer_sequence<int, TN>;
#define NF_W4_READ(KK, XB, WB)                                                                                  \
  lds_read_frags<0, 32 * RB>(fw[KK], w_addr[KK] + (WB), seq_w{});                                                \
  lds_read_frags<0, 32 * RB>(fx[KK], x_addr[KK] + (XB), std::make_integer_sequence<int, TM>{})

  // prologue: x rows of K-steps 0 and 1 and w rows of K-steps 0, 1 and 2 on their way (the w
  // rows of K-step 2 last, so that a wait can leave exactly them in flight), K-step 0 landed,
  // its first two slices requested
#pragma unroll
  for (int i = 0; i < LOADS; ++i) load_one(i, 0, 0);
#pragma unroll
  for (int i = 0; i < LOADS; ++i) load_one(i, XSTAGE, WSTAGE);
  if (2 < KT) {
    // K-step 2: its w rows, and with three x stages its x rows too
#pragma unroll
    for (int i = (XS == 3 ? 0 : XLOADS); i < LOADS; ++i) load_one(i, 2 * XSTAGE, 2 * WSTAGE);
  }
  if (2 < KT)
    wait_vmcnt<LOADS + (XS == 3 ? LOADS : WLOADS)>();
  else
    wait_vmcnt<LOADS>();
  __builtin_amdgcn_s_barrier();
  NF_W4_READ(0, 0, 0);
  NF_W4_READ(1, 0, 0);

#define NF_W4_MFMA(B, I, J)                                                                                     \
  if constexpr ((J) < TM && (I) < TN)                                                                           \
    acc[(I) < TN ? (I) : 0][(J) < TM ? (J) : 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                       \
        fw[B][(I) < TN ? (I) : 0], fx[B][(J) < TM ? (J) : 0], acc[(I) < TN ? (I) : 0][(J) < TM ? (J) : 0], 0, 0, \
        0);                                                                                                     \
  __builtin_amdgcn_sched_barrier(0)
#define NF_W4_LOAD(I)                                                                                           \
  if constexpr (XS == 3 ? (WRELOAD && (I) < LOADS) : ((I) < XLOADS ? XRELOAD : (WRELOAD && (I) < LOADS)))        \
    load_one(I, CUR, w_cur);                                                                                    \
  __builtin_amdgcn_sched_barrier(0)
  // fragment I (0..3: w, 4..7: x) of K-slice KK from the stage at BASE, if ON
#define NF_W4_RD1(ON, KK, XB, WB, I)                                                                            \
  if constexpr (ON) {                                                                                           \
    if constexpr ((I) < 4) {                                                                                    \
      if constexpr (((I) & 3) < TN)                                                                             \
        fw[KK][((I) & 3) < TN ? ((I) & 3) : 0] = lds_read_frag_at<((I) & 3) * 32 * RB>(w_addr[KK] + (WB));       \
    } else if constexpr (((I) & 3) < TM)                                                                        \
      fx[KK][((I) & 3) < TM ? ((I) & 3) : 0] = lds_read_frag_at<((I) & 3) * 32 * RB>(x_addr[KK] + (XB));         \
  }                                                                                                             \
  __builtin_amdgcn_sched_barrier(0)
  // 16 MFMAs of slice B; behind every second one a fragment read of slice KK (stage BASE)
#define NF_W4_SLICE_READS(B, ON, KK, XB, WB)                                                                      \
  NF_W4_MFMA(B, 0, 0); NF_W4_MFMA(B, 0, 1); NF_W4_RD1(ON, KK, XB, WB, 0);                                         \
  NF_W4_MFMA(B, 0, 2); NF_W4_MFMA(B, 0, 3); NF_W4_RD1(ON, KK, XB, WB, 1);                                         \
  NF_W4_MFMA(B, 1, 0); NF_W4_MFMA(B, 1, 1); NF_W4_RD1(ON, KK, XB, WB, 2);                                         \
  NF_W4_MFMA(B, 1, 2); NF_W4_MFMA(B, 1, 3); NF_W4_RD1(ON, KK, XB, WB, 3);                                         \
  NF_W4_MFMA(B, 2, 0); NF_W4_MFMA(B, 2, 1); NF_W4_RD1(ON, KK, XB, WB, 4);                                         \
  NF_W4_MFMA(B, 2, 2); NF_W4_MFMA(B, 2, 3); NF_W4_RD1(ON, KK, XB, WB, 5);                                         \
  NF_W4_MFMA(B, 3, 0); NF_W4_MFMA(B, 3, 1); NF_W4_RD1(ON, KK, XB, WB, 6);                                         \
  NF_W4_MFMA(B, 3, 2); NF_W4_MFMA(B, 3, 3); NF_W4_RD1(ON, KK, XB, WB, 7)
  // the same with a global load behind the other MFMAs
#define NF_W4_SLICE_READS_LOADS(B, ON, KK, XB, WB, L0)                                                            \
  NF_W4_MFMA(B, 0, 0); NF_W4_LOAD(L0 + 0); NF_W4_MFMA(B, 0, 1); NF_W4_RD1(ON, KK, XB, WB, 0);                     \
  NF_W4_MFMA(B, 0, 2); NF_W4_LOAD(L0 + 1); NF_W4_MFMA(B, 0, 3); NF_W4_RD1(ON, KK, XB, WB, 1);                     \
  NF_W4_MFMA(B, 1, 0); NF_W4_LOAD(L0 + 2); NF_W4_MFMA(B, 1, 1); NF_W4_RD1(ON, KK, XB, WB, 2);                     \
  NF_W4_MFMA(B, 1, 2); NF_W4_LOAD(L0 + 3); NF_W4_MFMA(B, 1, 3); NF_W4_RD1(ON, KK, XB, WB, 3);                     \
  NF_W4_MFMA(B, 2, 0); NF_W4_LOAD(L0 + 4); NF_W4_MFMA(B, 2, 1); NF_W4_RD1(ON, KK, XB, WB, 4);                     \
  NF_W4_MFMA(B, 2, 2); NF_W4_LOAD(L0 + 5); NF_W4_MFMA(B, 2, 3); NF_W4_RD1(ON, KK, XB, WB, 5);                     \
  NF_W4_MFMA(B, 3, 0); NF_W4_LOAD(L0 + 6); NF_W4_MFMA(B, 3, 1); NF_W4_RD1(ON, KK, XB, WB, 6);                     \
  NF_W4_MFMA(B, 3, 2); NF_W4_LOAD(L0 + 7); NF_W4_MFMA(B, 3, 3); NF_W4_RD1(ON, KK, XB, WB, 7)
  // K-step k with its x rows in stage STAGE = k & 1.  MORE: there is a K-step k + 1 (the tail
  // flags are compile-time, so that the steady state has no branches).  The fragments of a
  // slice are requested two slices ahead, one read behind every second MFMA: at the top of a
  // slice at most the eight reads of the next slice are outstanding behind its own.
  // w_cur / w_next: byte offsets of the w stages of K-steps k and k + 1 (k % 3 and (k + 1) % 3
  // stages in); the w rows of K-step k + 3 go where those of K-step k were.  XRELOAD: there is
  // a K-step k + 2; WRELOAD: a K-step k + 3.  The loads of a K-step are issued x rows first:
  // waiting until only WLOADS loads are outstanding leaves the w rows of K-step k + 2 in flight
  // and has everything of K-step k + 1 in LDS.
  // With three x stages the x rows rotate like the w rows: x_cur / x_next are the byte offsets
  // of the x stages of K-steps k and k + 1, and the x rows of K-step k + 3 are requested together
  // with its w rows (into the stages K-step k has left); the wait in front of the barrier then
  // leaves all loads of K-step k + 2 in flight.
  auto k_step = [&](auto stage_c, auto more_c, auto xreload_c, auto wreload_c, const uint32_t w_cur,
                    const uint32_t w_next, const uint32_t x_cur, const uint32_t x_next) {
    constexpr int STAGE = decltype(stage_c)::value;
    constexpr bool MORE = decltype(more_c)::value, XRELOAD = decltype(xreload_c)::value,
                   WRELOAD = decltype(wreload_c)::value;
    const uint32_t CUR = XS == 3 ? x_cur : (uint32_t)(STAGE * XSTAGE);
    const uint32_t NEXT = XS == 3 ? x_next : (uint32_t)((1 - STAGE) * XSTAGE);
    wait_frags<TN + TM, TN, TM>(fw[0], fx[0]);
    NF_W4_SLICE_READS(0, true, 2, CUR, w_cur);
    wait_frags<TN + TM, TN, TM>(fw[1], fx[1]);
    NF_W4_SLICE_READS(1, true, 3, CUR, w_cur);
    // this wavefront has read all it needs of K-step k, and its part of K-step k + 1 is in LDS
    wait_frags<0, TN, TM>(fw[2], fx[2]);
    wait_frags<0, TN, TM>(fw[3], fx[3]);
    if (MORE) {
      if (XRELOAD)
        wait_vmcnt<(XS == 3 ? LOADS : WLOADS)>();  // the w rows (and third-stage x rows) of K-step k + 2 stay in flight
      else
        wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    NF_W4_SLICE_READS_LOADS(2, MORE, 0, NEXT, w_next, 0);
    NF_W4_SLICE_READS_LOADS(3, MORE, 1, NEXT, w_next, 8);
  };
  using T = std::true_type;
  using F = std::false_type;
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  uint32_t w_cur = 0, w_next = WSTAGE, x_cur = 0, x_next = XSTAGE;
  auto advance = [&]() {
    w_cur = w_next;
    w_next = w_next == 2 * WSTAGE ? 0 : w_next + WSTAGE;
    x_cur = x_next;
    x_next = x_next == 2 * XSTAGE ? 0 : x_next + XSTAGE;
  };
  int k = 0;
  for (; k + 4 < KT; k += 2) {
    k_step(C0{}, T{}, T{}, T{}, w_cur, w_next, x_cur, x_next);
    advance();
    k_step(C1{}, T{}, T{}, T{}, w_cur, w_next, x_cur, x_next);
    advance();
  }
  if (k + 2 < KT) {  // K-steps KT - 4 and KT - 3
    k_step(C0{}, T{}, T{}, T{}, w_cur, w_next, x_cur, x_next);
    advance();
    k_step(C1{}, T{}, T{}, F{}, w_cur, w_next, x_cur, x_next);
    advance();
  }
  k_step(C0{}, T{}, F{}, F{}, w_cur, w_next, x_cur, x_next);
  advance();
  k_step(C1{}, F{}, F{}, F{}, w_cur, w_next, x_cur, x_next);
#undef NF_W4_MFMA
#undef NF_W4_LOAD
#undef NF_W4_SLICE_READS
#undef NF_W4_SLICE_READS_LOADS
#undef NF_W4_RD1
#undef NF_W4_READ

  if (EPI == EPI_PARTIAL) {
    store_tile<EPI, TM, TN, WM, WN>(acc, Y, R, M, N, m0, n0, wm, wn, lane,
                                    kr.partial + (size_t)blockIdx.y * (size_t)kr.seg_stride);
  } else {
    // WM x (2 * WN + 16) bytes per wavefront: the launcher sizes the LDS for it
    store_tile_rows<EPI, TM, TN, WM, WN>(acc, Y, R, M, N, m0, n0, wm, wn, lane,
                                         lds_base + (uint32_t)(wave * (WM * (WN * 2 + 16))));
  }
}

// out = bf16((p0 + p1) [+ residual]): the second step of a two-segment operation whose
// segments were summed by different workgroups.  One thread per 4 consecutive elements.
__global__ __launch_bounds__(256) void gemm_reduce2_kernel(const float* __restrict__ p0, const float* __restrict__ p1,
                                                          const bf16_t* __restrict__ R, bf16_t* __restrict__ Y,
                                                          size_t n_quads) {
  const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= n_quads) return;
  const f32x4 a = reinterpret_cast<const f32x4*>(p0)[q], b = reinterpret_cast<const f32x4*>(p1)[q];
  float o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = a[e] + b[e];
  if (R) {
    const u32x2 r = reinterpret_cast<const u32x2*>(R)[q];
    o[0] += __uint_as_float(r[0] << 16);
    o[1] += __uint_as_float(r[0] & 0xffff0000u);
    o[2] += __uint_as_float(r[1] << 16);
    o[3] += __uint_as_float(r[1] & 0xffff0000u);
  }
  const u32x2 pk = {pack_bf2(o[0], o[1]), pack_bf2(o[2], o[3])};
  reinterpret_cast<u32x2*>(Y)[q] = pk;
}

template <typename Kern>
hipError_t allow_lds(Kern kern, size_t lds_bytes, bool& done) {
  if (lds_bytes <= 64 * 1024 || done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  done = e == hipSuccess;
  return e;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool GROUPED, int BKT>
hipError_t launch_dl2(const void* x, const void* w, void* out, const void* residual, int M, int N, int K, int epilogue,
                      hipStream_t s, GroupedArgs grp) {
  const int tiles_m = GROUPED ? (M + BM - 1) / BM + grp.n_experts : (M + BM - 1) / BM;
  const int tiles_n = epilogue == EPI_SWIGLU ? (2 * N) / BN : N / BN;
  const dim3 grid(tiles_m * tiles_n), block(64 * WAVES_M * WAVES_N);
  const size_t lds_bytes = (size_t)STAGES * (BM + BN) * BKT * 2;
  const bf16_t* X = (const bf16_t*)x;
  const bf16_t* Wp = (const bf16_t*)w;
  bf16_t* Y = (bf16_t*)out;
  const bf16_t* R = (const bf16_t*)residual;
#define NF_DL2_LAUNCH(E)                                                                                           \
  do {                                                                                                             \
    auto kern = gemm_dl2_kernel<BM, BN, WAVES_M, WAVES_N, E, STAGES, GROUPED, BKT>;                                 \
    static bool attr_set = false;                                                                                  \
    if (lds_bytes > 64 * 1024 && !attr_set) {                                                                      \
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,            \
                                         (int)lds_bytes);                                                          \
      if (e != hipSuccess) return e;                                                                               \
      attr_set = true;                                                                                             \
    }                                                                                                              \
    kern<<<grid, block, lds_bytes, s>>>(X, Wp, Y, R, M, N, K, tiles_m, tiles_n, grp, KRange{K, nullptr, 0});       \
  } while (0)
  switch (epilogue) {
    case EPI_NONE: NF_DL2_LAUNCH(EPI_NONE); break;
    case EPI_RESIDUAL: NF_DL2_LAUNCH(EPI_RESIDUAL); break;
    default: NF_DL2_LAUNCH(EPI_SWIGLU); break;
  }
#undef NF_DL2_LAUNCH
  return hipGetLastError();
}

// One launch of the four-wavefront loop with tiles of 64 * TM rows over the tile columns
// [n_first, n_first + n_tiles).
template <bool GROUPED, int TM, int TN = 4, int XS = 2>
hipError_t launch_w4_columns(const void* x, const void* w, void* out, const void* residual, int M, int N, int K,
                             int epilogue, hipStream_t s, GroupedArgs grp, int n_first, int n_tiles) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  const int tiles_m = GROUPED ? (M + BM - 1) / BM + grp.n_experts : (M + BM - 1) / BM;
  const dim3 grid(tiles_m * n_tiles), block(256);
  // two x stages and three w stages; the epilogue reuses them as 4 regions of (BM / 2) rows x 272 bytes
  const size_t lds_bytes = std::max((size_t)(XS * BM + 3 * BN) * 128, (size_t)4 * (BM / 2) * (BN + 16));
  KRange kr{K, nullptr, 0};
  kr.n_first = n_first;
#define NF_W4_LAUNCH(E)                                                                                            \
  do {                                                                                                             \
    auto kern = gemm_w4_kernel<E, GROUPED, TM, TN, XS>;                                                             \
    static bool attr_set = false;                                                                                  \
    hipError_t e = allow_lds(kern, lds_bytes, attr_set);                                                           \
    if (e != hipSuccess) return e;                                                                                 \
    kern<<<grid, block, lds_bytes, s>>>((const bf16_t*)x, (const bf16_t*)w, (bf16_t*)out, (const bf16_t*)residual, \
                                        M, N, K, tiles_m, n_tiles, grp, kr);                                       \
  } while (0)
  switch (epilogue) {
    case EPI_NONE: NF_W4_LAUNCH(EPI_NONE); break;
    case EPI_RESIDUAL: NF_W4_LAUNCH(EPI_RESIDUAL); break;
    default:
      if constexpr (TN == 4) {
        NF_W4_LAUNCH(EPI_SWIGLU);
      } else {
        return hipErrorInvalidValue;
      }
      break;
  }
#undef NF_W4_LAUNCH
  return hipGetLastError();
}

// 256x256 tiles.  When the tiles beyond the last whole round of 256 fill at most half a round
// (the 8B layer's Up/Gate at 2048 rows: 896 tiles = 3.5 rounds), the tile columns of that
// remainder run as a second launch of 128x256 tiles - twice the workgroups of half the work,
// so the last round takes about two thirds as long.  Every output element is still one
// accumulation in ascending K order: the bits do not change.
template <bool GROUPED>
hipError_t launch_w4(const void* x, const void* w, void* out, const void* residual, int M, int N, int K, int epilogue,
                     hipStream_t s, GroupedArgs grp) {
  const int n_eff = epilogue == EPI_SWIGLU ? 2 * N : N;
  if (K % 128 != 0 || n_eff % 256 != 0) return hipErrorInvalidValue;
  const int tiles_n = n_eff / 256;
  if (!GROUPED) {
    const int tiles_m = (M + 255) / 256;
    const long tiles = (long)tiles_m * tiles_n, whole = tiles / 256 * 256, rest = tiles - whole;
    if (whole > 0 && rest > 0 && rest <= 128 && whole % tiles_m == 0) {
      const int n_whole = (int)(whole / tiles_m);
      hipError_t e = launch_w4_columns<false, 4>(x, w, out, residual, M, N, K, epilogue, s, grp, 0, n_whole);
      if (e != hipSuccess) return e;
      return launch_w4_columns<false, 2>(x, w, out, residual, M, N, K, epilogue, s, grp, n_whole, tiles_n - n_whole);
    }
  }
  return launch_w4_columns<GROUPED, 4>(x, w, out, residual, M, N, K, epilogue, s, grp, 0, tiles_n);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool GROUPED, bool PIPE = false>
hipError_t launch_dl(const void* x, const void* w, void* out, const void* residual, int M, int N, int K, int epilogue,
                     hipStream_t s, GroupedArgs grp) {
  const int tiles_m = GROUPED ? (M + BM - 1) / BM + grp.n_experts : (M + BM - 1) / BM;
  const int tiles_n = epilogue == EPI_SWIGLU ? (2 * N) / BN : N / BN;
  const dim3 grid(tiles_m * tiles_n), block(64 * WAVES_M * WAVES_N);
  const size_t lds_bytes = (size_t)STAGES * (BM + BN) * 128;
  const bf16_t* X = (const bf16_t*)x;
  const bf16_t* Wp = (const bf16_t*)w;
  bf16_t* Y = (bf16_t*)out;
  const bf16_t* R = (const bf16_t*)residual;
#define NF_DL_LAUNCH(E)                                                                                            \
  do {                                                                                                             \
    auto kern = gemm_dl_kernel<BM, BN, WAVES_M, WAVES_N, E, STAGES, GROUPED, PIPE>;                                      \
    static bool attr_set = false;                                                                                  \
    if (lds_bytes > 64 * 1024 && !attr_set) {                                                                      \
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,            \
                                         (int)lds_bytes);                                                          \
      if (e != hipSuccess) return e;                                                                               \
      attr_set = true;                                                                                             \
    }                                                                                                              \
    kern<<<grid, block, lds_bytes, s>>>(X, Wp, Y, R, M, N, K, tiles_m, tiles_n, grp, KRange{K, nullptr, 0});       \
  } while (0)
  switch (epilogue) {
    case EPI_NONE: NF_DL_LAUNCH(EPI_NONE); break;
    case EPI_RESIDUAL: NF_DL_LAUNCH(EPI_RESIDUAL); break;
    default: NF_DL_LAUNCH(EPI_SWIGLU); break;
  }
#undef NF_DL_LAUNCH
  return hipGetLastError();
}


// The two halves of K as separate workgroups (grid.y = 2), fp32 sums to scratch.  GROUPED:
// M is the total row count, every expert may add one partial tile (see GroupedArgs).
template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool PIPE, bool GROUPED = false>
hipError_t launch_dl_halves(const void* x, const void* w, int M, int N, int K, KRange kr, hipStream_t s,
                            GroupedArgs grp = GroupedArgs{nullptr, nullptr, 0, 0}) {
  const int tiles_m = GROUPED ? (M + BM - 1) / BM + grp.n_experts : (M + BM - 1) / BM, tiles_n = N / BN;
  const size_t lds_bytes = (size_t)STAGES * (BM + BN) * 128;
  auto kern = gemm_dl_kernel<BM, BN, WAVES_M, WAVES_N, EPI_PARTIAL, STAGES, GROUPED, PIPE>;
  static bool attr_set = false;
  hipError_t e = allow_lds(kern, lds_bytes, attr_set);
  if (e != hipSuccess) return e;
  kern<<<dim3(tiles_m * tiles_n, 2), dim3(64 * WAVES_M * WAVES_N), lds_bytes, s>>>(
      (const bf16_t*)x, (const bf16_t*)w, nullptr, nullptr, M, N, K / 2, tiles_m, tiles_n, grp, kr);
  return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int BKT, bool GROUPED = false>
hipError_t launch_dl2_halves(const void* x, const void* w, int M, int N, int K, KRange kr, hipStream_t s,
                             GroupedArgs grp = GroupedArgs{nullptr, nullptr, 0, 0}) {
  const int tiles_m = GROUPED ? (M + BM - 1) / BM + grp.n_experts : (M + BM - 1) / BM, tiles_n = N / BN;
  const size_t lds_bytes = (size_t)STAGES * (BM + BN) * BKT * 2;
  auto kern = gemm_dl2_kernel<BM, BN, WAVES_M, WAVES_N, EPI_PARTIAL, STAGES, GROUPED, BKT>;
  static bool attr_set = false;
  hipError_t e = allow_lds(kern, lds_bytes, attr_set);
  if (e != hipSuccess) return e;
  kern<<<dim3(tiles_m * tiles_n, 2), dim3(64 * WAVES_M * WAVES_N), lds_bytes, s>>>(
      (const bf16_t*)x, (const bf16_t*)w, nullptr, nullptr, M, N, K / 2, tiles_m, tiles_n, grp, kr);
  return hipGetLastError();
}

// Both halves of K in one workgroup (two accumulator sets).
template <int EPI>
hipError_t launch_dl2_two_sums(const void* x, const void* w, void* out, const void* residual, int M, int N, int K,
                               hipStream_t s) {
  constexpr int BM = 256, BN = 128, STAGES = 3, BKT = 64;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
  const size_t lds_bytes = (size_t)STAGES * (BM + BN) * BKT * 2;
  auto kern = gemm_dl2_kernel<BM, BN, 4, 2, EPI, STAGES, false, BKT, true>;
  static bool attr_set = false;
  hipError_t e = allow_lds(kern, lds_bytes, attr_set);
  if (e != hipSuccess) return e;
  kern<<<dim3(tiles_m * tiles_n), dim3(512), lds_bytes, s>>>((const bf16_t*)x, (const bf16_t*)w, (bf16_t*)out,
                                                            (const bf16_t*)residual, M, N, K, tiles_m, tiles_n,
                                                            GroupedArgs{nullptr, nullptr, 0, 0}, KRange{K, nullptr, 0});
  return hipGetLastError();
}

}  // namespace

// Two-segment operation, both segments summed inside each workgroup (256x128 tiles): needs
// no scratch.  K % 128 == 0, N % 128 == 0; epilogue EPI_NONE or EPI_RESIDUAL.
hipError_t nf_launch_gemm_dl_two_sums(const void* x, const void* w, void* out, const void* residual, int M, int N,
                                      int K, int epilogue, hipStream_t s) {
  if (epilogue == EPI_RESIDUAL) return launch_dl2_two_sums<EPI_RESIDUAL>(x, w, out, residual, M, N, K, s);
  if (epilogue == EPI_NONE) return launch_dl2_two_sums<EPI_NONE>(x, w, out, residual, M, N, K, s);
  return hipErrorInvalidValue;
}

// Two-segment operation with the segments on different workgroups: twice the workgroups of
// the one-launch form, for row counts that would leave most of the chip idle.  partial holds
// the two [M, N] fp32 sums seg_stride floats apart; a second kernel adds them (+ residual).
// variant: 7 = 128x128, 12 = 256x128, 13 = 256x256 (N % 256 == 0), 19 = 256x128 second main loop,
// 21 / 22 = the four-wavefront loop with 256x256 / 128x256 tiles (K % 256 == 0, N % 256 == 0).
hipError_t nf_launch_gemm_dl_halves(const void* x, const void* w, void* out, const void* residual, int M, int N,
                                    int K, float* partial, long long seg_stride, int variant, hipStream_t s) {
  const KRange kr{K, partial, seg_stride};
  hipError_t e;
  switch (variant) {
    case 7: e = launch_dl_halves<128, 128, 2, 2, 2, false>(x, w, M, N, K, kr, s); break;
    case 12: e = launch_dl_halves<256, 128, 4, 2, 3, true>(x, w, M, N, K, kr, s); break;
    case 13: e = launch_dl_halves<256, 256, 2, 4, 2, true>(x, w, M, N, K, kr, s); break;
    case 19: e = launch_dl2_halves<256, 128, 4, 2, 3, 64>(x, w, M, N, K, kr, s); break;
    case 21: {
      // the four-wavefront loop: each half of K must be a multiple of its 128-element period
      if (K % 256 != 0 || N % 256 != 0) return hipErrorInvalidValue;
      const int tiles_m = (M + 255) / 256, tiles_n = N / 256;
      const size_t lds_bytes = (size_t)(2 * 256 + 3 * 256) * 128;
      static bool attr_set = false;
      e = allow_lds(gemm_w4_kernel<EPI_PARTIAL>, lds_bytes, attr_set);
      if (e != hipSuccess) return e;
      gemm_w4_kernel<EPI_PARTIAL><<<dim3(tiles_m * tiles_n, 2), dim3(256), lds_bytes, s>>>(
          (const bf16_t*)x, (const bf16_t*)w, nullptr, nullptr, M, N, K / 2, tiles_m, tiles_n,
          GroupedArgs{nullptr, nullptr, 0, 0}, kr);
      e = hipGetLastError();
      break;
    }
    case 22: {  // the same with 128x256 tiles: twice the workgroups for few rows
      if (K % 256 != 0 || N % 256 != 0) return hipErrorInvalidValue;
      const int tiles_m = (M + 127) / 128, tiles_n = N / 256;
      const size_t lds_bytes = (size_t)(2 * 128 + 3 * 256) * 128;
      static bool attr_set = false;
      e = allow_lds(gemm_w4_kernel<EPI_PARTIAL, false, 2>, lds_bytes, attr_set);
      if (e != hipSuccess) return e;
      gemm_w4_kernel<EPI_PARTIAL, false, 2><<<dim3(tiles_m * tiles_n, 2), dim3(256), lds_bytes, s>>>(
          (const bf16_t*)x, (const bf16_t*)w, nullptr, nullptr, M, N, K / 2, tiles_m, tiles_n,
          GroupedArgs{nullptr, nullptr, 0, 0}, kr);
      e = hipGetLastError();
      break;
    }
    case 25: {  // 128x256 tiles with three stages of x rows
      if (K % 256 != 0 || N % 256 != 0) return hipErrorInvalidValue;
      const int tiles_m = (M + 127) / 128, tiles_n = N / 256;
      const size_t lds_bytes = (size_t)(3 * 128 + 3 * 256) * 128;
      static bool attr_set = false;
      e = allow_lds(gemm_w4_kernel<EPI_PARTIAL, false, 2, 4, 3>, lds_bytes, attr_set);
      if (e != hipSuccess) return e;
      gemm_w4_kernel<EPI_PARTIAL, false, 2, 4, 3><<<dim3(tiles_m * tiles_n, 2), dim3(256), lds_bytes, s>>>(
          (const bf16_t*)x, (const bf16_t*)w, nullptr, nullptr, M, N, K / 2, tiles_m, tiles_n,
          GroupedArgs{nullptr, nullptr, 0, 0}, kr);
      e = hipGetLastError();
      break;
    }
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  const size_t n_quads = (size_t)M * N / 4;
  gemm_reduce2_kernel<<<dim3((unsigned)((n_quads + 255) / 256)), dim3(256), 0, s>>>(
      partial, partial + seg_stride, (const bf16_t*)residual, (bf16_t*)out, n_quads);
  return hipGetLastError();
}

// Grouped mode of the two-segment operation (the experts' down projection): the fp32 sums of
// the two halves of K go to partial and partial + seg_stride, rows at their sorted positions;
// the consumer (the combine kernel) adds them.  variant: 12 / 19 = 256x128 tiles, 13 = 256x256,
// 21 = 256x256 with the four-wavefront loop.
hipError_t nf_launch_gemm_dl_grouped_halves(const void* x, const void* w, int rows, int N, int K, float* partial,
                                            long long seg_stride, const int32_t* expert_offset,
                                            const int32_t* row_index, int n_experts, long long w_stride, int variant,
                                            hipStream_t s) {
  const GroupedArgs grp{expert_offset, row_index, n_experts, w_stride};
  const KRange kr{K, partial, seg_stride};
  switch (variant) {
    case 12: return launch_dl_halves<256, 128, 4, 2, 3, true, true>(x, w, rows, N, K, kr, s, grp);
    case 13: return launch_dl_halves<256, 256, 2, 4, 2, true, true>(x, w, rows, N, K, kr, s, grp);
    case 19: return launch_dl2_halves<256, 128, 4, 2, 3, 64, true>(x, w, rows, N, K, kr, s, grp);
    case 21: {
      if (K % 256 != 0 || N % 256 != 0) return hipErrorInvalidValue;
      const int tiles_m = (rows + 255) / 256 + n_experts, tiles_n = N / 256;
      const size_t lds_bytes = (size_t)(2 * 256 + 3 * 256) * 128;
      static bool attr_set = false;
      hipError_t e = allow_lds(gemm_w4_kernel<EPI_PARTIAL, true>, lds_bytes, attr_set);
      if (e != hipSuccess) return e;
      gemm_w4_kernel<EPI_PARTIAL, true><<<dim3(tiles_m * tiles_n, 2), dim3(256), lds_bytes, s>>>(
          (const bf16_t*)x, (const bf16_t*)w, nullptr, nullptr, rows, N, K / 2, tiles_m, tiles_n, grp, kr);
      return hipGetLastError();
    }
    default: return hipErrorInvalidValue;
  }
}

// Variants: 7 = 128x128 tile, 4 wavefronts, 2 stages (two workgroups per CU);
//           8 = 128x128, 4 wavefronts, 4 stages (one workgroup per CU);
//           9 = 256x128, 8 wavefronts, 3 stages; 10 = 256x256, 8 wavefronts, 2 stages;
//           11..14 = 7, 9, 10, 8 with the explicitly scheduled main loop;
//           15..19 = the second main loop: 256x256 with K-step 32 and 4 / 5 stages, 256x256 with
//           K-step 64 and 2 stages, 256x128 with K-step 32 and 6 stages, 256x128 with K-step 64
//           and 3 stages; 20 = 256x192 with K-step 64 and 2 stages (N % 192 == 0, no SwiGLU).
// Requires K % 64 == 0 and the (stacked) N % 128 == 0 (% 256 for the 256-wide tiles).
hipError_t nf_launch_gemm_dl(const void* x, const void* w, void* out, const void* residual, int M, int N, int K,
                             int epilogue, int variant, hipStream_t s) {
  const GroupedArgs none{nullptr, nullptr, 0, 0};
  switch (variant) {
    case 7: return launch_dl<128, 128, 2, 2, 2, false>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 8: return launch_dl<128, 128, 2, 2, 4, false>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 9: return launch_dl<256, 128, 4, 2, 3, false>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 10: return launch_dl<256, 256, 2, 4, 2, false>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 11: return launch_dl<128, 128, 2, 2, 2, false, true>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 12: return launch_dl<256, 128, 4, 2, 3, false, true>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 13: return launch_dl<256, 256, 2, 4, 2, false, true>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 14: return launch_dl<128, 128, 2, 2, 4, false, true>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 15: return launch_dl2<256, 256, 2, 4, 4, false, 32>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 16: return launch_dl2<256, 256, 2, 4, 5, false, 32>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 17: return launch_dl2<256, 256, 2, 4, 2, false, 64>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 18: return launch_dl2<256, 128, 4, 2, 6, false, 32>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 19: return launch_dl2<256, 128, 4, 2, 3, false, 64>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 20:
      // 256x192: N = 6144 (the 8B layer's KQV) gives 8 x 32 = 256 tiles, one per CU; the SwiGLU
      // epilogue needs an even number of 32-column groups per wavefront and has no such form
      if (epilogue == EPI_SWIGLU) return hipErrorInvalidValue;
      return launch_dl2<256, 192, 4, 2, 2, false, 64>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 21: return launch_w4<false>(x, w, out, residual, M, N, K, epilogue, s, none);
    case 22: {  // the four-wavefront loop with 128x256 tiles
      const int n_eff = epilogue == EPI_SWIGLU ? 2 * N : N;
      if (K % 128 != 0 || n_eff % 256 != 0) return hipErrorInvalidValue;
      return launch_w4_columns<false, 2>(x, w, out, residual, M, N, K, epilogue, s, none, 0, n_eff / 256);
    }
    case 23:  // the four-wavefront loop with 256x192 tiles
      if (K % 128 != 0 || N % 192 != 0 || epilogue == EPI_SWIGLU) return hipErrorInvalidValue;
      return launch_w4_columns<false, 4, 3>(x, w, out, residual, M, N, K, epilogue, s, none, 0, N / 192);
    case 24:  // and with 128x192 tiles
      if (K % 128 != 0 || N % 192 != 0 || epilogue == EPI_SWIGLU) return hipErrorInvalidValue;
      return launch_w4_columns<false, 2, 3>(x, w, out, residual, M, N, K, epilogue, s, none, 0, N / 192);
    case 25: {  // 128x256 tiles with three stages of x rows: the form for CUs shared with streaming wavefronts
      const int n_eff = epilogue == EPI_SWIGLU ? 2 * N : N;
      if (K % 128 != 0 || n_eff % 256 != 0) return hipErrorInvalidValue;
      return launch_w4_columns<false, 2, 4, 3>(x, w, out, residual, M, N, K, epilogue, s, none, 0, n_eff / 256);
    }
    default: return hipErrorInvalidValue;
  }
}

// Grouped mode (see GroupedArgs): 7 / 11 = 128x128 tiles, 9 / 12 / 19 = 256x128 tiles, 13 / 21 = 256x256 tiles.
hipError_t nf_launch_gemm_dl_grouped(const void* x, const void* w, void* out, int rows, int N, int K, int epilogue,
                                     const int32_t* expert_offset, const int32_t* row_index, int n_experts,
                                     long long w_stride, int variant, hipStream_t s) {
  const GroupedArgs grp{expert_offset, row_index, n_experts, w_stride};
  switch (variant) {
    case 7: return launch_dl<128, 128, 2, 2, 2, true>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
    case 9: return launch_dl<256, 128, 4, 2, 3, true>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
    case 11: return launch_dl<128, 128, 2, 2, 2, true, true>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
    case 12: return launch_dl<256, 128, 4, 2, 3, true, true>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
    case 13: return launch_dl<256, 256, 2, 4, 2, true, true>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
    case 19: return launch_dl2<256, 128, 4, 2, 3, true, 64>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
    case 21: return launch_w4<true>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
    default: return hipErrorInvalidValue;
  }
}
