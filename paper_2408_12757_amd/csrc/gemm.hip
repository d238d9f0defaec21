// Dense operations (paper Sec. 2.2): out[M, N] = epilogue(x[M, K] . w[N, K]^T), bf16 in,
// fp32 accumulation on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Tiling: one workgroup of 4 wavefronts computes a BM x BN output tile and walks K in
// steps of 64.  The x and w tiles are staged through LDS (register-staged double
// buffering: the global loads of step k+1 are in flight while step k is multiplied).
// The product is formed transposed - w rows feed the A operand, x rows the B operand -
// so that each lane ends up with 4 consecutive output columns of one token row and can
// store 8 bytes at a time.
//
// The K loop order and the MFMA instruction are the same for every M, so an output row
// is bit-identical no matter which token range (nano-batch) it was computed in.  Operations
// with a long K and few output columns (the FFN down projection) sum the two halves of K
// separately and add the sums - for every M alike - so that a nano-batch with few rows can
// spread each output tile over two workgroups (Sec. 4.1.2 and the ablation of Sec. 6.4 count
// the weaker batching effect of the smaller nano-operations as the price of nano-batching;
// this removes most of that price for the down projection).
#include <math.h>

#include "gemm_common.h"
#include "nf_kernels.h"

namespace {

using namespace nfgemm;

// BM x BN tile, 2 x 2 wavefronts, each wavefront (BM/2) x (BN/2).
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int PF, bool GROUPED>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, (BM * BN > 128 * 128) ? (WAVES_M * WAVES_N) / 4 : 2) void gemm_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, bf16_t* __restrict__ Y, const bf16_t* __restrict__ R,
    int M, int N, int K, int tiles_m, int tiles_n, GroupedArgs grp) {
  constexpr int NT = 64 * WAVES_M * WAVES_N;        // threads per workgroup
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wavefront tile
  constexpr int TM = WM / 32, TN = WN / 32;          // 32x32 MFMA tiles per wavefront
  constexpr int A_CHUNKS = BM * 8 / NT;              // 16-byte chunks per thread per stage
  constexpr int B_CHUNKS = BN * 8 / NT;
  __shared__ __attribute__((aligned(16))) bf16_t sX[2][BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) bf16_t sW[2][BN * LDS_STRIDE];

  int m0, n0;
  size_t w_off;
  if (!locate_tile<BM, BN, GROUPED>(tiles_m, tiles_n, grp, m0, n0, M, w_off)) return;  // before any barrier
  W += w_off;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  // global -> register staging
  const bf16_t* xg[A_CHUNKS];
  const bf16_t* wg[B_CHUNKS];
  int xs[A_CHUNKS], ws[B_CHUNKS];
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int q = i * NT + tid, row = q >> 3, c = q & 7;
    int gm = m0 + row;
    gm = gm < M ? gm : M - 1;  // rows past M are computed on a copy of the last row and never stored
    if (GROUPED && grp.row_index) gm = grp.row_index[gm];
    xg[i] = X + (size_t)gm * K + c * 8;
    xs[i] = row * LDS_STRIDE + c * 8;
  }
#pragma unroll
  for (int i = 0; i < B_CHUNKS; ++i) {
    const int q = i * NT + tid, row = q >> 3, c = q & 7;
    const int gn = weight_row<EPI>(row, n0, N);
    wg[i] = W + (size_t)gn * K + c * 8;
    ws[i] = row * LDS_STRIDE + c * 8;
  }

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Global -> LDS pipeline.  Tile kt is multiplied out of LDS stage kt & 1 while tile kt + 1
  // is written into the other stage from registers and tiles kt + 2 .. kt + 1 + PF are in
  // flight from global memory into a ring of PF register sets, so a load has PF K-steps
  // to arrive before anything waits on it.
  u32x4 xr[PF][A_CHUNKS], wr[PF][B_CHUNKS];
  const int KT = K / BK;
  {
    u32x4 x0[A_CHUNKS], w0[B_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) x0[i] = *reinterpret_cast<const u32x4*>(xg[i]);
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) w0[i] = *reinterpret_cast<const u32x4*>(wg[i]);
#pragma unroll
    for (int d = 0; d < PF; ++d) {
      if (d + 1 < KT) {
        const int koff = (d + 1) * BK;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) xr[d][i] = *reinterpret_cast<const u32x4*>(xg[i] + koff);
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) wr[d][i] = *reinterpret_cast<const u32x4*>(wg[i] + koff);
      }
    }
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<u32x4*>(&sX[0][xs[i]]) = x0[i];
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<u32x4*>(&sW[0][ws[i]]) = w0[i];
  }
  __syncthreads();

  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  for (int kt0 = 0; kt0 < KT; kt0 += PF) {
#pragma unroll
    for (int d = 0; d < PF; ++d) {
      const int kt = kt0 + d;
      if (kt < KT) {
        const int cur = kt & 1;
        const bf16_t* cx = &sX[cur][(wm * WM + frag_row) * LDS_STRIDE + frag_k];
        const bf16_t* cw = &sW[cur][(wn * WN + frag_row) * LDS_STRIDE + frag_k];
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
          bf16x8 fw[TN], fx[TM];
#pragma unroll
          for (int i = 0; i < TN; ++i) fw[i] = *reinterpret_cast<const bf16x8*>(cw + i * 32 * LDS_STRIDE + kk * 16);
#pragma unroll
          for (int j = 0; j < TM; ++j) fx[j] = *reinterpret_cast<const bf16x8*>(cx + j * 32 * LDS_STRIDE + kk * 16);
#pragma unroll
          for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fx[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) {
          const int nxt = cur ^ 1;
#pragma unroll
          for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<u32x4*>(&sX[nxt][xs[i]]) = xr[d][i];
#pragma unroll
          for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<u32x4*>(&sW[nxt][ws[i]]) = wr[d][i];
        }
        if (kt + 1 + PF < KT) {
          const int koff = (kt + 1 + PF) * BK;
#pragma unroll
          for (int i = 0; i < A_CHUNKS; ++i) xr[d][i] = *reinterpret_cast<const u32x4*>(xg[i] + koff);
#pragma unroll
          for (int i = 0; i < B_CHUNKS; ++i) wr[d][i] = *reinterpret_cast<const u32x4*>(wg[i] + koff);
        }
        __syncthreads();
      }
    }
  }

  store_tile<EPI, TM, TN, WM, WN>(acc, Y, R, M, N, m0, n0, wm, wn, lane);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int PF, bool GROUPED = false>
hipError_t launch(const void* x, const void* w, void* out, const void* residual, int M, int N, int K, int epilogue,
                  hipStream_t s, GroupedArgs grp = GroupedArgs{nullptr, nullptr, 0, 0}) {
  // grouped: M is the total row count; every expert may add one partial tile
  const int tiles_m = GROUPED ? (M + BM - 1) / BM + grp.n_experts : (M + BM - 1) / BM;
  // SwiGLU: a BN-wide tile of the stacked [2N, K] weight yields BN/2 output columns
  const int tiles_n = epilogue == EPI_SWIGLU ? (2 * N) / BN : N / BN;
  const dim3 grid(tiles_m * tiles_n), block(64 * WAVES_M * WAVES_N);
  const bf16_t* X = (const bf16_t*)x;
  const bf16_t* W = (const bf16_t*)w;
  bf16_t* Y = (bf16_t*)out;
  const bf16_t* R = (const bf16_t*)residual;
  switch (epilogue) {
    case EPI_NONE:
      gemm_kernel<BM, BN, WAVES_M, WAVES_N, EPI_NONE, PF, GROUPED><<<grid, block, 0, s>>>(X, W, Y, R, M, N, K, tiles_m, tiles_n, grp);
      break;
    case EPI_RESIDUAL:
      gemm_kernel<BM, BN, WAVES_M, WAVES_N, EPI_RESIDUAL, PF, GROUPED><<<grid, block, 0, s>>>(X, W, Y, R, M, N, K, tiles_m, tiles_n, grp);
      break;
    default:
      gemm_kernel<BM, BN, WAVES_M, WAVES_N, EPI_SWIGLU, PF, GROUPED><<<grid, block, 0, s>>>(X, W, Y, R, M, N, K, tiles_m, tiles_n, grp);
      break;
  }
  return hipGetLastError();
}

}  // namespace

// Tile choice.  0 = heuristic; 1 = 128x128; 2 = 256x128 (BM x BN); 3 = 128x256; 4 = 256x256;
// 5 = 256x256 and 6 = 256x128 with 8 wavefronts (512 threads); 7..20 = the direct-to-LDS
// kernels of gemm_dl.hip.  Every variant walks K in the
// same order with the same MFMA, so the choice never changes an output bit.  Two-segment
// operations (nf_gemm_k_segments) have their own launch forms and take the tile as a hint.
static int g_gemm_tile = 0;
void nf_set_gemm_tile(int v) { g_gemm_tile = v; }
static int g_grouped_tile = 0;  // implementation of the grouped (mixture-of-experts) GEMM; 0 = automatic
void nf_set_grouped_gemm_tile(int v) { g_grouped_tile = v; }

static int g_gemm_ksplit = 0;
void nf_set_gemm_ksplit(int v) { g_gemm_ksplit = v; }

int nf_gemm_k_segments(int N, int K, int epilogue) {
  return (epilogue != EPI_SWIGLU && K >= 8192 && K >= 2 * N && N < 8192 && K % 128 == 0 && N % 128 == 0) ? 2 : 1;
}

// Fill of the 256 CUs by `units` workgroups dealt out in whole rounds.
static double round_fill(long units) { return (double)units / (double)(((units + 255) / 256) * 256); }

// A two-segment operation.  One workgroup per tile needs no scratch and no second kernel, so
// it is the form for row counts that fill the chip; with scratch, few rows run as two
// workgroups per tile (the down projection of a 1024-row nano-batch of the 8B model has
// 128 tiles of 256x128).
static hipError_t launch_two_segments(const void* x, const void* w, void* out, const void* residual, int M, int N,
                                      int K, int epilogue, int tile, hipStream_t s, NfGemmSplit split) {
  if (g_gemm_tile) tile = g_gemm_tile;
  const long tiles = (long)((M + 255) / 256) * (N / 128);
  bool halves = false;
  if (split.partial) {
    if (g_gemm_ksplit)
      halves = g_gemm_ksplit == 2;
    else
      halves = round_fill(2 * tiles) > 1.15 * round_fill(tiles);  // the scratch traffic costs about a tenth
  }
  // Rows that fill the chip with 256x256 tiles of half K each take the four-wavefront loop
  // (measured on the 8B layer's down projection at 2048 rows: 240 -> 217 us including the
  // second kernel); its accumulators leave no room for two sums in one workgroup.
  const long units21 = 2L * ((M + 255) / 256) * (N / 256);
  const bool w4 = split.partial && K % 256 == 0 && N % 256 == 0 && g_gemm_ksplit != 1 &&
                  (tile == 21 || (tile == 0 && round_fill(units21) >= 0.9));
  if (w4) return nf_launch_gemm_dl_halves(x, w, out, residual, M, N, K, split.partial, split.seg_stride, 21, s);
  // the same loop with 128x256 tiles, when the profile asks for it (few rows)
  if ((tile == 22 || tile == 25) && split.partial && K % 256 == 0 && N % 256 == 0 && g_gemm_ksplit != 1)
    return nf_launch_gemm_dl_halves(x, w, out, residual, M, N, K, split.partial, split.seg_stride, tile, s);
  if (!halves) return nf_launch_gemm_dl_two_sums(x, w, out, residual, M, N, K, epilogue, s);
  int variant = (tile == 7 || tile == 11) ? 7 : (tile == 13 || tile == 10 || tile == 17) ? 13 : tile == 12 ? 12 : 19;
  if (variant == 13 && N % 256 != 0) variant = 12;
  return nf_launch_gemm_dl_halves(x, w, out, residual, M, N, K, split.partial, split.seg_stride, variant, s);
}

// Requires K % 64 == 0 and N % 64 == 0 (checked by the caller on the host).
hipError_t nf_launch_gemm(const void* x, const void* w, void* out, const void* residual, int M, int N, int K,
                          int epilogue, int tile, hipStream_t s, NfGemmSplit split) {
  if (M <= 0) return hipSuccess;
  if (nf_gemm_k_segments(N, K, epilogue) == 2)
    return launch_two_segments(x, w, out, residual, M, N, K, epilogue, tile, s, split);
  const int n_eff = epilogue == EPI_SWIGLU ? 2 * N : N;
  if (n_eff % 128 != 0) return launch<128, 64, 2, 2, 1>(x, w, out, residual, M, N, K, epilogue, s);
  if (g_gemm_tile) tile = g_gemm_tile;  // process-wide override for tuning runs
  if (tile == 0) {
    // No profile: pick among 256x256, 256x128 and 128x128 by (relative speed of the shape on
    // activation-like data) x sqrt(fill of the 256 CUs over whole rounds of workgroups).  The
    // square root is empirical: the chip is power-limited on these kernels, and the busy CUs
    // of a partly filled round run faster than those of a full one.
    auto score = [&](int bm, int bn, double speed) {
      if (n_eff % bn) return 0.0;
      const long tiles = (long)((M + bm - 1) / bm) * (n_eff / bn);
      const long rounds = (tiles + 255) / 256;
      return speed * sqrt((double)tiles / (double)(rounds * 256));
    };
    const double s13 = score(256, 256, 1.0), s12 = score(256, 128, 0.92), s7 = score(128, 128, 0.84);
    const double s20 = (epilogue != EPI_SWIGLU && n_eff % 192 == 0) ? score(256, 192, 0.97) : 0.0;
    // 256x256 has two loops: four wavefronts with 128x128 shares (21; needs K % 128 == 0,
    // measured 20-25 % faster) and eight wavefronts with 128x64 shares (13)
    const bool four_waves = K % 128 == 0;
    const double s21 = four_waves ? score(256, 256, 1.25) : 0.0;
    tile = (s13 >= s12 && s13 >= s7) ? 13 : (s12 >= s7 ? 19 : 7);
    if (s20 > s13 && s20 > s12 && s20 > s7) tile = 20;
    if (s21 > s20 && s21 > s12 && s21 > s7) tile = 21;
    // the same loop with 128x256 tiles, for shapes whose 256x256 tiles leave CUs idle (measured
    // on the 8B layer's O projection: 63 us against 74 with 256x128 and 83 with 256x256)
    const double s22 = four_waves ? score(128, 256, 0.95) : 0.0;
    if (s22 > s21 && s22 > s20 && s22 > s12 && s22 > s7 && s22 > s13) tile = 22;
    // and with 256x192 tiles (the 8B layer's KQV at 2048 rows: one tile per CU instead of 192 tiles)
    const double s23 = (four_waves && epilogue != EPI_SWIGLU && n_eff % 192 == 0) ? score(256, 192, 1.15) : 0.0;
    if (s23 > s22 && s23 > s21 && s23 > s20 && s23 > s12 && s23 > s7 && s23 > s13) tile = 23;
    // and with 128x192 tiles (the same operation at 1024 rows: 49 us against 51 with 128x256)
    const double s24 = s23 > 0.0 ? score(128, 192, 1.05) : 0.0;
    if (s24 > s23 && s24 > s22 && s24 > s21 && s24 > s20 && s24 > s12 && s24 > s7 && s24 > s13) tile = 24;
  }
  if (tile >= 7 && tile <= 25) {
    if (tile == 24 && (K % 128 != 0 || n_eff % 192 != 0 || epilogue == EPI_SWIGLU)) tile = 22;
    if (tile == 23 && (K % 128 != 0 || n_eff % 192 != 0 || epilogue == EPI_SWIGLU)) tile = 21;
    if ((tile == 21 || tile == 22 || tile == 25) && (K % 128 != 0 || n_eff % 256 != 0)) tile = 13;
    if (tile == 20 && (n_eff % 192 != 0 || epilogue == EPI_SWIGLU)) tile = 19;
    if (tile == 10 && n_eff % 256 != 0) tile = 9;
    if (tile == 13 && n_eff % 256 != 0) tile = 12;
    if ((tile == 15 || tile == 16) && n_eff % 256 != 0) tile = 18;
    if (tile == 17 && n_eff % 256 != 0) tile = 19;
    return nf_launch_gemm_dl(x, w, out, residual, M, N, K, epilogue, tile, s);
  }
  if ((tile == 3 || tile == 4) && n_eff % 256 != 0) tile = tile == 4 ? 2 : 1;
  switch (tile) {
    case 2: return launch<256, 128, 2, 2, 1>(x, w, out, residual, M, N, K, epilogue, s);
    case 3: return launch<128, 256, 2, 2, 1>(x, w, out, residual, M, N, K, epilogue, s);
    case 4: return launch<256, 256, 2, 2, 1>(x, w, out, residual, M, N, K, epilogue, s);
    case 5: return launch<256, 256, 2, 4, 1>(x, w, out, residual, M, N, K, epilogue, s);
    case 6: return launch<256, 128, 4, 2, 1>(x, w, out, residual, M, N, K, epilogue, s);
    default: return launch<128, 128, 2, 2, 1>(x, w, out, residual, M, N, K, epilogue, s);
  }
}

// Grouped GEMM over experts (see GroupedArgs).  rows = total routed rows; N % 64 == 0
// (N % 128 == 0 for SwiGLU counts the stacked 2N rows), K % 64 == 0.
hipError_t nf_launch_grouped_gemm(const void* x, const void* w, void* out, int rows, int N, int K, int epilogue,
                                  const int32_t* expert_offset, const int32_t* row_index, int n_experts,
                                  long long w_stride, hipStream_t s, NfGemmSplit split) {
  if (rows <= 0) return hipSuccess;
  const GroupedArgs grp{expert_offset, row_index, n_experts, w_stride};
  const int n_eff = epilogue == EPI_SWIGLU ? 2 * N : N;
  if (split.partial && epilogue == EPI_NONE && nf_gemm_k_segments(N, K, epilogue) == 2) {
    // The experts' down projection: few output columns and a long K.  Every (expert, tile)
    // splits into its two K halves, which doubles the workgroups (the 8-expert layer at 2048
    // tokens has about 320 tiles of 256x256 for 256 CUs) and halves the work a partly
    // filled tile wastes.
    int variant = g_grouped_tile == 12 ? 12 : (g_grouped_tile == 19 ? 19 : (g_grouped_tile == 13 ? 13 : 21));
    if (variant == 21 && (K % 256 != 0 || N % 256 != 0)) variant = 13;
    if (variant == 13 && N % 256 != 0) variant = 19;
    return nf_launch_gemm_dl_grouped_halves(x, w, rows, N, K, split.partial, split.seg_stride, expert_offset,
                                            row_index, n_experts, w_stride, variant, s);
  }
  if (n_eff % 128 != 0) return launch<128, 64, 2, 2, 1, true>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
  // 256x256 tiles halve the re-reads of the gathered rows; 256x128 where the width does not allow them
  int tile = g_grouped_tile ? g_grouped_tile : (n_eff % 256 == 0 ? 21 : 19);
  if (tile == 21 && (n_eff % 256 != 0 || K % 128 != 0)) tile = 13;
  if (tile == 13 && n_eff % 256 != 0) tile = 19;
  if (tile == 7 || tile == 9 || tile == 11 || tile == 12 || tile == 13 || tile == 19 || tile == 21)
    return nf_launch_gemm_dl_grouped(x, w, out, rows, N, K, epilogue, expert_offset, row_index, n_experts, w_stride,
                                     tile, s);
  return launch<128, 128, 2, 2, 1, true>(x, w, out, nullptr, rows, N, K, epilogue, s, grp);
}
