// Pieces shared by the GEMM kernels: tile mapping, grouped-mode arguments, the epilogues.
#pragma once
#include "nf_device.h"

namespace nfgemm {

constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // bf16 elements per staged row: 144 B keeps ds_read_b128 conflict-free

// EPI_PARTIAL is internal: the fp32 sums of one K segment, written to scratch (see KRange).
enum { EPI_NONE = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_PARTIAL = 3 };

// The part of K a launch walks.  x and w rows are `ldk` elements apart (the full K of the
// operation); workgroups with blockIdx.y = s walk K elements starting at s * K.  With
// EPI_PARTIAL segment s stores its fp32 sums, row-major [M, N], at partial + s * seg_stride.
// n_first is honoured by the four-wavefront loop only.
struct KRange {
  int ldk;
  float* partial;
  long long seg_stride;
  int n_first = 0;  // output columns start at this tile column (a launch that covers a column range)
};

// Workgroup index -> tile index so that the tiles one XCD works on are consecutive
// (workgroups are dealt round-robin to the 8 XCDs; each XCD has its own L2).
__device__ __forceinline__ int xcd_remap(int b, int nblocks) {
  const int q = nblocks >> 3, r = nblocks & 7;
  const int xcd = b & 7, idx = b >> 3;
  return xcd * q + (xcd < r ? xcd : r) + idx;
}

__device__ __forceinline__ float silu_f(float a) { return a / (1.0f + __expf(-a)); }

// Grouped mode (mixture-of-experts FFN as a grouped GEMM): the M rows are the routed
// (token, expert) pairs sorted by expert; expert e owns rows [expert_offset[e],
// expert_offset[e+1]) and multiplies them with its own weight W + e * w_stride.  The row
// counts live on the device, so the grid covers the worst case and a workgroup whose
// M-tile index is past the last expert's tiles exits.  row_index (optional) gathers the
// input rows; outputs are written at the sorted row position.
struct GroupedArgs {
  const int32_t* expert_offset;
  const int32_t* row_index;
  int n_experts;
  long long w_stride;
};


// Workgroup -> (m0, n0, M limit, element offset of the expert's weight).  Returns false when a grouped workgroup has no tile.
template <int BM, int BN, bool GROUPED>
__device__ __forceinline__ bool locate_tile(int tiles_m, int tiles_n, const GroupedArgs& grp, int& m0, int& n0, int& M,
                                            size_t& w_off) {
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tm = tile % tiles_m, tn = tile / tiles_m;
  m0 = tm * BM;
  n0 = tn * BN;
  w_off = 0;
  if (GROUPED) {
    int acc_tiles = 0;
    for (int e = 0; e < grp.n_experts; ++e) {
      const int lo = grp.expert_offset[e], hi = grp.expert_offset[e + 1];
      const int nt = (hi - lo + BM - 1) / BM;
      if (tm < acc_tiles + nt) {
        m0 = lo + (tm - acc_tiles) * BM;
        M = hi;  // this expert's rows end here
        w_off = (size_t)e * (size_t)grp.w_stride;
        return true;
      }
      acc_tiles += nt;
    }
    return false;  // uniform for the whole workgroup
  }
  return true;
}

// Row of the stacked weight a tile row reads.  SwiGLU tiles alternate 32 gate rows of 32
// output columns with their 32 up rows, so both land in the same lane of the accumulators.
template <int EPI>
__device__ __forceinline__ int weight_row(int row, int n0, int N) {
  if (EPI == EPI_SWIGLU) {
    const int grp = row >> 5, within = row & 31;
    const int col = (n0 >> 1) + (grp >> 1) * 32 + within;  // output column (N = ffn inner)
    return (grp & 1) * N + col;
  }
  return n0 + row;
}

// Epilogue.  acc[i][j][v]: token row m = m0 + wm*WM + j*32 + (lane & 31);
// tile column c = wn*WN + i*32 + 8*(v/4) + 4*(lane >> 5) + (v & 3).
template <int EPI, int TM, int TN, int WM, int WN>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[TN][TM], bf16_t* __restrict__ Y,
                                           const bf16_t* __restrict__ R, int M, int N, int m0, int n0, int wm, int wn,
                                           int lane, float* __restrict__ P = nullptr) {
  const int col4 = 4 * (lane >> 5);
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int m = m0 + wm * WM + j * 32 + (lane & 31);
    if (m >= M) continue;
    if (EPI == EPI_PARTIAL) {
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const size_t off = (size_t)m * N + n0 + wn * WN + i * 32 + q * 8 + col4;
          const f32x4 o = {acc[i][j][q * 4], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
          *reinterpret_cast<f32x4*>(P + off) = o;
        }
    } else if (EPI == EPI_SWIGLU) {
      // 32-column groups come in (gate, up) pairs: acc[2p] is gate, acc[2p+1] is up
#pragma unroll
      for (int p = 0; p < TN / 2; ++p) {
        const int ocol0 = (n0 >> 1) + (wn * (TN / 2) + p) * 32;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = silu_f(acc[2 * p][j][q * 4 + e]) * acc[2 * p + 1][j][q * 4 + e];
          u32x2 pk = {pack_bf2(o[0], o[1]), pack_bf2(o[2], o[3])};
          *reinterpret_cast<u32x2*>(Y + (size_t)m * N + ocol0 + q * 8 + col4) = pk;
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < TN; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const size_t off = (size_t)m * N + n0 + wn * WN + i * 32 + q * 8 + col4;
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = acc[i][j][q * 4 + e];
          if (EPI == EPI_RESIDUAL) {
            const u32x2 r = *reinterpret_cast<const u32x2*>(R + off);
            o[0] += __uint_as_float(r[0] << 16);
            o[1] += __uint_as_float(r[0] & 0xffff0000u);
            o[2] += __uint_as_float(r[1] << 16);
            o[3] += __uint_as_float(r[1] & 0xffff0000u);
          }
          u32x2 pk = {pack_bf2(o[0], o[1]), pack_bf2(o[2], o[3])};
          *reinterpret_cast<u32x2*>(Y + off) = pk;
        }
      }
    }
  }
}

}  // namespace nfgemm
