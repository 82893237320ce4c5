// Global -> register -> LDS staging of [rows][D] bf16 tiles, with the row L2 normalisation
// of Sec. 3.2 fused into the register -> LDS step (sum of squares reduced over the lanes
// that share a row with wavefront shuffles).
#pragma once
#include "device_common.h"

namespace cottn {

// A workgroup of NT threads moves a tile of C rows x D columns.  Each lane owns 8
// consecutive columns (16 bytes) of a row; D/8 neighbouring lanes share a row, so a
// wavefront reads whole 2*D-byte rows: fully coalesced.
template <int D, int C, int NT>
struct TileStage {
  static constexpr int LPR = D / 8;       // lanes per row
  static constexpr int RPP = NT / LPR;    // rows per pass
  static constexpr int PASSES = (C + RPP - 1) / RPP;
  static_assert(NT % LPR == 0, "thread count must cover whole rows");
  static_assert(C % RPP == 0 || C < RPP, "tile rows must be a multiple of rows per pass");

  uint4 regs[PASSES];

  // rows >= n_rows (end of the sequence or of the segment) read as zero
  __device__ __forceinline__ void fetch(const bf16_t* __restrict__ base, int row0, int n_rows) {
    const int tid = threadIdx.x;
    const int col = (tid % LPR) * 8;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int lr = p * RPP + tid / LPR;
      const int row = row0 + lr;
      uint4 v = {0u, 0u, 0u, 0u};
      if (lr < C && row < n_rows) v = *reinterpret_cast<const uint4*>(base + size_t(row) * D + col);
      regs[p] = v;
    }
  }

  // tile[lr][:] = x / max(||x||, eps) rounded to bf16; rinv[lr] (may be null) = 1/max(||x||, eps)
  __device__ __forceinline__ void commit_normalised(bf16_t* tile, float eps, float* rinv) const {
    const int tid = threadIdx.x;
    const int col = (tid % LPR) * 8;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int lr = p * RPP + tid / LPR;
      float f[8];
      unpack8(regs[p], f);
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
      ss = group_sum<LPR>(ss);
      const float r = inv_norm(ss, eps);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] *= r;
      if (lr < C) {
        *reinterpret_cast<uint4*>(tile + lr * lds_pitch(D) + col) = pack8(f);
        if (rinv != nullptr && col == 0) rinv[lr] = r;
      }
    }
  }

  __device__ __forceinline__ void commit_plain(bf16_t* tile) const {
    const int tid = threadIdx.x;
    const int col = (tid % LPR) * 8;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int lr = p * RPP + tid / LPR;
      if (lr < C) *reinterpret_cast<uint4*>(tile + lr * lds_pitch(D) + col) = regs[p];
    }
  }
};

// Which 16x16 tiles of a D x D fp32 accumulator matrix a wave owns, for a workgroup of NW
// waves.  The matrix is cut into (D/16)^2 tiles indexed (row tile, column tile).  A wave
// keeps one or more whole tile columns when there are fewer waves than columns (so the
// column-side operand is loaded once per wave); otherwise the waves that share a tile column
// split its row tiles.
template <int D, int NW>
struct AccTiles {
  static constexpr int DT = D / 16;
  static constexpr int NCT = (NW >= DT) ? 1 : DT / NW;      // column tiles per wave
  static constexpr int WPC = (NW >= DT) ? NW / DT : 1;      // waves per tile column
  static constexpr int NRT = (WPC >= DT) ? 1 : DT / WPC;    // row tiles per wave
  __device__ static __forceinline__ bool active(int w) { return (w / DT) * NRT < DT; }
  __device__ static __forceinline__ int col_tile(int w, int x) { return (w % DT) + x * NW; }
  __device__ static __forceinline__ int row_tile(int w, int y) {
    return (NW >= DT) ? (w / DT) * NRT + y : y;
  }
};

}  // namespace cottn
