// Global -> register -> LDS staging of [rows][D] tiles of 16-bit elements, with the row L2 norm
// of Sec. 3.2 computed on the way (sum of squares with the packed 16-bit dot instruction, reduced
// over the lanes that share a row with DPP moves).
//
// The normalisation x / max(||x||, eps) is applied element by element only where it must be.
// With r_i = 1 / max(||q_i||, eps) and r_j likewise for k_j, every product of the method is
// linear in qh_i = r_i q_i and kh_j = r_j k_j.  Where the rows of a result belong to the
// normalised operand's rows, the raw rows are the MFMA operand and the factor multiplies the
// finished fp32 result row; only an operand that is contracted over the token index is
// rescaled on its way into LDS (K in the forward and dQ passes, Q in the dK/dV pass).  A
// rescaled row has norm at most 1, so this is safe in IEEE half precision too: no row is
// ever multiplied by the factor of another row, which is 1/eps when that row is zero.
#pragma once
#include "device_common.h"

namespace cottn {

// A workgroup of NT threads moves a tile of C rows x D columns.  Each lane owns 8
// consecutive columns (16 bytes) of a row; D/8 neighbouring lanes share a row, so a
// wavefront reads whole 2*D-byte rows: fully coalesced.
__device__ __forceinline__ uint4 load_rows(const e16_t* p, bool stream) {
  if (stream) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return uint4{v.x, v.y, v.z, v.w};
  }
  return *reinterpret_cast<const uint4*>(p);
}

template <int D, int C, int NT>
struct TileStage {
  static constexpr int LPR = D / 8;       // lanes per row
  static constexpr int RPP = NT / LPR;    // rows per pass
  static constexpr int PASSES = (C + RPP - 1) / RPP;
  static_assert(NT % LPR == 0, "thread count must cover whole rows");
  static_assert(C % RPP == 0 || C < RPP, "tile rows must be a multiple of rows per pass");

  uint4 regs[PASSES];

  // rows >= n_rows (end of the sequence or of the segment) read as zero; `stream` (uniform
  // over the workgroup) marks the loads non-temporal: rows nothing will find in a cache again
  __device__ __forceinline__ void fetch(const e16_t* __restrict__ base, int row0, int n_rows,
                                        bool stream = false) {
    const int tid = threadIdx.x;
    const int col = (tid % LPR) * 8;
    const e16_t* p0 = base + size_t(row0) * D + (tid / LPR) * D + col;
    if (C % RPP == 0 && row0 + C <= n_rows) {
      // whole tile in range (workgroup-uniform): plain loads at constant strides
#pragma unroll
      for (int p = 0; p < PASSES; ++p)
        regs[p] = load_rows(p0 + p * RPP * D, stream);
      return;
    }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int lr = p * RPP + tid / LPR;
      uint4 v = {0u, 0u, 0u, 0u};
      if (lr < C && row0 + lr < n_rows) v = load_rows(p0 + p * RPP * D, stream);
      regs[p] = v;
    }
  }

  // rinv[p] = min(1/||row||, inv_eps) = 1 / max(||row||, eps) for the row this lane holds in
  // pass p (every lane of the row gets the same value).
  __device__ __forceinline__ void row_rinv(float inv_eps, float* rinv) const {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      float ss = 0.f;
      const uint32_t w[4] = {regs[p].x, regs[p].y, regs[p].z, regs[p].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        ss = dot2_self(w[e], ss);
      }
      ss = group_sum<LPR>(ss);
      rinv[p] = fminf(__builtin_amdgcn_rsqf(ss), inv_eps);
    }
  }

  // out[local row] = rinv of that row (one lane per row writes)
  __device__ __forceinline__ void store_rinv(float* out, const float* rinv) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int lr = p * RPP + tid / LPR;
      if ((C % RPP == 0 || lr < C) && (tid % LPR) == 0) out[lr] = rinv[p];
    }
  }

  // tile[lr][:] = row / max(||row||, eps) rounded to the element type; rinv_out[lr] (may be null) = that
  // factor.  For the places that need the normalised rows themselves as an operand.
  __device__ __forceinline__ void commit_normalised(e16_t* tile, float eps, float* rinv_out) const {
    float rinv[PASSES];
    row_rinv(1.0f / eps, rinv);
    commit_scaled(tile, rinv);
    if (rinv_out != nullptr) store_rinv(rinv_out, rinv);
  }

  __device__ __forceinline__ void commit_plain(e16_t* tile) const {
    const int tid = threadIdx.x;
    const int col = (tid % LPR) * 8;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int lr = p * RPP + tid / LPR;
      if (C % RPP == 0 || lr < C) *reinterpret_cast<uint4*>(tile + lr * tile_pitch(D, C) + col) = regs[p];
    }
  }

  // tile[lr][:] = scale[p] * row, rounded to the element type
  __device__ __forceinline__ void commit_scaled(e16_t* tile, const float* scale) const {
    const int tid = threadIdx.x;
    const int col = (tid % LPR) * 8;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      const int lr = p * RPP + tid / LPR;
      float f[8];
      unpack8(regs[p], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] *= scale[p];
      if (C % RPP == 0 || lr < C) *reinterpret_cast<uint4*>(tile + lr * tile_pitch(D, C) + col) = pack8(f);
    }
  }
};

// Which 16x16 tiles of a DR x DC fp32 accumulator matrix a wave owns, for a workgroup of NW
// waves.  The matrix is cut into (DR/16) x (DC/16) tiles indexed (row tile, column tile).  A
// wave keeps one or more whole tile columns when there are fewer waves than columns (so the
// column-side operand is loaded once per wave); otherwise the waves that share a tile column
// split its row tiles.  (The state K^T V is d_key x d_value; which of the two is the row side
// depends on the kernel's accumulator orientation.)
template <int DR, int DC, int NW>
struct AccTiles {
  static constexpr int RT = DR / 16, CT = DC / 16;
  static constexpr int NCT = (NW >= CT) ? 1 : CT / NW;      // column tiles per wave
  static constexpr int WPC = (NW >= CT) ? NW / CT : 1;      // waves per tile column
  static constexpr int NRT = (WPC >= RT) ? 1 : RT / WPC;    // row tiles per wave
  // stored states a wave loads at once when it seeds its accumulators (register budget)
  static constexpr int STATE_BATCH = NCT * NRT <= 4 ? 3 : NCT * NRT <= 8 ? 2 : 1;
  __device__ static __forceinline__ bool active(int w) { return (w / CT) * NRT < RT; }
  __device__ static __forceinline__ int col_tile(int w, int x) { return (w % CT) + x * NW; }
  __device__ static __forceinline__ int row_tile(int w, int y) {
    return (NW >= CT) ? (w / CT) * NRT + y : y;
  }
};

// The same ownership when the C/16 row groups of a chunk are each served by CS waves that
// split the result columns between them (wave = (row group rg, column part cp)).  CS = 1 is
// AccTiles over the row groups.  CS > 1 (square matrices only): a wave owns the key tiles rg,
// rg + RG, ... and the value tiles of its own column part, which are the tiles whose V
// fragments it reads anyway.
template <int DR, int DC, int RG, int CS>
struct SplitTiles {
  using One = AccTiles<DR, DC, RG>;
  static_assert(CS == 1 || DR == DC, "column parts are implemented for square matrices");
  static constexpr int DT = DC / 16;
  static constexpr int NCT = CS == 1 ? One::NCT : (RG >= DT ? 1 : DT / RG);
  static constexpr int NRT = CS == 1 ? One::NRT : DT / CS;
  // whether the row-side operand of the state update is among the V fragments of the wave's
  // output columns (else it is read separately)
  static constexpr bool ROW_OPERAND_IS_OUTPUT_V = CS == 1 ? One::WPC == 1 : true;
  static constexpr int STATE_BATCH = NCT * NRT <= 4 ? 3 : NCT * NRT <= 8 ? 2 : 1;
  static_assert(CS == 1 || DT % CS == 0, "column parts must be whole tiles");
  __device__ static __forceinline__ bool active(int rg, int cp) {
    return CS == 1 ? One::active(rg) : rg < DT;
  }
  __device__ static __forceinline__ int col_tile(int rg, int cp, int x) {
    return CS == 1 ? One::col_tile(rg, x) : rg % DT + x * RG;
  }
  __device__ static __forceinline__ int row_tile(int rg, int cp, int y) {
    return CS == 1 ? One::row_tile(rg, y) : cp * NRT + y;
  }
};

// acc += the wave's tiles of the stored states first..last, `load(state, x, y)` returning
// tile (x, y) of one of them.  States are taken BATCH at a time with every load of a batch
// issued before the first addition, so a batch costs one memory latency, not one per state.
// Slots of the last batch beyond `last` re-read `last` (an address already in flight) and
// are discarded.
template <int BATCH, int NCT, int NRT, class LoadTile>
__device__ __forceinline__ void add_stored_states(f32x4 (&acc)[NCT][NRT], int first, int last,
                                                  LoadTile load) {
  for (int base = first; base <= last; base += BATCH) {
    f32x4 t[BATCH][NCT][NRT];
#pragma unroll
    for (int i = 0; i < BATCH; ++i)
#pragma unroll
      for (int x = 0; x < NCT; ++x)
#pragma unroll
        for (int y = 0; y < NRT; ++y) t[i][x][y] = load(min(base + i, last), x, y);
#pragma unroll
    for (int i = 0; i < BATCH; ++i) {
      const bool keep = base + i <= last;
#pragma unroll
      for (int x = 0; x < NCT; ++x)
#pragma unroll
        for (int y = 0; y < NRT; ++y)
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[x][y][v] += keep ? t[i][x][y][v] : 0.f;
    }
  }
}

// A wave's finished result block (16 rows x NTILES*16 columns, by default all D columns) as
// whole 16-byte pieces of rows, one or more per lane, ready for coalesced global stores.
template <int D, int NTILES = D / 16>
struct RowPieces {
  static constexpr int PPR = 2 * NTILES;     // 16-byte pieces per row
  static constexpr int PIECES = 16 * PPR;    // in the wave's 16 rows
  static constexpr int PER_LANE = (PIECES + 63) / 64;
  uint4 v[PER_LANE];
};

// Turns a wave's result block whose accumulators are laid out TRANSPOSED (acc[nt][v] =
// result[row r][column col0 + 16 nt + 4 q4 + v], i.e. each lane holds 4 consecutive columns
// of one row) into row pieces: scales by the per-lane row factor, rounds to the element type, passes the
// block through a staging area private to the wave (16 rows of lds_pitch(D) elements from
// stage_rows on, columns col0..; it fits the wave's 16 rows of an operand tile, whose pitch is
// larger) with 8-byte writes and reads it back as 16-byte pieces.
template <int D, int NTILES = D / 16>
__device__ __forceinline__ void gather_rows_transposed(const f32x4* acc, float row_factor,
                                                       e16_t* stage_rows, int l,
                                                       RowPieces<D, NTILES>& out, int col0 = 0) {
  using RP = RowPieces<D, NTILES>;
  constexpr int PITCH = lds_pitch(D);
  const int r = l % 16, q4 = l / 16;
#pragma unroll
  for (int nt = 0; nt < NTILES; ++nt) {
    uint2 pk;
    pk.x = pack2(row_factor * acc[nt][0], row_factor * acc[nt][1]);
    pk.y = pack2(row_factor * acc[nt][2], row_factor * acc[nt][3]);
    *reinterpret_cast<uint2*>(stage_rows + r * PITCH + col0 + 16 * nt + 4 * q4) = pk;
  }
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < RP::PER_LANE; ++j) {
    const int i = l + 64 * j;
    const int lr = i / RP::PPR, col = col0 + (i % RP::PPR) * 8;
    if (RP::PIECES % 64 == 0 || i < RP::PIECES)
      out.v[j] = *reinterpret_cast<const uint4*>(stage_rows + lr * PITCH + col);
  }
}

// Writes the pieces to rows first_row.. (columns col0..) of dst; rows at or beyond row_end are
// not written.  The scan kernels call this one chunk late (after the next chunk's loads have
// been issued): the wait for those loads at the top of a chunk step is a wait for every
// outstanding memory operation, and must not find stores that were issued a moment ago.
template <int D, int NTILES = D / 16>
__device__ __forceinline__ void store_row_pieces(const RowPieces<D, NTILES>& p,
                                                 e16_t* __restrict__ dst, int first_row,
                                                 int row_end, int l, int col0 = 0) {
  using RP = RowPieces<D, NTILES>;
#pragma unroll
  for (int j = 0; j < RP::PER_LANE; ++j) {
    const int i = l + 64 * j;
    const int lr = i / RP::PPR, col = col0 + (i % RP::PPR) * 8;
    const int row = first_row + lr;
    if ((RP::PIECES % 64 == 0 || i < RP::PIECES) && row < row_end)
      store_streaming(dst + size_t(row) * D + col, p.v[j]);
  }
}

// Both at once, for the kernels that do not defer their stores.
template <int D>
__device__ __forceinline__ void store_rows_transposed(const f32x4* acc, float row_factor,
                                                      e16_t* stage_rows, e16_t* __restrict__ dst,
                                                      int first_row, int row_end, int l) {
  RowPieces<D> p;
  gather_rows_transposed<D>(acc, row_factor, stage_rows, l, p);
  store_row_pieces<D>(p, dst, first_row, row_end, l);
}

// Sum of x over the four 16-lane rows of the wave (lanes r, r+16, r+32, r+48); every lane
// gets the total of its column.
__device__ __forceinline__ float sum_over_lane_rows(float x) {
  x += __shfl_xor(x, 16, 64);
  x += __shfl_xor(x, 32, 64);
  return x;
}

// Chain rule through the row normalisation on a wave's transposed 16 x D block:
// acc[nt][v] = dxh[row r][column 16 nt + 4 q4 + v].  Reads the row from `x_rows` (the wave's
// 16 rows of its LDS tile, row pitch PITCH), which holds either the raw row x (NORMALISED = false) or
// xh = r x (true); forms the dot product with dxh over the whole row (16 columns per lane,
// then across the four lane rows) and replaces acc by dxh - xh (xh . dxh)  (no projection
// for rows at or below eps).  Returns xh . dxh.
template <int D, int PITCH, bool NORMALISED>
__device__ __forceinline__ float project_out_row(f32x4* acc, const e16_t* x_rows, float rinv,
                                                 float inv_eps, int r, int q4) {
  constexpr int DT = D / 16;
  float xv[DT][4];
  float t = 0.f;
#pragma unroll
  for (int nt = 0; nt < DT; ++nt) {
    const uint2 raw = *reinterpret_cast<const uint2*>(x_rows + r * PITCH + 16 * nt + 4 * q4);
    unpack2(raw.x, xv[nt][0], xv[nt][1]);
    unpack2(raw.y, xv[nt][2], xv[nt][3]);
#pragma unroll
    for (int v = 0; v < 4; ++v) t += xv[nt][v] * acc[nt][v];
  }
  t = sum_over_lane_rows(t);
  const float c = (rinv == inv_eps) ? 0.f : (NORMALISED ? t : rinv * rinv * t);
#pragma unroll
  for (int nt = 0; nt < DT; ++nt)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[nt][v] -= xv[nt][v] * c;
  return NORMALISED ? t : rinv * t;
}

}  // namespace cottn
