// Causal cosine attention forward, bf16 storage / bf16 MFMA / fp32 accumulation (gfx950).
//
// Sec. 4 eq. attn_2 writes the causal output as an inclusive cumulative sum over the sequence
// of the outer products kh_j^T v_j, contracted with qh_i.  Regrouping that sum exactly:
//   * the sequence of one (batch, head) is cut into G segments, each a whole number of chunks
//     of C rows;
//   * kernel 1 (segment totals) reduces kh^T v over every segment but the last;
//   * kernel 2 (carry) turns the totals into exclusive prefixes: the state at each segment start;
//   * kernel 3 (scan) walks the chunks of its segment with the d x d state in fp32
//     accumulators:  O_c = s_h [ (Qh_c Kh_c^T (.) M) V_c + Qh_c S ],  S += Kh_c^T V_c,
//     where the first term is eq. attn_1 restricted to the chunk.
// With G = 1 only the scan kernel runs; with one chunk per segment this is the fully
// chunk-parallel form.
//
// Work split inside the scan workgroup (C/16 waves): wave w owns query rows 16w..16w+15 of
// the chunk for the output, and a fixed set of 16x16 tiles of the state for the update.
// Tiles of normalised Q, K and raw V sit row-major in LDS; operands whose contraction
// index is the token are read with the transposing LDS read, so no transposed copy is kept.
// The masked similarity tile is produced as P^T = Kh Qh^T, whose accumulator layout is
// exactly the A-operand layout of the following P V product (with the token slots
// permuted the same way on the V side), so P never touches LDS.
#include "device_common.h"
#include "launch.h"
#include "tile_io.h"

namespace cottn {
namespace {

template <int D, int C>
struct FwdCfg {
  static constexpr int NW = C / 16;
  static constexpr int NT = NW * 64;
  static constexpr int DT = D / 16;
  static constexpr int KS = D / 32;     // k steps of a contraction over the feature dim
  static constexpr int PITCH = lds_pitch(D);
  static constexpr int TILE = C * PITCH;            // elements of one [C][D] LDS tile
  static constexpr int STATE = D * PITCH;           // elements of the [D][D] bf16 state copy
};

// ---------------------------------------------------------------------------------------
// Kernel 1: T[unit][g] = sum over the rows of segment g of kh^T v   (fp32, [d_key][d_value])
// grid = units * n_compute workgroups; segment g of a unit writes slot g of the unit's
// n_slots slots.  The causal forward computes all segments but the last (n_compute =
// n_slots - 1), the bidirectional forward all of them.
template <int D, int C>
__global__ __launch_bounds__(C * 4) void fwd_segment_state_bf16(
    const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, float* __restrict__ seg_state,
    int N, int n_slots, int n_compute, int seg_rows, float eps) {
  using Cfg = FwdCfg<D, C>;
  using ST = AccTiles<D, Cfg::NW>;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[Cfg::TILE];

  const int unit = blockIdx.x / n_compute, g = blockIdx.x % n_compute;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64, r = l % 16, q4 = l / 16;
  const bf16_t* Ku = K + size_t(unit) * N * D;
  const bf16_t* Vu = V + size_t(unit) * N * D;
  const int row_begin = g * seg_rows;
  const int row_end = min(N, row_begin + seg_rows);

  f32x4 acc[ST::NCT][ST::NRT];
#pragma unroll
  for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
    for (int y = 0; y < ST::NRT; ++y) acc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};

  TileStage<D, C, Cfg::NT> kst, vst;
  kst.fetch(Ku, row_begin, row_end);
  vst.fetch(Vu, row_begin, row_end);
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    __syncthreads();  // previous chunk's reads of Ks/Vs are done
    kst.commit_normalised(Ks, eps, nullptr);
    vst.commit_plain(Vs);
    if (row0 + C < row_end) {
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
    }
    __syncthreads();
    if (ST::active(w)) {
#pragma unroll
      for (int p = 0; p < C / 32; ++p) {
        bf16x8 bv[ST::NCT];
#pragma unroll
        for (int x = 0; x < ST::NCT; ++x)
          bv[x] = lds_col_frag(Vs, Cfg::PITCH, 32 * p + 8 * q4, 32 * p + 8 * q4 + 4,
                               16 * ST::col_tile(w, x), r);
#pragma unroll
        for (int y = 0; y < ST::NRT; ++y) {
          bf16x8 ak = lds_col_frag(Ks, Cfg::PITCH, 32 * p + 8 * q4, 32 * p + 8 * q4 + 4,
                                   16 * ST::row_tile(w, y), r);
#pragma unroll
          for (int x = 0; x < ST::NCT; ++x) acc[x][y] = mma16(ak, bv[x], acc[x][y]);
        }
      }
    }
  }
  if (ST::active(w)) {
    float* out = seg_state + (size_t(unit) * n_slots + g) * D * D;
#pragma unroll
    for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
      for (int y = 0; y < ST::NRT; ++y)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          out[(16 * ST::row_tile(w, y) + 4 * q4 + v) * D + 16 * ST::col_tile(w, x) + r] =
              acc[x][y][v];
  }
}

// ---------------------------------------------------------------------------------------
// Kernel 2: in place, per (unit, element): slot g <- sum of slots < g (exclusive prefix
// along the segment axis); slot n_slots-1 never held a total and only receives its prefix.
__global__ __launch_bounds__(256) void fwd_state_carry(float* __restrict__ seg_state, int n_slots,
                                                       int elems_per_state, long total) {
  const long idx = long(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= total) return;
  const long unit = idx / elems_per_state, e = idx % elems_per_state;
  float* p = seg_state + unit * n_slots * elems_per_state + e;
  float run = 0.f;
  for (int g = 0; g < n_slots; ++g) {
    const float t = (g + 1 < n_slots) ? p[size_t(g) * elems_per_state] : 0.f;
    p[size_t(g) * elems_per_state] = run;
    run += t;
  }
}

// ---------------------------------------------------------------------------------------
// Kernel 3: the chunk scan of one segment.
template <int D, int C>
__global__ __launch_bounds__(C * 4) void fwd_causal_scan_bf16(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ s, bf16_t* __restrict__ O, float* __restrict__ state_out,
    const float* __restrict__ seg_prefix, int H, int N, int G, int seg_rows, float eps) {
  using Cfg = FwdCfg<D, C>;
  using ST = AccTiles<D, Cfg::NW>;
  constexpr int PITCH = Cfg::PITCH;
  __shared__ __attribute__((aligned(16))) bf16_t Qs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Ks[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t St[Cfg::STATE];  // [d_value][d_key]

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64, r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const bf16_t* Qu = Q + ubase;
  const bf16_t* Ku = K + ubase;
  const bf16_t* Vu = V + ubase;
  bf16_t* Ou = O + ubase;
  const float scale = s[unit % H];
  const int row_begin = g * seg_rows;
  const int row_end = min(N, row_begin + seg_rows);

  // running state in fp32 accumulators, seeded with the segment's prefix
  f32x4 sacc[ST::NCT][ST::NRT];
  const float* init = (seg_prefix != nullptr && g > 0)
                          ? seg_prefix + (size_t(unit) * G + g) * D * D : nullptr;
#pragma unroll
  for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
    for (int y = 0; y < ST::NRT; ++y)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        sacc[x][y][v] = (init != nullptr && ST::active(w))
            ? init[(16 * ST::row_tile(w, y) + 4 * q4 + v) * D + 16 * ST::col_tile(w, x) + r] : 0.f;

  TileStage<D, C, Cfg::NT> qst, kst, vst;
  qst.fetch(Qu, row_begin, row_end);
  kst.fetch(Ku, row_begin, row_end);
  vst.fetch(Vu, row_begin, row_end);

  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    // ---- publish the state (bf16, transposed) and this chunk's tiles
    if (ST::active(w)) {
#pragma unroll
      for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
        for (int y = 0; y < ST::NRT; ++y) {
          uint2 pk;
          pk.x = pack_bf16(sacc[x][y][0], sacc[x][y][1]);
          pk.y = pack_bf16(sacc[x][y][2], sacc[x][y][3]);
          *reinterpret_cast<uint2*>(St + (16 * ST::col_tile(w, x) + r) * PITCH +
                                    16 * ST::row_tile(w, y) + 4 * q4) = pk;
        }
    }
    qst.commit_normalised(Qs, eps, nullptr);
    kst.commit_normalised(Ks, eps, nullptr);
    vst.commit_plain(Vs);
    if (row0 + C < row_end) {
      qst.fetch(Qu, row0 + C, row_end);
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
    }
    __syncthreads();

    // ---- output rows 16w..16w+15 of the chunk
    bf16x8 qf[Cfg::KS];  // Qh rows of this wave: B operand of P^T, A operand of Qh S
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks)
      qf[ks] = lds_row_frag(Qs + (16 * w + r) * PITCH + 32 * ks + 8 * q4);

    f32x4 oacc[Cfg::DT];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt) oacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // inter-chunk part: Qh S_prev  (contraction over d_key; St rows are d_value)
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks)
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt)
        oacc[nt] = mma16(qf[ks], lds_row_frag(St + (16 * nt + r) * PITCH + 32 * ks + 8 * q4),
                         oacc[nt]);

    // intra-chunk part, two key tiles (32 tokens) at a time
#pragma unroll
    for (int p = 0; p < Cfg::NW / 2; ++p) {
      if (2 * p <= w) {  // wave-uniform: key tiles above the diagonal are all masked
        bf16x8 pf = zero_frag();
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int jt = 2 * p + half;
          if (jt <= w) {
            f32x4 pacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < Cfg::KS; ++ks)
              pacc = mma16(lds_row_frag(Ks + (16 * jt + r) * PITCH + 32 * ks + 8 * q4), qf[ks],
                           pacc);
            // pacc[v] = P[query 16w + r][key 16jt + 4*q4 + v]; diagonal tile: keep key <= query
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const bool keep = (jt < w) || (4 * q4 + v <= r);
              pf[4 * half + v] = static_cast<__bf16>(keep ? pacc[v] : 0.f);
            }
          }
        }
        // k slot (q4, e) of pf is token 32p + 16*(e/4) + 4*q4 + e%4: read V the same way
#pragma unroll
        for (int nt = 0; nt < Cfg::DT; ++nt)
          oacc[nt] = mma16(pf, lds_col_frag(Vs, PITCH, 32 * p + 4 * q4, 32 * p + 16 + 4 * q4,
                                            16 * nt, r),
                           oacc[nt]);
      }
    }

    // ---- state update S += Kh^T V over the chunk's tokens
    if (ST::active(w)) {
#pragma unroll
      for (int p = 0; p < C / 32; ++p) {
        bf16x8 bv[ST::NCT];
#pragma unroll
        for (int x = 0; x < ST::NCT; ++x)
          bv[x] = lds_col_frag(Vs, PITCH, 32 * p + 8 * q4, 32 * p + 8 * q4 + 4,
                               16 * ST::col_tile(w, x), r);
#pragma unroll
        for (int y = 0; y < ST::NRT; ++y) {
          bf16x8 ak = lds_col_frag(Ks, PITCH, 32 * p + 8 * q4, 32 * p + 8 * q4 + 4,
                                   16 * ST::row_tile(w, y), r);
#pragma unroll
          for (int x = 0; x < ST::NCT; ++x) sacc[x][y] = mma16(ak, bv[x], sacc[x][y]);
        }
      }
    }

    // ---- store O: through this wave's own (now dead) rows of Qs for 16-byte row writes
    wave_lds_sync();
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        Qs[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r] = f32_to_bf16(scale * oacc[nt][v]);
    wave_lds_sync();
    constexpr int PIECES = 16 * D / 8;  // 16-byte pieces in this wave's 16 rows
#pragma unroll
    for (int i = l; i < PIECES; i += 64) {
      const int lr = i / (D / 8), col = (i % (D / 8)) * 8;
      const int row = row0 + 16 * w + lr;
      if (row < row_end)
        *reinterpret_cast<uint4*>(Ou + size_t(row) * D + col) =
            *reinterpret_cast<const uint4*>(Qs + (16 * w + lr) * PITCH + col);
    }
    __syncthreads();  // all reads of Ks, Vs, St done before the next chunk overwrites them
  }

  if (state_out != nullptr && g == G - 1 && ST::active(w)) {
    float* out = state_out + size_t(unit) * D * D;
#pragma unroll
    for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
      for (int y = 0; y < ST::NRT; ++y)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          out[(16 * ST::row_tile(w, y) + 4 * q4 + v) * D + 16 * ST::col_tile(w, x) + r] =
              sacc[x][y][v];
  }
}

template <int D, int C>
hipError_t run_fwd_causal(const CausalArgs& a) {
  using Cfg = FwdCfg<D, C>;
  const int units = a.B * a.H;
  const bf16_t* Q = static_cast<const bf16_t*>(a.Q);
  const bf16_t* K = static_cast<const bf16_t*>(a.K);
  const bf16_t* V = static_cast<const bf16_t*>(a.V);
  float* ws = static_cast<float*>(a.workspace);  // [units][G][D][D] when G > 1
  hipError_t err = hipSuccess;
  if (a.G > 1) {
    err = launch("fwd_segment_state_bf16", a.stream, [&] {
      fwd_segment_state_bf16<D, C><<<units * (a.G - 1), Cfg::NT, 0, a.stream>>>(
          K, V, ws, a.N, a.G, a.G - 1, a.seg_rows, a.eps);
    });
    if (err != hipSuccess) return err;
    err = launch_fwd_state_carry(ws, units, a.G, D * D, a.stream);
    if (err != hipSuccess) return err;
  }
  return launch("fwd_causal_scan_bf16", a.stream, [&] {
    fwd_causal_scan_bf16<D, C><<<units * a.G, Cfg::NT, 0, a.stream>>>(
        Q, K, V, a.s, static_cast<bf16_t*>(a.O), a.state, a.G > 1 ? ws : nullptr, a.H, a.N, a.G,
        a.seg_rows, a.eps);
  });
}

}  // namespace

hipError_t launch_fwd_state_carry(float* seg_state, int units, int G, int elems, hipStream_t st) {
  const long total = long(units) * elems;
  return launch("fwd_state_carry", st, [&] {
    fwd_state_carry<<<unsigned((total + 255) / 256), 256, 0, st>>>(seg_state, G, elems, total);
  });
}

hipError_t fwd_causal_bf16(const CausalArgs& a) {
  switch (a.d * 1000 + a.C) {
    case 32064: return run_fwd_causal<32, 64>(a);
    case 32128: return run_fwd_causal<32, 128>(a);
    case 32256: return run_fwd_causal<32, 256>(a);
    case 64064: return run_fwd_causal<64, 64>(a);
    case 64128: return run_fwd_causal<64, 128>(a);
    case 64256: return run_fwd_causal<64, 256>(a);
    case 128064: return run_fwd_causal<128, 64>(a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cottn
