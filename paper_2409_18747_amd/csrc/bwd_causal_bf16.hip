// Causal cosine attention backward, bf16 storage / bf16 MFMA / fp32 accumulation (gfx950).
//
// Sec. 4 gives, for the normalised operands Qh, Kh (A = dO V^T, P = Qh Kh^T, M the
// lower-triangular mask),
//     dQh = (A (.) M) Kh,    dKh = (A (.) M)^T Qh,    dV = (P (.) M)^T dO,
// and notes that dQh is a cumulative sum running forward in time while dKh and dV use one
// running backward.  With S_t = sum_{j<=t} kh_j^T v_j and R_t = sum_{i>=t} qh_i^T dO_i:
//     dqh_t = s dO_t S_t^T,    dkh_t = s v_t R_t^T,    dv_t = s kh_t R_t.
// Both sums are regrouped exactly into chunks of C rows inside G segments per (batch, head):
//   kernel 1  per-segment totals of Kh^T V (forward states) and Qh^T dO (reverse states),
//             both stored [d_key][d_value];
//   kernel 2  exclusive prefix of the first and exclusive suffix of the second along the
//             segment axis;
//   kernel 3  forward-time scan: dQ of a segment, chunk by chunk, first to last;
//   kernel 4  reverse-time scan: dK and dV of a segment, chunk by chunk, last to first;
//   kernel 5  ds[h] from per-workgroup partial sums.
// The chain rule through x/max(||x||, eps) (dx = r (dxh - xh (xh . dxh)), r = 1/||x||; rows
// at or below eps: dx = dxh/eps) and the scale s_h are applied in the scan kernels'
// epilogues, on the fp32 accumulators.  ds_h = sum over rows of qh_i . dqh_i before scaling.
//
// Inside a chunk the masked A and P tiles are produced directly in the register layout the
// next product needs as its A operand (A^T = V dO^T for dQ; A and P themselves for dK, dV),
// so they never pass through LDS; operands contracted over the token index are read from
// the row-major LDS tiles with the transposing LDS read, and the fragments read for the
// intra-chunk products are reused as operands of the state updates.  Scheduling follows
// the same two rules as the forward file: all LDS reads of a group of MFMAs are issued
// first, and registers are capped for three workgroups per compute unit.
#include "device_common.h"
#include "launch.h"
#include "tile_io.h"
#include "workspace.h"

namespace cottn {
namespace {

template <int D, int C>
struct BwdCfg {
  static constexpr int NW = C / 16;
  static constexpr int NT = NW * 64;
  static constexpr int DT = D / 16;
  static constexpr int KS = D / 32;
  static constexpr int NP = C / 32;
  static constexpr int PITCH = lds_pitch(D);
  static constexpr int TILE = C * PITCH;
  static constexpr int STATE = D * PITCH;
  static constexpr int LDS_BYTES = 2 * (4 * TILE + STATE) + 4 * C + 64;
  static constexpr int WG_PER_CU = (160 * 1024) / LDS_BYTES;
  static constexpr bool PREFETCH = true;
  static constexpr int WAVES_RAW = (WG_PER_CU >= 2 ? 2 : 1) * NW / 4;
  static constexpr int WAVES_PER_EU = WAVES_RAW > 4 ? 4 : WAVES_RAW;
};

// pack a masked accumulator tile into half of an A-operand fragment
__device__ __forceinline__ void put_half(bf16x8& frag, int half, f32x4 acc, bool k0, bool k1,
                                         bool k2, bool k3) {
  frag[4 * half + 0] = static_cast<__bf16>(k0 ? acc[0] : 0.f);
  frag[4 * half + 1] = static_cast<__bf16>(k1 ? acc[1] : 0.f);
  frag[4 * half + 2] = static_cast<__bf16>(k2 ? acc[2] : 0.f);
  frag[4 * half + 3] = static_cast<__bf16>(k3 ? acc[3] : 0.f);
}

// ---------------------------------------------------------------------------------------
// Kernel 1: per-segment totals, both [d_key][d_value]:
//   fwd_tot[unit][g] = sum_rows kh^T v   (needed by later segments: computed for g < G-1)
//   rev_tot[unit][g] = sum_rows qh^T dO  (needed by earlier segments: computed for g > 0)
template <int D, int C>
__global__ __launch_bounds__(C * 4) void bwd_segment_states_bf16(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, float* __restrict__ fwd_tot, float* __restrict__ rev_tot,
    int N, int G, int seg_rows, float eps) {
  using Cfg = BwdCfg<D, C>;
  using AT = AccTiles<D, Cfg::NW>;
  constexpr int PITCH = Cfg::PITCH;
  __shared__ __attribute__((aligned(16))) bf16_t Xs[Cfg::TILE];  // Kh or Qh
  __shared__ __attribute__((aligned(16))) bf16_t Ys[Cfg::TILE];  // V  or dO

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const int row_begin = g * seg_rows;
  const int row_end = min(N, row_begin + seg_rows);

#pragma unroll 1
  for (int which = 0; which < 2; ++which) {
    if (which == 0 ? (g >= G - 1) : (g == 0)) continue;
    const bf16_t* X = (which == 0 ? K : Q) + ubase;
    const bf16_t* Y = (which == 0 ? V : dO) + ubase;
    float* out = (which == 0 ? fwd_tot : rev_tot) + (size_t(unit) * G + g) * D * D;

    // acc[x][y]: rows = features of X (row tile y), columns = features of Y (col tile x)
    f32x4 acc[AT::NCT][AT::NRT];
#pragma unroll
    for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
      for (int y = 0; y < AT::NRT; ++y) acc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};

    TileStage<D, C, Cfg::NT> xst, yst;
    for (int row0 = row_begin; row0 < row_end; row0 += C) {
      xst.fetch(X, row0, row_end);
      yst.fetch(Y, row0, row_end);
      __syncthreads();
      xst.commit_normalised(Xs, eps, nullptr);
      yst.commit_plain(Ys);
      __syncthreads();
      if (AT::active(w)) {
#pragma unroll
        for (int p = 0; p < Cfg::NP; ++p) {
          const int k0 = 32 * p + 8 * q4;
          bf16x8 by[AT::NCT], ax[AT::NRT];
#pragma unroll
          for (int x = 0; x < AT::NCT; ++x)
            by[x] = lds_col_frag(Ys, PITCH, k0, k0 + 4, 16 * AT::col_tile(w, x), r);
#pragma unroll
          for (int y = 0; y < AT::NRT; ++y)
            ax[y] = lds_col_frag(Xs, PITCH, k0, k0 + 4, 16 * AT::row_tile(w, y), r);
          __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
          for (int y = 0; y < AT::NRT; ++y)
#pragma unroll
            for (int x = 0; x < AT::NCT; ++x) acc[x][y] = mma16(ax[y], by[x], acc[x][y]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (AT::active(w)) {
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            out[(16 * AT::row_tile(w, y) + 4 * q4 + v) * D + 16 * AT::col_tile(w, x) + r] =
                acc[x][y][v];
    }
  }
}

// ---------------------------------------------------------------------------------------
// Kernel 2: blockIdx.y == 0: slot g <- sum of fwd totals of segments < g;
//           blockIdx.y == 1: slot g <- sum of rev totals of segments > g.
// Totals that were never computed (fwd slot G-1, rev slot 0) are not read.
__global__ __launch_bounds__(256) void bwd_state_carry(float* __restrict__ fwd_tot,
                                                       float* __restrict__ rev_tot, int G,
                                                       int elems_per_state, long total) {
  const long idx = long(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= total) return;
  const long unit = idx / elems_per_state, e = idx % elems_per_state;
  float run = 0.f;
  if (blockIdx.y == 0) {
    float* p = fwd_tot + unit * G * elems_per_state + e;
    for (int g = 0; g < G; ++g) {
      const float t = (g + 1 < G) ? p[size_t(g) * elems_per_state] : 0.f;
      p[size_t(g) * elems_per_state] = run;
      run += t;
    }
  } else {
    float* p = rev_tot + unit * G * elems_per_state + e;
    for (int g = G - 1; g >= 0; --g) {
      const float t = (g > 0) ? p[size_t(g) * elems_per_state] : 0.f;
      p[size_t(g) * elems_per_state] = run;
      run += t;
    }
  }
}

// ---------------------------------------------------------------------------------------
// Kernel 3: dQ of one segment, chunks in forward order.  Wave w owns query rows 16w..16w+15.
// The running state S ([d_key][d_value]) sits in accumulators with key rows and value
// columns: element [v] of lane (r, q4) of tile (y, x) is S[16 rt + 4 q4 + v][16 ct + r].  A
// lane thus holds 4 consecutive keys of one value column and publishes them with one 8-byte
// write to the transposed LDS copy St[d_value][d_key]; the update's row-side operand is the
// Kh fragment already read for the intra-chunk product.
template <int D, int C>
__global__ __launch_bounds__(C * 4, (BwdCfg<D, C>::WAVES_PER_EU)) void bwd_dq_scan_bf16(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ s, bf16_t* __restrict__ dQ,
    const float* __restrict__ fwd_prefix, float* __restrict__ ds_partial, int H, int N, int G,
    int seg_rows, float eps) {
  using Cfg = BwdCfg<D, C>;
  using AT = AccTiles<D, Cfg::NW>;
  constexpr int PITCH = Cfg::PITCH;
  __shared__ __attribute__((aligned(16))) bf16_t Qs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Ks[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Gs[Cfg::TILE];   // dO
  __shared__ __attribute__((aligned(16))) bf16_t St[Cfg::STATE];  // state, [d_value][d_key]
  __shared__ float rq[C];
  __shared__ float ds_wave[Cfg::NW];

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const bf16_t* Qu = Q + ubase;
  const bf16_t* Ku = K + ubase;
  const bf16_t* Vu = V + ubase;
  const bf16_t* Gu = dO + ubase;
  bf16_t* dQu = dQ + ubase;
  const float scale = s[unit % H];
  const float r_clamped = 1.0f / eps;
  const int row_begin = g * seg_rows;
  const int row_end = min(N, row_begin + seg_rows);

  f32x4 sacc[AT::NCT][AT::NRT];
  const float* init = (fwd_prefix != nullptr && g > 0)
                          ? fwd_prefix + (size_t(unit) * G + g) * D * D : nullptr;
#pragma unroll
  for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
    for (int y = 0; y < AT::NRT; ++y)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        sacc[x][y][v] = (init != nullptr && AT::active(w))
            ? init[(16 * AT::row_tile(w, y) + 4 * q4 + v) * D + 16 * AT::col_tile(w, x) + r] : 0.f;

  float ds_lane = 0.f;
  TileStage<D, C, Cfg::NT> qst, kst, vst, gst;
  if (Cfg::PREFETCH) {
    qst.fetch(Qu, row_begin, row_end);
    kst.fetch(Ku, row_begin, row_end);
    vst.fetch(Vu, row_begin, row_end);
    gst.fetch(Gu, row_begin, row_end);
  }

  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    if (!Cfg::PREFETCH) {
      qst.fetch(Qu, row0, row_end);
      kst.fetch(Ku, row0, row_end);
      vst.fetch(Vu, row0, row_end);
      gst.fetch(Gu, row0, row_end);
    }
    if (AT::active(w)) {
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y) {
          uint2 pk;
          pk.x = pack_bf16(sacc[x][y][0], sacc[x][y][1]);
          pk.y = pack_bf16(sacc[x][y][2], sacc[x][y][3]);
          *reinterpret_cast<uint2*>(St + (16 * AT::col_tile(w, x) + r) * PITCH +
                                    16 * AT::row_tile(w, y) + 4 * q4) = pk;
        }
    }
    qst.commit_normalised(Qs, eps, rq);
    kst.commit_normalised(Ks, eps, nullptr);
    vst.commit_plain(Vs);
    gst.commit_plain(Gs);
    if (Cfg::PREFETCH && row0 + C < row_end) {
      qst.fetch(Qu, row0 + C, row_end);
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
      gst.fetch(Gu, row0 + C, row_end);
    }
    __syncthreads();

    // earlier chunks: dO S^T (contraction over d_value = rows of St)
    bf16x8 gf[Cfg::KS];  // dO rows of this wave
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks)
      gf[ks] = lds_row_frag(Gs + (16 * w + r) * PITCH + 32 * ks + 8 * q4);
    f32x4 dq[Cfg::DT];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt) dq[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks) {
      bf16x8 sf[Cfg::DT];
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt)
        sf[nt] = lds_col_frag(St, PITCH, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, 16 * nt, r);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) dq[nt] = mma16(gf[ks], sf[nt], dq[nt]);
      __builtin_amdgcn_sched_barrier(0);
    }

    // this chunk: (A (.) M) Kh with A^T = V dO^T, and the state update, 32 tokens at a time
#pragma unroll
    for (int p = 0; p < Cfg::NP; ++p) {
      const bool diag_or_below = 2 * p <= w;
      const int t0 = 32 * p + 4 * q4, t1 = 32 * p + 16 + 4 * q4;  // token order of the A slots
      bf16x8 kc[Cfg::DT], vcol[AT::NCT], krow[AT::NRT], vr[2][Cfg::KS];
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) kc[nt] = lds_col_frag(Ks, PITCH, t0, t1, 16 * nt, r);
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
        vcol[x] = lds_col_frag(Vs, PITCH, t0, t1, 16 * AT::col_tile(w, x), r);
      if (AT::WPC != 1) {
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
          krow[y] = lds_col_frag(Ks, PITCH, t0, t1, 16 * AT::row_tile(w, y), r);
      }
      if (diag_or_below) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
          for (int ks = 0; ks < Cfg::KS; ++ks)
            vr[half][ks] = lds_row_frag(Vs + (16 * (2 * p + half) + r) * PITCH + 32 * ks + 8 * q4);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (diag_or_below) {
        bf16x8 af;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int jt = 2 * p + half;
          f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < Cfg::KS; ++ks) t = mma16(vr[half][ks], gf[ks], t);
          // t[v] = dO_(16w + r) . v_(16jt + 4 q4 + v); keep key <= query
          const bool full = jt < w, diag = jt == w;
          put_half(af, half, t, full || (diag && 4 * q4 + 0 <= r), full || (diag && 4 * q4 + 1 <= r),
                   full || (diag && 4 * q4 + 2 <= r), full || (diag && 4 * q4 + 3 <= r));
        }
#pragma unroll
        for (int nt = 0; nt < Cfg::DT; ++nt) dq[nt] = mma16(af, kc[nt], dq[nt]);
      }
      // state update: S += Kh^T V over these 32 tokens
      if (AT::active(w)) {
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
#pragma unroll
          for (int x = 0; x < AT::NCT; ++x)
            sacc[x][y] = mma16(AT::WPC == 1 ? kc[y] : krow[y], vcol[x], sacc[x][y]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // epilogue: rho_i = qh_i . dqh_i ; dq_i = s r_i (dqh_i - qh_i rho_i)
    float rho[4] = {0.f, 0.f, 0.f, 0.f};
    float qv[Cfg::DT][4];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        qv[nt][v] = bf16_to_f32(Qs[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r]);
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) rho[v] += qv[nt][v] * dq[nt][v];
    wave_lds_sync();  // this wave's reads of its Gs rows (gf) precede the staging writes
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      rho[v] = group_sum<16>(rho[v]);
      if (r == 0) ds_lane += rho[v];
      const float ri = rq[16 * w + 4 * q4 + v];
      const float proj = (ri == r_clamped) ? 0.f : rho[v];
      const float f = scale * ri;
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt)
        Gs[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r] =
            f32_to_bf16(f * (dq[nt][v] - qv[nt][v] * proj));
    }
    wave_lds_sync();
    constexpr int PIECES = 16 * D / 8;
#pragma unroll
    for (int i = l; i < PIECES; i += 64) {
      const int lr = i / (D / 8), col = (i % (D / 8)) * 8;
      const int row = row0 + 16 * w + lr;
      if (row < row_end)
        *reinterpret_cast<uint4*>(dQu + size_t(row) * D + col) =
            *reinterpret_cast<const uint4*>(Gs + (16 * w + lr) * PITCH + col);
    }
    __syncthreads();
  }

  // per-workgroup partial of ds: lanes with r == 0 hold the row sums
  ds_lane = group_sum<64>(ds_lane);
  if (l == 0) ds_wave[w] = ds_lane;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < Cfg::NW; ++i) t += ds_wave[i];
    ds_partial[size_t(unit) * G + g] = t;
  }
}

// ---------------------------------------------------------------------------------------
// Kernel 4: dK and dV of one segment, chunks in reverse order.  Wave w owns key rows
// 16w..16w+15 of the chunk.  The running reverse state R ([d_key][d_value]) sits transposed
// in the accumulators (value rows, key columns): element [v] of lane (r, q4) of tile (y, x)
// is R[16 ct + r][16 rt + 4 q4 + v], published with one 8-byte write to the row-major LDS
// copy Rl[d_key][d_value]; the update's row-side operand is the dO fragment already read
// for the intra-chunk dV product.
template <int D, int C>
__global__ __launch_bounds__(C * 4, (BwdCfg<D, C>::WAVES_PER_EU)) void bwd_dkdv_scan_bf16(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ s, bf16_t* __restrict__ dK,
    bf16_t* __restrict__ dV, const float* __restrict__ rev_suffix, int H, int N, int G,
    int seg_rows, float eps) {
  using Cfg = BwdCfg<D, C>;
  using AT = AccTiles<D, Cfg::NW>;
  constexpr int PITCH = Cfg::PITCH;
  __shared__ __attribute__((aligned(16))) bf16_t Qs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Ks[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Gs[Cfg::TILE];   // dO
  __shared__ __attribute__((aligned(16))) bf16_t Rl[Cfg::STATE];  // reverse state, [d_key][d_value]
  __shared__ float rk[C];

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const bf16_t* Qu = Q + ubase;
  const bf16_t* Ku = K + ubase;
  const bf16_t* Vu = V + ubase;
  const bf16_t* Gu = dO + ubase;
  bf16_t* dKu = dK + ubase;
  bf16_t* dVu = dV + ubase;
  const float scale = s[unit % H];
  const float r_clamped = 1.0f / eps;
  const int row_begin = g * seg_rows;
  const int row_end = min(N, row_begin + seg_rows);
  const int n_chunks = (row_end - row_begin + C - 1) / C;

  f32x4 racc[AT::NCT][AT::NRT];
  const float* init = (rev_suffix != nullptr && g < G - 1)
                          ? rev_suffix + (size_t(unit) * G + g) * D * D : nullptr;
#pragma unroll
  for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
    for (int y = 0; y < AT::NRT; ++y) {
      f32x4 t = {0.f, 0.f, 0.f, 0.f};
      if (init != nullptr && AT::active(w))
        t = *reinterpret_cast<const f32x4*>(init + (16 * AT::col_tile(w, x) + r) * D +
                                            16 * AT::row_tile(w, y) + 4 * q4);
      racc[x][y] = t;
    }

  TileStage<D, C, Cfg::NT> qst, kst, vst, gst;
  if (Cfg::PREFETCH) {
    const int first = row_begin + (n_chunks - 1) * C;
    qst.fetch(Qu, first, row_end);
    kst.fetch(Ku, first, row_end);
    vst.fetch(Vu, first, row_end);
    gst.fetch(Gu, first, row_end);
  }

  for (int c = n_chunks - 1; c >= 0; --c) {
    const int row0 = row_begin + c * C;
    if (!Cfg::PREFETCH) {
      qst.fetch(Qu, row0, row_end);
      kst.fetch(Ku, row0, row_end);
      vst.fetch(Vu, row0, row_end);
      gst.fetch(Gu, row0, row_end);
    }
    if (AT::active(w)) {
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y) {
          uint2 pk;
          pk.x = pack_bf16(racc[x][y][0], racc[x][y][1]);
          pk.y = pack_bf16(racc[x][y][2], racc[x][y][3]);
          *reinterpret_cast<uint2*>(Rl + (16 * AT::col_tile(w, x) + r) * PITCH +
                                    16 * AT::row_tile(w, y) + 4 * q4) = pk;
        }
    }
    qst.commit_normalised(Qs, eps, nullptr);
    kst.commit_normalised(Ks, eps, rk);
    vst.commit_plain(Vs);
    gst.commit_plain(Gs);
    if (Cfg::PREFETCH && c > 0) {
      qst.fetch(Qu, row0 - C, row_end);
      kst.fetch(Ku, row0 - C, row_end);
      vst.fetch(Vu, row0 - C, row_end);
      gst.fetch(Gu, row0 - C, row_end);
    }
    __syncthreads();

    bf16x8 kf[Cfg::KS], vf[Cfg::KS];  // this wave's key rows and value rows
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks) {
      kf[ks] = lds_row_frag(Ks + (16 * w + r) * PITCH + 32 * ks + 8 * q4);
      vf[ks] = lds_row_frag(Vs + (16 * w + r) * PITCH + 32 * ks + 8 * q4);
    }
    f32x4 dk[Cfg::DT], dv[Cfg::DT];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt) {
      dk[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
      dv[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // later chunks: dv += kh R (over d_key), dkh += v R^T (over d_value)
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks) {
      bf16x8 rcol[Cfg::DT], rrow[Cfg::DT];
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) {
        rcol[nt] = lds_col_frag(Rl, PITCH, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, 16 * nt, r);
        rrow[nt] = lds_row_frag(Rl + (16 * nt + r) * PITCH + 32 * ks + 8 * q4);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) {
        dv[nt] = mma16(kf[ks], rcol[nt], dv[nt]);
        dk[nt] = mma16(vf[ks], rrow[nt], dk[nt]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // this chunk: query tiles it >= w two at a time, and the reverse state update
#pragma unroll
    for (int p = 0; p < Cfg::NP; ++p) {
      const bool diag_or_above = 2 * p + 1 >= w;
      const int t0 = 32 * p + 4 * q4, t1 = 32 * p + 16 + 4 * q4;  // token order of the A slots
      bf16x8 gc[Cfg::DT], qcol[AT::NCT], grow[AT::NRT];
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) gc[nt] = lds_col_frag(Gs, PITCH, t0, t1, 16 * nt, r);
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
        qcol[x] = lds_col_frag(Qs, PITCH, t0, t1, 16 * AT::col_tile(w, x), r);
      if (AT::WPC != 1) {
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
          grow[y] = lds_col_frag(Gs, PITCH, t0, t1, 16 * AT::row_tile(w, y), r);
      }
      __builtin_amdgcn_sched_barrier(0);
      // reverse state update: R^T += dO^T Qh over these 32 tokens
      if (AT::active(w)) {
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
#pragma unroll
          for (int x = 0; x < AT::NCT; ++x)
            racc[x][y] = mma16(AT::WPC == 1 ? gc[y] : grow[y], qcol[x], racc[x][y]);
      }
      if (diag_or_above) {
        bf16x8 qr[2][Cfg::KS], gr[2][Cfg::KS], qc[Cfg::DT];
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
          for (int ks = 0; ks < Cfg::KS; ++ks) {
            const int off = (16 * (2 * p + half) + r) * PITCH + 32 * ks + 8 * q4;
            qr[half][ks] = lds_row_frag(Qs + off);
            gr[half][ks] = lds_row_frag(Gs + off);
          }
#pragma unroll
        for (int nt = 0; nt < Cfg::DT; ++nt) qc[nt] = lds_col_frag(Qs, PITCH, t0, t1, 16 * nt, r);
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 pf, af;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int it = 2 * p + half;
          f32x4 tp = {0.f, 0.f, 0.f, 0.f}, ta = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < Cfg::KS; ++ks) {
            tp = mma16(qr[half][ks], kf[ks], tp);
            ta = mma16(gr[half][ks], vf[ks], ta);
          }
          // t*[v]: query 16 it + 4 q4 + v, key 16 w + r; keep key <= query
          const bool full = it > w, diag = it == w;
          const bool k0 = full || (diag && r <= 4 * q4 + 0), k1 = full || (diag && r <= 4 * q4 + 1),
                     k2 = full || (diag && r <= 4 * q4 + 2), k3 = full || (diag && r <= 4 * q4 + 3);
          put_half(pf, half, tp, k0, k1, k2, k3);
          put_half(af, half, ta, k0, k1, k2, k3);
        }
#pragma unroll
        for (int nt = 0; nt < Cfg::DT; ++nt) {
          dv[nt] = mma16(pf, gc[nt], dv[nt]);
          dk[nt] = mma16(af, qc[nt], dk[nt]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // epilogue: dk_j = s r_j (dkh_j - kh_j (kh_j . dkh_j)), dv_j = s dv_j
    float rho[4] = {0.f, 0.f, 0.f, 0.f};
    float kv[Cfg::DT][4];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        kv[nt][v] = bf16_to_f32(Ks[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r]);
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) rho[v] += kv[nt][v] * dk[nt][v];
    wave_lds_sync();  // own Ks / Vs rows are dead from here on: reuse them as staging
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      rho[v] = group_sum<16>(rho[v]);
      const float rj = rk[16 * w + 4 * q4 + v];
      const float proj = (rj == r_clamped) ? 0.f : rho[v];
      const float f = scale * rj;
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) {
        Ks[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r] =
            f32_to_bf16(f * (dk[nt][v] - kv[nt][v] * proj));
        Vs[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r] = f32_to_bf16(scale * dv[nt][v]);
      }
    }
    wave_lds_sync();
    constexpr int PIECES = 16 * D / 8;
#pragma unroll
    for (int i = l; i < PIECES; i += 64) {
      const int lr = i / (D / 8), col = (i % (D / 8)) * 8;
      const int row = row0 + 16 * w + lr;
      if (row < row_end) {
        *reinterpret_cast<uint4*>(dKu + size_t(row) * D + col) =
            *reinterpret_cast<const uint4*>(Ks + (16 * w + lr) * PITCH + col);
        *reinterpret_cast<uint4*>(dVu + size_t(row) * D + col) =
            *reinterpret_cast<const uint4*>(Vs + (16 * w + lr) * PITCH + col);
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
// Kernel 5: ds[h] = sum over batches b and segments g of partial[(b H + h) G + g].
__global__ __launch_bounds__(256) void bwd_reduce_ds(const float* __restrict__ partial,
                                                     float* __restrict__ ds, int B, int H, int G) {
  __shared__ float red[256];
  const int h = blockIdx.x;
  float acc = 0.f;
  const long n = long(B) * G;
  for (long i = threadIdx.x; i < n; i += 256) {
    const long b = i / G, g = i % G;
    acc += partial[(b * H + h) * G + g];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int stride = 128; stride > 0; stride >>= 1) {
    if (int(threadIdx.x) < stride) red[threadIdx.x] += red[threadIdx.x + stride];
    __syncthreads();
  }
  if (threadIdx.x == 0) ds[h] = red[0];
}

template <int D, int C>
hipError_t run_bwd_causal(const CausalArgs& a) {
  using Cfg = BwdCfg<D, C>;
  const int units = a.B * a.H;
  const bf16_t* Q = static_cast<const bf16_t*>(a.Q);
  const bf16_t* K = static_cast<const bf16_t*>(a.K);
  const bf16_t* V = static_cast<const bf16_t*>(a.V);
  const bf16_t* dO = static_cast<const bf16_t*>(a.dO);
  char* ws = static_cast<char*>(a.workspace);
  float* fwd_states = nullptr;
  float* rev_states = nullptr;
  if (a.G > 1) {
    fwd_states = reinterpret_cast<float*>(ws);
    rev_states = reinterpret_cast<float*>(ws + state_array_bytes(a.B, a.H, D, a.G));
    ws += 2 * state_array_bytes(a.B, a.H, D, a.G);
  }
  float* ds_partial = reinterpret_cast<float*>(ws);
  const dim3 grid(units * a.G), block(Cfg::NT);
  hipError_t err;
  if (a.G > 1) {
    err = launch_kernel("bwd_segment_states_bf16", bwd_segment_states_bf16<D, C>, grid, block, 0,
                        a.stream, Q, K, V, dO, fwd_states, rev_states, a.N, a.G, a.seg_rows, a.eps);
    if (err != hipSuccess) return err;
    err = launch_bwd_state_carry(fwd_states, rev_states, units, a.G, D * D, a.stream);
    if (err != hipSuccess) return err;
  }
  err = launch_kernel("bwd_dq_scan_bf16", bwd_dq_scan_bf16<D, C>, grid, block, 0, a.stream, Q, K, V,
                      dO, a.s, static_cast<bf16_t*>(a.dQ), fwd_states, ds_partial, a.H, a.N, a.G,
                      a.seg_rows, a.eps);
  if (err != hipSuccess) return err;
  err = launch_kernel("bwd_dkdv_scan_bf16", bwd_dkdv_scan_bf16<D, C>, grid, block, 0, a.stream, Q, K,
                      V, dO, a.s, static_cast<bf16_t*>(a.dK), static_cast<bf16_t*>(a.dV), rev_states,
                      a.H, a.N, a.G, a.seg_rows, a.eps);
  if (err != hipSuccess) return err;
  return launch_reduce_ds(ds_partial, a.ds, a.B, a.H, a.G, a.stream);
}

}  // namespace

hipError_t launch_bwd_state_carry(float* fwd_tot, float* rev_tot, int units, int G, int elems,
                                  hipStream_t st) {
  const long total = long(units) * elems;
  return launch_kernel("bwd_state_carry", bwd_state_carry, dim3(unsigned((total + 255) / 256), 2),
                       dim3(256), 0, st, fwd_tot, rev_tot, G, elems, total);
}

hipError_t launch_reduce_ds(const float* partial, float* ds, int B, int H, int G, hipStream_t st) {
  return launch_kernel("bwd_reduce_ds", bwd_reduce_ds, dim3(H), dim3(256), 0, st, partial, ds, B, H,
                       G);
}

hipError_t bwd_causal_bf16(const CausalArgs& a) {
  switch (a.d * 1000 + a.C) {
    case 32064: return run_bwd_causal<32, 64>(a);
    case 32128: return run_bwd_causal<32, 128>(a);
    case 32256: return run_bwd_causal<32, 256>(a);
    case 64064: return run_bwd_causal<64, 64>(a);
    case 64128: return run_bwd_causal<64, 128>(a);
    case 64256: return run_bwd_causal<64, 256>(a);
    case 128064: return run_bwd_causal<128, 64>(a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cottn
