// Bidirectional cosine attention, forward and backward, bf16 storage / bf16 MFMA / fp32
// accumulation (gfx950).
//
// Sec. 4 eq. subQuadCos: without a mask the product reassociates to O = s_h Qh (Kh^T V), so
// the d x d matrix S = Kh^T V is reduced once over the whole sequence and then applied to
// every query row.  The gradient formulas of Sec. 4 with M removed collapse the same way:
// with G = Qh^T dO (also d x d),
//     dQh = s dO S^T,   dKh = s V G^T,   dV = s Kh G,   ds = <S, G> (Frobenius product),
// followed by the chain rule through the row normalisation.
//
// Three launches per call:
//   totals   each workgroup reduces N(X)^T Y over one segment of rows (split over the
//            sequence because B*H alone does not fill the chip);
//   combine  sums the segment totals per (batch, head) into slot 0 (and into `state`);
//            in the backward it also forms the per-(b,h) share of ds in fp32;
//   apply    streams the rows once more and multiplies them with the d x d totals.
#include "device_common.h"
#include "launch.h"
#include "tile_io.h"
#include "workspace.h"

namespace cottn {
namespace {

template <int D, int C>
struct BiCfg {
  static constexpr int NW = C / 16;
  static constexpr int NT = NW * 64;
  static constexpr int DT = D / 16;
  static constexpr int KS = D / 32;
  static constexpr int PITCH = lds_pitch(D);
  static constexpr int TILE = C * PITCH;
  static constexpr int STATE = D * PITCH;
};

// totals[pair][unit][g] = sum over the rows of segment g of N(X)^T Y, stored [feature of X]
// [feature of Y] in fp32.  pair = blockIdx.y selects (X, Y) = (K, V) or (Q, dO).
template <int D, int C>
__global__ __launch_bounds__(C * 4) void bidir_totals_bf16(
    const bf16_t* __restrict__ X0, const bf16_t* __restrict__ Y0, const bf16_t* __restrict__ X1,
    const bf16_t* __restrict__ Y1, float* __restrict__ totals, size_t pair_stride, int N, int G,
    int seg_rows, float eps) {
  using Cfg = BiCfg<D, C>;
  using AT = AccTiles<D, Cfg::NW>;
  constexpr int PITCH = Cfg::PITCH;
  __shared__ __attribute__((aligned(16))) bf16_t Xs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Ys[Cfg::TILE];

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const bf16_t* X = (blockIdx.y == 0 ? X0 : X1) + ubase;
  const bf16_t* Y = (blockIdx.y == 0 ? Y0 : Y1) + ubase;
  float* out = totals + blockIdx.y * pair_stride + (size_t(unit) * G + g) * D * D;
  const int row_begin = g * seg_rows;
  const int row_end = min(N, row_begin + seg_rows);

  f32x4 acc[AT::NCT][AT::NRT];
#pragma unroll
  for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
    for (int y = 0; y < AT::NRT; ++y) acc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};

  TileStage<D, C, Cfg::NT> xst, yst;
  xst.fetch(X, row_begin, row_end);
  yst.fetch(Y, row_begin, row_end);
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    __syncthreads();
    xst.commit_normalised(Xs, eps, nullptr);
    yst.commit_plain(Ys);
    if (row0 + C < row_end) {
      xst.fetch(X, row0 + C, row_end);
      yst.fetch(Y, row0 + C, row_end);
    }
    __syncthreads();
    if (AT::active(w)) {
      bf16x8 by[C / 32][AT::NCT], ax[C / 32][AT::NRT];
#pragma unroll
      for (int p = 0; p < C / 32; ++p) {
        const int k0 = 32 * p + 8 * q4;
#pragma unroll
        for (int x = 0; x < AT::NCT; ++x)
          by[p][x] = lds_col_frag(Ys, PITCH, k0, k0 + 4, 16 * AT::col_tile(w, x), r);
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
          ax[p][y] = lds_col_frag(Xs, PITCH, k0, k0 + 4, 16 * AT::row_tile(w, y), r);
      }
      __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
      for (int p = 0; p < C / 32; ++p)
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
#pragma unroll
          for (int x = 0; x < AT::NCT; ++x) acc[x][y] = mma16(ax[p][y], by[p][x], acc[x][y]);
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

// One workgroup per (batch, head): slot 0 of each pair <- sum over g of the slots; `state`
// (may be null) receives pair 0; with n_pairs == 2, ds_partial[unit] = sum_e S[e] * G[e].
__global__ __launch_bounds__(256) void bidir_combine(float* __restrict__ totals, size_t pair_stride,
                                                     int n_pairs, int G, int elems,
                                                     float* __restrict__ state,
                                                     float* __restrict__ ds_partial) {
  __shared__ float red[256];
  const int unit = blockIdx.x;
  float* p0 = totals + size_t(unit) * G * elems;
  float* p1 = p0 + pair_stride;
  float prod = 0.f;
  for (int e = threadIdx.x; e < elems; e += 256) {
    float a = 0.f;
    for (int g = 0; g < G; ++g) a += p0[size_t(g) * elems + e];
    p0[e] = a;
    if (state != nullptr) state[size_t(unit) * elems + e] = a;
    if (n_pairs == 2) {
      float b = 0.f;
      for (int g = 0; g < G; ++g) b += p1[size_t(g) * elems + e];
      p1[e] = b;
      prod += a * b;
    }
  }
  if (n_pairs == 2) {
    red[threadIdx.x] = prod;
    __syncthreads();
    for (int stride = 128; stride > 0; stride >>= 1) {
      if (int(threadIdx.x) < stride) red[threadIdx.x] += red[threadIdx.x + stride];
      __syncthreads();
    }
    if (threadIdx.x == 0) ds_partial[unit] = red[0];
  }
}

// Copy a [D][D] fp32 matrix M (global) into LDS as bf16, either as is (dst[a][b] = M[a][b])
// or transposed (dst[b][a] = M[a][b]).
template <int D, int NT, bool TRANSPOSE>
__device__ __forceinline__ void stage_matrix(bf16_t* dst, const float* __restrict__ M) {
  constexpr int PITCH = lds_pitch(D);
  for (int e = threadIdx.x; e < D * D; e += NT) {
    const int a = e / D, b = e % D;
    const bf16_t x = f32_to_bf16(M[e]);
    if (TRANSPOSE) dst[b * PITCH + a] = x; else dst[a * PITCH + b] = x;
  }
}

// O rows of one segment: O = s Qh S.
template <int D, int C>
__global__ __launch_bounds__(C * 4) void fwd_bidir_apply_bf16(
    const bf16_t* __restrict__ Q, const float* __restrict__ s, bf16_t* __restrict__ O,
    const float* __restrict__ totals, int H, int N, int G, int seg_rows, float eps) {
  using Cfg = BiCfg<D, C>;
  constexpr int PITCH = Cfg::PITCH;
  __shared__ __attribute__((aligned(16))) bf16_t Qs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t St[Cfg::STATE];  // [d_value][d_key]

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const bf16_t* Qu = Q + ubase;
  bf16_t* Ou = O + ubase;
  const float scale = s[unit % H];
  const int row_begin = g * seg_rows;
  const int row_end = min(N, row_begin + seg_rows);

  TileStage<D, C, Cfg::NT> qst;
  qst.fetch(Qu, row_begin, row_end);
  stage_matrix<D, Cfg::NT, true>(St, totals + size_t(unit) * G * D * D);

  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    qst.commit_normalised(Qs, eps, nullptr);
    if (row0 + C < row_end) qst.fetch(Qu, row0 + C, row_end);
    __syncthreads();
    f32x4 oacc[Cfg::DT];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt) oacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 qf[Cfg::KS], sf[Cfg::KS][Cfg::DT];
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks) {
      qf[ks] = lds_row_frag(Qs + (16 * w + r) * PITCH + 32 * ks + 8 * q4);
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt)
        sf[ks][nt] = lds_row_frag(St + (16 * nt + r) * PITCH + 32 * ks + 8 * q4);
    }
    __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks)
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) oacc[nt] = mma16(qf[ks], sf[ks][nt], oacc[nt]);
    wave_lds_sync();
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        Qs[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r] = f32_to_bf16(scale * oacc[nt][v]);
    wave_lds_sync();
    constexpr int PIECES = 16 * D / 8;
#pragma unroll
    for (int i = l; i < PIECES; i += 64) {
      const int lr = i / (D / 8), col = (i % (D / 8)) * 8;
      const int row = row0 + 16 * w + lr;
      if (row < row_end)
        *reinterpret_cast<uint4*>(Ou + size_t(row) * D + col) =
            *reinterpret_cast<const uint4*>(Qs + (16 * w + lr) * PITCH + col);
    }
    __syncthreads();
  }
}

// row-wise chain rule through the normalisation on a wave's 16 x D accumulator block:
// out = f_row * (acc - xh * (xh . acc)), written as bf16 into `stage` (the wave's own rows
// of a dead LDS tile); xh is read from `xs` (same rows).  Returns per-lane (xh . acc) sums.
template <int D>
__device__ __forceinline__ void normalise_backward_rows(const f32x4* acc, const bf16_t* xs,
                                                        bf16_t* stage, const float* rinv,
                                                        float scale, float r_clamped, int w,
                                                        int r, int q4) {
  constexpr int DT = D / 16, PITCH = lds_pitch(D);
  float rho[4] = {0.f, 0.f, 0.f, 0.f};
  float xv[DT][4];
#pragma unroll
  for (int nt = 0; nt < DT; ++nt)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      xv[nt][v] = bf16_to_f32(xs[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r]);
      rho[v] += xv[nt][v] * acc[nt][v];
    }
  wave_lds_sync();
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    rho[v] = group_sum<16>(rho[v]);
    const float ri = rinv[16 * w + 4 * q4 + v];
    const float proj = (ri == r_clamped) ? 0.f : rho[v];
    const float f = scale * ri;
#pragma unroll
    for (int nt = 0; nt < DT; ++nt)
      stage[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r] =
          f32_to_bf16(f * (acc[nt][v] - xv[nt][v] * proj));
  }
}

// dQ, dK, dV rows of one segment; the first H workgroups also finish ds.
template <int D, int C>
__global__ __launch_bounds__(C * 4) void bwd_bidir_apply_bf16(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ s, bf16_t* __restrict__ dQ,
    bf16_t* __restrict__ dK, bf16_t* __restrict__ dV, const float* __restrict__ totals,
    size_t pair_stride, const float* __restrict__ ds_partial, float* __restrict__ ds, int B, int H,
    int N, int G, int seg_rows, float eps) {
  using Cfg = BiCfg<D, C>;
  constexpr int PITCH = Cfg::PITCH;
  __shared__ __attribute__((aligned(16))) bf16_t Qs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Ks[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) bf16_t Gs[Cfg::TILE];   // dO
  __shared__ __attribute__((aligned(16))) bf16_t Sl[Cfg::STATE];  // Kh^T V,  [d_key][d_value]
  __shared__ __attribute__((aligned(16))) bf16_t Gl[Cfg::STATE];  // Qh^T dO, [d_key][d_value]
  __shared__ float rq[C], rk[C];

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const bf16_t* Qu = Q + ubase;
  const bf16_t* Ku = K + ubase;
  const bf16_t* Vu = V + ubase;
  const bf16_t* Gu = dO + ubase;
  const float scale = s[unit % H];
  const float r_clamped = 1.0f / eps;
  const int row_begin = g * seg_rows;
  const int row_end = min(N, row_begin + seg_rows);

  if (int(blockIdx.x) < H && tid == 0) {  // ds[h] = sum over batches of the per-(b,h) shares
    float t = 0.f;
    for (int b = 0; b < B; ++b) t += ds_partial[size_t(b) * H + blockIdx.x];
    ds[blockIdx.x] = t;
  }

  TileStage<D, C, Cfg::NT> qst, kst, vst, gst;
  qst.fetch(Qu, row_begin, row_end);
  kst.fetch(Ku, row_begin, row_end);
  vst.fetch(Vu, row_begin, row_end);
  gst.fetch(Gu, row_begin, row_end);
  stage_matrix<D, Cfg::NT, false>(Sl, totals + size_t(unit) * G * D * D);
  stage_matrix<D, Cfg::NT, false>(Gl, totals + pair_stride + size_t(unit) * G * D * D);

  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    qst.commit_normalised(Qs, eps, rq);
    kst.commit_normalised(Ks, eps, rk);
    vst.commit_plain(Vs);
    gst.commit_plain(Gs);
    if (row0 + C < row_end) {
      qst.fetch(Qu, row0 + C, row_end);
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
      gst.fetch(Gu, row0 + C, row_end);
    }
    __syncthreads();

    f32x4 dq[Cfg::DT], dk[Cfg::DT], dv[Cfg::DT];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt) {
      dq[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
      dk[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
      dv[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks) {
      const int off = (16 * w + r) * PITCH + 32 * ks + 8 * q4;
      const bf16x8 gf = lds_row_frag(Gs + off), vf = lds_row_frag(Vs + off),
                   kf = lds_row_frag(Ks + off);
      bf16x8 srow[Cfg::DT], grow[Cfg::DT], gcol[Cfg::DT];
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) {
        const int soff = (16 * nt + r) * PITCH + 32 * ks + 8 * q4;
        srow[nt] = lds_row_frag(Sl + soff);
        grow[nt] = lds_row_frag(Gl + soff);
        gcol[nt] = lds_col_frag(Gl, PITCH, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, 16 * nt, r);
      }
      __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) {
        dq[nt] = mma16(gf, srow[nt], dq[nt]);   // dO S^T  (over d_value)
        dk[nt] = mma16(vf, grow[nt], dk[nt]);   // V G^T   (over d_value)
        dv[nt] = mma16(kf, gcol[nt], dv[nt]);   // Kh G    (over d_key)
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // every tile row is private to its wave here: stage the results in place
    normalise_backward_rows<D>(dq, Qs, Gs, rq, scale, r_clamped, w, r, q4);
    normalise_backward_rows<D>(dk, Ks, Ks, rk, scale, r_clamped, w, r, q4);
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        Vs[(16 * w + 4 * q4 + v) * PITCH + 16 * nt + r] = f32_to_bf16(scale * dv[nt][v]);
    wave_lds_sync();
    constexpr int PIECES = 16 * D / 8;
#pragma unroll
    for (int i = l; i < PIECES; i += 64) {
      const int lr = i / (D / 8), col = (i % (D / 8)) * 8;
      const int row = row0 + 16 * w + lr;
      if (row < row_end) {
        const size_t goff = ubase + size_t(row) * D + col;
        const int loff = (16 * w + lr) * PITCH + col;
        *reinterpret_cast<uint4*>(dQ + goff) = *reinterpret_cast<const uint4*>(Gs + loff);
        *reinterpret_cast<uint4*>(dK + goff) = *reinterpret_cast<const uint4*>(Ks + loff);
        *reinterpret_cast<uint4*>(dV + goff) = *reinterpret_cast<const uint4*>(Vs + loff);
      }
    }
    __syncthreads();
  }
}

template <int D>
hipError_t run_fwd_bidir(const CausalArgs& a) {
  constexpr int C = 64;
  using Cfg = BiCfg<D, C>;
  const int units = a.B * a.H;
  const bf16_t* Q = static_cast<const bf16_t*>(a.Q);
  const bf16_t* K = static_cast<const bf16_t*>(a.K);
  const bf16_t* V = static_cast<const bf16_t*>(a.V);
  float* totals = static_cast<float*>(a.workspace);
  hipError_t err = launch_kernel("bidir_totals_bf16", bidir_totals_bf16<D, C>, dim3(units * a.G, 1),
                                 dim3(Cfg::NT), 0, a.stream, K, V, K, V, totals, size_t(0), a.N, a.G,
                                 a.seg_rows, a.eps);
  if (err != hipSuccess) return err;
  err = launch_bidir_combine(totals, 0, 1, units, a.G, D * D, a.state, nullptr, a.stream);
  if (err != hipSuccess) return err;
  return launch_kernel("fwd_bidir_apply_bf16", fwd_bidir_apply_bf16<D, C>, dim3(units * a.G),
                       dim3(Cfg::NT), 0, a.stream, Q, a.s, static_cast<bf16_t*>(a.O), totals, a.H,
                       a.N, a.G, a.seg_rows, a.eps);
}

template <int D>
hipError_t run_bwd_bidir(const CausalArgs& a) {
  constexpr int C = 64;
  using Cfg = BiCfg<D, C>;
  const int units = a.B * a.H;
  const bf16_t* Q = static_cast<const bf16_t*>(a.Q);
  const bf16_t* K = static_cast<const bf16_t*>(a.K);
  const bf16_t* V = static_cast<const bf16_t*>(a.V);
  const bf16_t* dO = static_cast<const bf16_t*>(a.dO);
  char* ws = static_cast<char*>(a.workspace);
  float* totals = reinterpret_cast<float*>(ws);
  const size_t pair_stride = state_array_bytes(a.B, a.H, D, a.G) / sizeof(float);
  float* ds_partial = reinterpret_cast<float*>(ws + 2 * state_array_bytes(a.B, a.H, D, a.G));
  hipError_t err = launch_kernel("bidir_totals_bf16", bidir_totals_bf16<D, C>, dim3(units * a.G, 2),
                                 dim3(Cfg::NT), 0, a.stream, K, V, Q, dO, totals, pair_stride, a.N,
                                 a.G, a.seg_rows, a.eps);
  if (err != hipSuccess) return err;
  err = launch_bidir_combine(totals, pair_stride, 2, units, a.G, D * D, nullptr, ds_partial,
                             a.stream);
  if (err != hipSuccess) return err;
  return launch_kernel("bwd_bidir_apply_bf16", bwd_bidir_apply_bf16<D, C>, dim3(units * a.G),
                       dim3(Cfg::NT), 0, a.stream, Q, K, V, dO, a.s, static_cast<bf16_t*>(a.dQ),
                       static_cast<bf16_t*>(a.dK), static_cast<bf16_t*>(a.dV), totals, pair_stride,
                       ds_partial, a.ds, a.B, a.H, a.N, a.G, a.seg_rows, a.eps);
}

}  // namespace

hipError_t launch_bidir_combine(float* totals, size_t pair_stride, int n_pairs, int units, int G,
                                int elems, float* state, float* ds_partial, hipStream_t st) {
  return launch_kernel("bidir_combine", bidir_combine, dim3(units), dim3(256), 0, st, totals,
                       pair_stride, n_pairs, G, elems, state, ds_partial);
}

hipError_t fwd_bidir_bf16(const CausalArgs& a) {
  switch (a.d) {
    case 32: return run_fwd_bidir<32>(a);
    case 64: return run_fwd_bidir<64>(a);
    case 128: return run_fwd_bidir<128>(a);
    default: return hipErrorInvalidValue;
  }
}

hipError_t bwd_bidir_bf16(const CausalArgs& a) {
  switch (a.d) {
    case 32: return run_bwd_bidir<32>(a);
    case 64: return run_bwd_bidir<64>(a);
    case 128: return run_bwd_bidir<128>(a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cottn
