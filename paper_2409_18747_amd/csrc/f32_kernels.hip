// fp32 storage / fp32 arithmetic path of every operation (vector-ALU FMAs, no MFMA).
//
// Same regrouping of the cumulative sums of Sec. 4 as the bf16 path (segments of chunks,
// segment totals -> carry -> chunk scan with the d x d state resident in the workgroup),
// with chunks of 32 rows and every tile and the state held in LDS as fp32.  This path
// exists for exactness checks and fp32 callers; it is written for clarity, not speed.
//
// Thread layout of a 256-thread workgroup on a [32][D] row tile: thread t owns row t/8 and
// the D/8 consecutive columns starting at (t%8)*D/8, so the 8 lanes of a row are adjacent
// (row reductions are 3 wavefront shuffles) and global rows are read and written whole.
// Templates take DK and DV, the widths of the Q / K rows and of the V / O rows (Sec. 2.1:
// d_H_key, d_H_value); a state is [DK][DV] with the pitch of a DV-wide tile.
#include <type_traits>

#include "device_common.h"
#include "launch.h"
#include "workspace.h"

namespace cottn {
namespace {

constexpr int CR = 32;    // rows per chunk
constexpr int NT = 256;
constexpr int PP = CR + 1;  // pitch of the [32][32] pair tiles

template <int D> struct FCfg {
  static constexpr int P = D + 4;     // pitch of row tiles and of the state
  static constexpr int CPT = D / 8;   // columns per thread
};

// acc[e] += sum_{k<n} coef[k*cstride] * X[k*px + c0 + e]
template <int CPT>
__device__ __forceinline__ void mac_rows(float* acc, const float* coef, int cstride, int n,
                                         const float* X, int px, int c0) {
  for (int k = 0; k < n; ++k) {
    const float a = coef[k * cstride];
    const float* x = X + k * px + c0;
#pragma unroll
    for (int e = 0; e < CPT; ++e) acc[e] += a * x[e];
  }
}
// acc[e] += sum_{k<n} coef[k] * X[(r0+e)*px + k]
template <int CPT>
__device__ __forceinline__ void mac_rows_t(float* acc, const float* coef, int n, const float* X,
                                           int px, int r0) {
#pragma unroll
  for (int e = 0; e < CPT; ++e) {
    const float* x = X + (r0 + e) * px;
    float t = 0.f;
    for (int k = 0; k < n; ++k) t += coef[k] * x[k];
    acc[e] += t;
  }
}

// tile[i][:] = src row (row0 + i) (zero beyond row_end), optionally L2-normalised
// (Sec. 3.2); rinv[i] = 1/max(||x||, eps) when requested.
template <int D>
__device__ __forceinline__ void load_rows(float* tile, const float* __restrict__ src, int row0,
                                          int row_end, bool normalise, float eps, float* rinv) {
  constexpr int CPT = FCfg<D>::CPT, P = FCfg<D>::P;
  const int i = threadIdx.x / 8, c0 = (threadIdx.x % 8) * CPT;
  float x[CPT];
  const int row = row0 + i;
#pragma unroll
  for (int e = 0; e < CPT; e += 4) {
    float4 v = {0.f, 0.f, 0.f, 0.f};
    if (row < row_end) v = *reinterpret_cast<const float4*>(src + size_t(row) * D + c0 + e);
    x[e] = v.x; x[e + 1] = v.y; x[e + 2] = v.z; x[e + 3] = v.w;
  }
  if (normalise) {
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < CPT; ++e) ss += x[e] * x[e];
    ss = group_sum<8>(ss);
    const float r = inv_norm(ss, eps);
#pragma unroll
    for (int e = 0; e < CPT; ++e) x[e] *= r;
    if (rinv != nullptr && (threadIdx.x % 8) == 0) rinv[i] = r;
  }
#pragma unroll
  for (int e = 0; e < CPT; ++e) tile[i * P + c0 + e] = x[e];
}

template <int D>
__device__ __forceinline__ void store_rows(float* __restrict__ dst, const float* x, int row0,
                                           int row_end) {
  constexpr int CPT = FCfg<D>::CPT;
  const int i = threadIdx.x / 8, c0 = (threadIdx.x % 8) * CPT;
  const int row = row0 + i;
  if (row < row_end) {
#pragma unroll
    for (int e = 0; e < CPT; e += 4)
      *reinterpret_cast<float4*>(dst + size_t(row) * D + c0 + e) =
          float4{x[e], x[e + 1], x[e + 2], x[e + 3]};
  }
}

// pair[i][j] = X_i . Y_j, zeroed where `causal` and j > i  (Sec. 4: M keeps j <= i)
template <int D>
__device__ __forceinline__ void pair_tile(float* pair, const float* X, const float* Y, bool causal) {
  constexpr int P = FCfg<D>::P;
  const int i = threadIdx.x / 8;
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int j = (threadIdx.x % 8) + 8 * m;
    float t = 0.f;
    if (!causal || j <= i)
      for (int k = 0; k < D; ++k) t += X[i * P + k] * Y[j * P + k];
    pair[i * PP + j] = t;
  }
}

// M[a][c] += sum_j X[j][a] * Y[j][c] over the tile's 32 rows (X rows DK wide, Y rows DV wide)
template <int DK, int DV>
__device__ __forceinline__ void state_update(float* M, const float* X, const float* Y) {
  constexpr int CPT = FCfg<DV>::CPT, P = FCfg<DV>::P, PX = FCfg<DK>::P;
  const int c0 = (threadIdx.x % 8) * CPT;
  for (int a = threadIdx.x / 8; a < DK; a += CR) {
    float acc[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) acc[e] = 0.f;
    mac_rows<CPT>(acc, X + a, PX, CR, Y, P, c0);
#pragma unroll
    for (int e = 0; e < CPT; ++e) M[a * P + c0 + e] += acc[e];
  }
}

template <int DK, int DV>
__device__ __forceinline__ void state_load(float* M, const float* __restrict__ src) {
  constexpr int P = FCfg<DV>::P;
  for (int e = threadIdx.x; e < DK * DV; e += NT) M[(e / DV) * P + (e % DV)] = src ? src[e] : 0.f;
}
// the same with a second (optional) matrix added: M = src + more
template <int DK, int DV>
__device__ __forceinline__ void state_load2(float* M, const float* __restrict__ src,
                                            const float* __restrict__ more) {
  constexpr int P = FCfg<DV>::P;
  for (int e = threadIdx.x; e < DK * DV; e += NT)
    M[(e / DV) * P + (e % DV)] = (src ? src[e] : 0.f) + (more ? more[e] : 0.f);
}
template <int DK, int DV>
__device__ __forceinline__ void state_store(float* __restrict__ dst, const float* M) {
  constexpr int P = FCfg<DV>::P;
  for (int e = threadIdx.x; e < DK * DV; e += NT) dst[e] = M[(e / DV) * P + (e % DV)];
}

// zeros rows row_lo..row_hi-1 of a [.][D] fp32 tensor (rows of a padded batch that do not exist)
template <int D>
__device__ __forceinline__ void zero_rows_f32(float* __restrict__ dst, int row_lo, int row_hi) {
  const long n4 = long(max(0, row_hi - row_lo)) * (D / 4);
  float4* p = reinterpret_cast<float4*>(dst + size_t(row_lo) * D);
  for (long i = threadIdx.x; i < n4; i += NT) p[i] = float4{0.f, 0.f, 0.f, 0.f};
}

// dynamic LDS carve-up helper
struct Carver {
  float* p;
  __device__ float* take(int n) { float* r = p; p += n; return r; }
};

// ---------------------------------------------------------------------------------------
// Segment totals of N(X)^T Y ([feature of X][feature of Y]).  pair = blockIdx.y.
// skip_mode 0: every segment; 1 (causal): pair 0 skips the last segment, pair 1 the first.
template <int DK, int DV>
__global__ __launch_bounds__(NT) void segment_totals_f32(
    const float* __restrict__ X0, const float* __restrict__ Y0, const float* __restrict__ X1,
    const float* __restrict__ Y1, float* __restrict__ totals, size_t pair_stride, int N, int G,
    int seg_rows, float eps, int skip_mode, const int* __restrict__ seq_len, int H) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  constexpr int PK = FCfg<DK>::P, PV = FCfg<DV>::P;
  Carver cv{lds};
  float* xs = cv.take(CR * PK);
  float* ys = cv.take(CR * PV);
  float* M = cv.take(DK * PV);
  const int unit = blockIdx.x / G, g = blockIdx.x % G, pair = blockIdx.y;
  if (skip_mode == 1 && (pair == 0 ? g == G - 1 : g == 0)) return;
  const float* X = (pair == 0 ? X0 : X1) + size_t(unit) * N * DK;
  const float* Y = (pair == 0 ? Y0 : Y1) + size_t(unit) * N * DV;
  const int row_begin = g * seg_rows;
  const int row_end = min(valid_rows(seq_len, unit, H, N), row_begin + seg_rows);
  state_load<DK, DV>(M, nullptr);
  for (int row0 = row_begin; row0 < row_end; row0 += CR) {
    __syncthreads();
    load_rows<DK>(xs, X, row0, row_end, true, eps, nullptr);
    load_rows<DV>(ys, Y, row0, row_end, false, eps, nullptr);
    __syncthreads();
    state_update<DK, DV>(M, xs, ys);
  }
  __syncthreads();
  state_store<DK, DV>(totals + pair * pair_stride + (size_t(unit) * G + g) * DK * DV, M);
}

// ---------------------------------------------------------------------------------------
// Forward chunk scan of one segment.  causal: O = s [(Qh Kh^T (.) M) V + Qh S], S += Kh^T V.
// !causal (bidirectional apply): O = s Qh S with S fixed.
template <int DK, int DV>
__global__ __launch_bounds__(NT) void fwd_scan_f32(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ s, float* __restrict__ O, float* __restrict__ state_out,
    const float* __restrict__ states, const float* __restrict__ state_in, int H, int N, int G,
    int seg_rows, float eps, int causal, const int* __restrict__ seq_len, int s_per_unit) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  constexpr int PK = FCfg<DK>::P, PV = FCfg<DV>::P, CPT = FCfg<DV>::CPT;
  Carver cv{lds};
  float* qs = cv.take(CR * PK);
  float* ks = cv.take(CR * PK);
  float* vs = cv.take(CR * PV);
  float* pt = cv.take(CR * PP);
  float* S = cv.take(DK * PV);
  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const size_t kbase = size_t(unit) * N * DK, vbase = size_t(unit) * N * DV;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows, seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));
  const int i = threadIdx.x / 8, c0 = (threadIdx.x % 8) * CPT;
  // causal: state at the segment start (slot g); bidirectional: the full total (slot 0)
  const float* init = nullptr;
  if (!causal) init = states + size_t(unit) * G * DK * DV;
  else if (states != nullptr && g > 0) init = states + (size_t(unit) * G + g) * DK * DV;
  // the state the sequence starts from (causal only) is part of every segment's start state
  state_load2<DK, DV>(S, init, state_in ? state_in + size_t(unit) * DK * DV : nullptr);
  for (int row0 = row_begin; row0 < row_end; row0 += CR) {
    __syncthreads();
    load_rows<DK>(qs, Q + kbase, row0, row_end, true, eps, nullptr);
    if (causal) {
      load_rows<DK>(ks, K + kbase, row0, row_end, true, eps, nullptr);
      load_rows<DV>(vs, V + vbase, row0, row_end, false, eps, nullptr);
    }
    __syncthreads();
    if (causal) {
      pair_tile<DK>(pt, qs, ks, true);
      __syncthreads();
    }
    float acc[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) acc[e] = 0.f;
    if (causal) mac_rows<CPT>(acc, pt + i * PP, 1, CR, vs, PV, c0);
    mac_rows<CPT>(acc, qs + i * PK, 1, DK, S, PV, c0);
#pragma unroll
    for (int e = 0; e < CPT; ++e) acc[e] *= scale;
    store_rows<DV>(O + vbase, acc, row0, row_end);
    if (causal) {
      __syncthreads();
      state_update<DK, DV>(S, ks, vs);
    }
  }
  if (seq_len != nullptr) zero_rows_f32<DV>(O + vbase, row_end, seg_end);
  if (causal && state_out != nullptr && g == G - 1) {
    __syncthreads();
    state_store<DK, DV>(state_out + size_t(unit) * DK * DV, S);
  }
}

// dx = f (dxh - xh (xh . dxh)) per row, f = scale / max(||x||, eps); rows at or below eps
// skip the projection.  Returns rho = xh . dxh (same for the 8 lanes of the row).
template <int CPT>
__device__ __forceinline__ float normalise_backward(float* dx, const float* xh, float rinv,
                                                    float scale, float r_clamped) {
  float rho = 0.f;
#pragma unroll
  for (int e = 0; e < CPT; ++e) rho += xh[e] * dx[e];
  rho = group_sum<8>(rho);
  const float proj = (rinv == r_clamped) ? 0.f : rho;
  const float f = scale * rinv;
#pragma unroll
  for (int e = 0; e < CPT; ++e) dx[e] = f * (dx[e] - xh[e] * proj);
  return rho;
}

// ---------------------------------------------------------------------------------------
// dQ of one segment (forward-time scan).  causal: dqh = (A (.) M) Kh + dO S^T, S += Kh^T V;
// !causal: dqh = dO S^T with S the full total.  S is [d_key][d_value].
template <int DK, int DV>
__global__ __launch_bounds__(NT) void bwd_dq_scan_f32(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ dO, const float* __restrict__ s, float* __restrict__ dQ,
    const float* __restrict__ states, float* __restrict__ ds_partial, int H, int N, int G,
    int seg_rows, float eps, int causal, const int* __restrict__ seq_len, int s_per_unit,
    const float* __restrict__ state_in) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  constexpr int PK = FCfg<DK>::P, PV = FCfg<DV>::P, CPT = FCfg<DK>::CPT;
  Carver cv{lds};
  float* qs = cv.take(CR * PK);
  float* ks = cv.take(CR * PK);
  float* vs = cv.take(CR * PV);
  float* gs = cv.take(CR * PV);
  float* at = cv.take(CR * PP);
  float* S = cv.take(DK * PV);
  float* rq = cv.take(CR);
  float* red = cv.take(NT / 64);
  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const size_t kbase = size_t(unit) * N * DK, vbase = size_t(unit) * N * DV;
  const float scale = unit_scale(s, unit, H, s_per_unit), r_clamped = 1.0f / eps;
  const int row_begin = g * seg_rows, seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));
  const int i = threadIdx.x / 8, c0 = (threadIdx.x % 8) * CPT;
  const float* init = nullptr;
  if (!causal) init = states + size_t(unit) * G * DK * DV;
  else if (states != nullptr && g > 0) init = states + (size_t(unit) * G + g) * DK * DV;
  // the state of the rows before this piece of the sequence belongs to every segment's start
  state_load2<DK, DV>(S, init, state_in ? state_in + size_t(unit) * DK * DV : nullptr);
  float ds_lane = 0.f;
  for (int row0 = row_begin; row0 < row_end; row0 += CR) {
    __syncthreads();
    load_rows<DK>(qs, Q + kbase, row0, row_end, true, eps, rq);
    load_rows<DV>(gs, dO + vbase, row0, row_end, false, eps, nullptr);
    if (causal) {
      load_rows<DK>(ks, K + kbase, row0, row_end, true, eps, nullptr);
      load_rows<DV>(vs, V + vbase, row0, row_end, false, eps, nullptr);
    }
    __syncthreads();
    if (causal) {
      pair_tile<DV>(at, gs, vs, true);  // A_ij = dO_i . v_j, j <= i
      __syncthreads();
    }
    float acc[CPT], xh[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
      acc[e] = 0.f;
      xh[e] = qs[i * PK + c0 + e];
    }
    if (causal) mac_rows<CPT>(acc, at + i * PP, 1, CR, ks, PK, c0);
    mac_rows_t<CPT>(acc, gs + i * PV, DV, S, PV, c0);
    const float rho = normalise_backward<CPT>(acc, xh, rq[i], scale, r_clamped);
    if ((threadIdx.x % 8) == 0) ds_lane += rho;
    store_rows<DK>(dQ + kbase, acc, row0, row_end);
    if (causal) {
      __syncthreads();
      state_update<DK, DV>(S, ks, vs);
    }
  }
  if (seq_len != nullptr) zero_rows_f32<DK>(dQ + kbase, row_end, seg_end);
  if (ds_partial != nullptr) {
    ds_lane = group_sum<64>(ds_lane);
    __syncthreads();
    if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = ds_lane;
    __syncthreads();
    if (threadIdx.x == 0) ds_partial[size_t(unit) * G + g] = red[0] + red[1] + red[2] + red[3];
  }
}

// ---------------------------------------------------------------------------------------
// dK, dV of one segment (reverse-time scan).  causal: dv = (P (.) M)^T dO + Kh R,
// dkh = (A (.) M)^T Qh + V R^T, R += Qh^T dO, chunks last to first; !causal: R is the full
// total Qh^T dO and the intra-chunk terms vanish.  R is [d_key][d_value].
template <int DK, int DV>
__global__ __launch_bounds__(NT) void bwd_dkdv_scan_f32(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ dO, const float* __restrict__ s, float* __restrict__ dK,
    float* __restrict__ dV, const float* __restrict__ states, int H, int N, int G, int seg_rows,
    float eps, int causal, const int* __restrict__ seq_len, int s_per_unit,
    const float* __restrict__ rev_in, float* __restrict__ rev_out) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  constexpr int PK = FCfg<DK>::P, PV = FCfg<DV>::P, CPK = FCfg<DK>::CPT, CPV = FCfg<DV>::CPT;
  Carver cv{lds};
  float* qs = cv.take(CR * PK);
  float* ks = cv.take(CR * PK);
  float* vs = cv.take(CR * PV);
  float* gs = cv.take(CR * PV);
  float* pt = cv.take(CR * PP);
  float* at = cv.take(CR * PP);
  float* R = cv.take(DK * PV);
  float* rk = cv.take(CR);
  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const size_t kbase = size_t(unit) * N * DK, vbase = size_t(unit) * N * DV;
  const float scale = unit_scale(s, unit, H, s_per_unit), r_clamped = 1.0f / eps;
  const int row_begin = g * seg_rows, seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));
  const int n_chunks = (row_end - row_begin + CR - 1) / CR;
  const int j = threadIdx.x / 8, ck = (threadIdx.x % 8) * CPK, cv0 = (threadIdx.x % 8) * CPV;
  const float* init = nullptr;
  if (!causal) init = states + size_t(unit) * G * DK * DV;
  else if (states != nullptr && g < G - 1) init = states + (size_t(unit) * G + g) * DK * DV;
  // the reverse state of the rows after this piece of the sequence belongs to every segment
  state_load2<DK, DV>(R, init, rev_in ? rev_in + size_t(unit) * DK * DV : nullptr);
  for (int c = n_chunks - 1; c >= 0; --c) {
    const int row0 = row_begin + c * CR;
    __syncthreads();
    load_rows<DK>(ks, K + kbase, row0, row_end, true, eps, rk);
    load_rows<DV>(vs, V + vbase, row0, row_end, false, eps, nullptr);
    if (causal) {
      load_rows<DK>(qs, Q + kbase, row0, row_end, true, eps, nullptr);
      load_rows<DV>(gs, dO + vbase, row0, row_end, false, eps, nullptr);
    }
    __syncthreads();
    if (causal) {
      pair_tile<DK>(pt, qs, ks, true);  // P_ij, j <= i
      pair_tile<DV>(at, gs, vs, true);  // A_ij, j <= i
      __syncthreads();
    }
    float dv[CPV], dk[CPK], xh[CPK];
#pragma unroll
    for (int e = 0; e < CPV; ++e) dv[e] = 0.f;
#pragma unroll
    for (int e = 0; e < CPK; ++e) {
      dk[e] = 0.f;
      xh[e] = ks[j * PK + ck + e];
    }
    if (causal) {
      mac_rows<CPV>(dv, pt + j, PP, CR, gs, PV, cv0);   // sum_i P_ij dO_i
      mac_rows<CPK>(dk, at + j, PP, CR, qs, PK, ck);    // sum_i A_ij qh_i
    }
    mac_rows<CPV>(dv, ks + j * PK, 1, DK, R, PV, cv0);  // kh_j R
    mac_rows_t<CPK>(dk, vs + j * PV, DV, R, PV, ck);    // v_j R^T
    normalise_backward<CPK>(dk, xh, rk[j], scale, r_clamped);
#pragma unroll
    for (int e = 0; e < CPV; ++e) dv[e] *= scale;
    store_rows<DK>(dK + kbase, dk, row0, row_end);
    store_rows<DV>(dV + vbase, dv, row0, row_end);
    if (causal) {
      __syncthreads();
      state_update<DK, DV>(R, qs, gs);
    }
  }
  if (seq_len != nullptr) {
    zero_rows_f32<DK>(dK + kbase, row_end, seg_end);
    zero_rows_f32<DV>(dV + vbase, row_end, seg_end);
  }
  // the first segment ends with the reverse state of the whole piece and what followed it
  if (causal && rev_out != nullptr && g == 0) {
    __syncthreads();
    state_store<DK, DV>(rev_out + size_t(unit) * DK * DV, R);
  }
}

template <int DK, int DV> size_t lds_fwd() {
  return sizeof(float) * (2 * CR * FCfg<DK>::P + CR * FCfg<DV>::P + CR * PP + DK * FCfg<DV>::P);
}
template <int DK, int DV> size_t lds_tot() {
  return sizeof(float) * (CR * FCfg<DK>::P + CR * FCfg<DV>::P + DK * FCfg<DV>::P);
}
template <int DK, int DV> size_t lds_dq() {
  return sizeof(float) * (2 * CR * FCfg<DK>::P + 2 * CR * FCfg<DV>::P + CR * PP + DK * FCfg<DV>::P + CR + NT / 64);
}
template <int DK, int DV> size_t lds_dkdv() {
  return sizeof(float) * (2 * CR * FCfg<DK>::P + 2 * CR * FCfg<DV>::P + 2 * CR * PP + DK * FCfg<DV>::P + CR);
}

template <class Kern>
hipError_t allow_lds(Kern kern, size_t bytes) {
  return bytes > 65536 ? hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, int(bytes))
                       : hipSuccess;
}

template <int DK, int DV>
hipError_t run_fwd(const CausalArgs& a, bool causal) {
  const int units = a.B * a.H;
  const float* Q = static_cast<const float*>(a.Q);
  const float* K = static_cast<const float*>(a.K);
  const float* V = static_cast<const float*>(a.V);
  float* ws = static_cast<float*>(a.workspace);
  hipError_t err;
  if ((err = allow_lds(segment_totals_f32<DK, DV>, lds_tot<DK, DV>())) != hipSuccess) return err;
  if ((err = allow_lds(fwd_scan_f32<DK, DV>, lds_fwd<DK, DV>())) != hipSuccess) return err;
  if (!causal || a.G > 1) {
    err = launch_kernel("segment_totals_f32", segment_totals_f32<DK, DV>, dim3(units * a.G, 1), dim3(NT),
                        lds_tot<DK, DV>(), a.stream, K, V, K, V, ws, size_t(0), a.N, a.G, a.seg_rows,
                        a.eps, causal ? 1 : 0, a.seq_len, a.H);
    if (err != hipSuccess) return err;
    err = causal ? launch_fwd_state_carry(ws, units, a.G, DK * DV, a.stream)
                 : launch_bidir_combine(ws, 0, 1, units, a.G, DK * DV, a.state, nullptr, a.stream);
    if (err != hipSuccess) return err;
  }
  return launch_kernel("fwd_scan_f32", fwd_scan_f32<DK, DV>, dim3(units * a.G), dim3(NT), lds_fwd<DK, DV>(),
                       a.stream, Q, K, V, a.s, static_cast<float*>(a.O),
                       causal ? a.state : nullptr, (!causal || a.G > 1) ? ws : nullptr,
                       causal ? a.state_in : nullptr, a.H, a.N, a.G, a.seg_rows, a.eps,
                       causal ? 1 : 0, a.seq_len, a.s_per_unit);
}

template <int DK, int DV>
hipError_t run_bwd(const CausalArgs& a, bool causal) {
  const int units = a.B * a.H;
  const float* Q = static_cast<const float*>(a.Q);
  const float* K = static_cast<const float*>(a.K);
  const float* V = static_cast<const float*>(a.V);
  const float* dO = static_cast<const float*>(a.dO);
  char* ws = static_cast<char*>(a.workspace);
  const size_t arr = state_array_bytes(a.B, a.H, DK, DV, a.G);
  const bool have_states = !causal || a.G > 1;
  float* st0 = have_states ? reinterpret_cast<float*>(ws) : nullptr;
  float* st1 = have_states ? reinterpret_cast<float*>(ws + arr) : nullptr;
  float* ds_partial = reinterpret_cast<float*>(ws + (have_states ? 2 * arr : 0));
  hipError_t err;
  if ((err = allow_lds(segment_totals_f32<DK, DV>, lds_tot<DK, DV>())) != hipSuccess) return err;
  if ((err = allow_lds(bwd_dq_scan_f32<DK, DV>, lds_dq<DK, DV>())) != hipSuccess) return err;
  if ((err = allow_lds(bwd_dkdv_scan_f32<DK, DV>, lds_dkdv<DK, DV>())) != hipSuccess) return err;
  if (have_states) {
    err = launch_kernel("segment_totals_f32", segment_totals_f32<DK, DV>, dim3(units * a.G, 2), dim3(NT),
                        lds_tot<DK, DV>(), a.stream, K, V, Q, dO, st0, arr / sizeof(float), a.N, a.G,
                        a.seg_rows, a.eps, causal ? 1 : 0, a.seq_len, a.H);
    if (err != hipSuccess) return err;
    err = causal ? launch_bwd_state_carry(st0, st1, units, a.G, DK * DV, a.stream)
                 : launch_bidir_combine(st0, arr / sizeof(float), 2, units, a.G, DK * DV, nullptr,
                                        ds_partial, a.stream);
    if (err != hipSuccess) return err;
  }
  err = launch_kernel("bwd_dq_scan_f32", bwd_dq_scan_f32<DK, DV>, dim3(units * a.G), dim3(NT),
                      lds_dq<DK, DV>(), a.stream, Q, K, V, dO, a.s, static_cast<float*>(a.dQ), st0,
                      causal ? ds_partial : nullptr, a.H, a.N, a.G, a.seg_rows, a.eps,
                      causal ? 1 : 0, a.seq_len, a.s_per_unit, causal ? a.state_in : nullptr);
  if (err != hipSuccess) return err;
  err = launch_kernel("bwd_dkdv_scan_f32", bwd_dkdv_scan_f32<DK, DV>, dim3(units * a.G), dim3(NT),
                      lds_dkdv<DK, DV>(), a.stream, Q, K, V, dO, a.s, static_cast<float*>(a.dK),
                      static_cast<float*>(a.dV), st1, a.H, a.N, a.G, a.seg_rows, a.eps,
                      causal ? 1 : 0, a.seq_len, a.s_per_unit, causal ? a.rev_state_in : nullptr,
                      causal ? a.rev_state_out : nullptr);
  if (err != hipSuccess) return err;
  // causal: partials per (unit, segment); bidirectional: d*d/256 per unit from the combine
  return launch_reduce_ds(ds_partial, a.ds, a.B, a.H, causal ? a.G : DK * DV / 256, a.s_per_unit,
                          a.stream);
}

template <class F>
hipError_t by_d(int dk, int dv, F&& f) {
#define COTTN_F32_CASE(A, B) \
  case A * 1000 + B: return f(std::integral_constant<int, A>{}, std::integral_constant<int, B>{});
  switch (dk * 1000 + dv) {
    COTTN_F32_CASE(32, 32) COTTN_F32_CASE(32, 64) COTTN_F32_CASE(32, 128)
    COTTN_F32_CASE(64, 32) COTTN_F32_CASE(64, 64) COTTN_F32_CASE(64, 128)
    COTTN_F32_CASE(128, 32) COTTN_F32_CASE(128, 64) COTTN_F32_CASE(128, 128)
    default: return hipErrorInvalidValue;
  }
#undef COTTN_F32_CASE
}

}  // namespace

hipError_t fwd_causal_f32(const CausalArgs& a) {
  return by_d(a.dk, a.dv, [&](auto DK, auto DV) { return run_fwd<decltype(DK)::value, decltype(DV)::value>(a, true); });
}
hipError_t fwd_bidir_f32(const CausalArgs& a) {
  return by_d(a.dk, a.dv, [&](auto DK, auto DV) { return run_fwd<decltype(DK)::value, decltype(DV)::value>(a, false); });
}
hipError_t bwd_causal_f32(const CausalArgs& a) {
  return by_d(a.dk, a.dv, [&](auto DK, auto DV) { return run_bwd<decltype(DK)::value, decltype(DV)::value>(a, true); });
}
hipError_t bwd_bidir_f32(const CausalArgs& a) {
  return by_d(a.dk, a.dv, [&](auto DK, auto DV) { return run_bwd<decltype(DK)::value, decltype(DV)::value>(a, false); });
}

}  // namespace cottn
