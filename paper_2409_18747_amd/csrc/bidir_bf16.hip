// Bidirectional cosine attention, forward and backward, 16-bit storage / 16-bit MFMA / fp32
// accumulation (gfx950).  Written for a 16-bit element type: this file builds the bfloat16
// kernels, and the IEEE half ones when it is included with COTTN_ELEM_F16 defined.
//
// Sec. 4 eq. subQuadCos: without a mask the product reassociates to O = s_h Qh (Kh^T V), so
// the d x d matrix S = Kh^T V is reduced once over the whole sequence and then applied to
// every query row.  The gradient formulas of Sec. 4 with M removed collapse the same way:
// with G = Qh^T dO (also d x d),
//     dQh = s dO S^T,   dKh = s V G^T,   dV = s Kh G,   ds = <S, G> (Frobenius product),
// followed by the chain rule through the row normalisation.
//
// Launches per call:
//   totals   the segment-totals kernel of the causal forward reduces N(X)^T Y over one
//            segment of rows per workgroup (split over the sequence because B*H alone may
//            not fill the chip), for (X, Y) = (K, V) and, in the backward, (Q, dO);
//   combine  only with many segments, or in a backward that was not handed the forward's
//            totals: sums the segment totals per (batch, head) into slot 0 and forms the
//            per-(b,h) share of ds;
//   apply    streams the rows once more and multiplies them with the d x d matrices; with
//            few segments it adds up the segment totals itself while staging them.
// A backward that is handed the forward's workspace does not reduce Kh^T V again, and its
// totals kernel forms <S, G_segment> on the fly, so it is two launches.
//
// The apply kernels follow the scheme of the causal kernels: raw rows as MFMA operands,
// normalisation factors on result rows, results accumulated transposed and staged through
// the wave's own (dead) tile rows, stores one chunk late.
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
  static constexpr int TP = tile_pitch(D, C);   // operand tiles
  // the d x d matrices are written once per workgroup and then only read, as row fragments
  // too: they take the operand tiles' pitch
  static constexpr int SP = tile_pitch(D, C);
  static constexpr int TILE = C * TP;
  static constexpr int STATE = D * SP;
};

// Slot 0 of each pair <- sum over g of the slots, one matrix element per thread (grid:
// elems/256 workgroups per (batch, head)); `state` (may be null) receives pair 0; with
// n_pairs == 2 every workgroup leaves sum_e S[e] * G[e] over its 256 elements in
// ds_partial[unit][blockIdx.x], i.e. elems/256 partial sums per (batch, head).
__global__ __launch_bounds__(256) void bidir_combine(float* __restrict__ totals, size_t pair_stride,
                                                     int n_pairs, int G, int elems,
                                                     float* __restrict__ state,
                                                     float* __restrict__ ds_partial) {
  __shared__ float red[4];
  // one grid dimension: (unit, 256-element block of the matrix), so that B*H is not limited to
  // the 65535 of the other grid dimensions
  const int blocks_per_unit = elems / 256;
  const int unit = blockIdx.x / blocks_per_unit, blk = blockIdx.x % blocks_per_unit;
  const int e = blk * 256 + threadIdx.x;
  float* p0 = totals + size_t(unit) * G * elems;
  float* p1 = p0 + pair_stride;
  float a = 0.f;
  for (int g = 0; g < G; ++g) a += p0[size_t(g) * elems + e];
  p0[e] = a;
  if (state != nullptr) state[size_t(unit) * elems + e] = a;
  if (n_pairs == 2) {
    float b = 0.f;
    for (int g = 0; g < G; ++g) b += p1[size_t(g) * elems + e];
    p1[e] = b;
    const float prod = group_sum<64>(a * b);
    if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = prod;
    __syncthreads();
    if (threadIdx.x == 0)
      ds_partial[size_t(unit) * blocks_per_unit + blk] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

// dst (LDS, bf16, row-major [D][D] with row pitch SP) <- sum of the first n_sum of the
// [D][D] fp32 matrices at src; the fp32 sum also goes to `copy` when that is not null.
template <int D, int NT, int SP>
__device__ __forceinline__ void stage_summed_matrix(e16_t* dst, const float* __restrict__ src,
                                                    int n_sum, float* __restrict__ copy) {
  for (int e = 4 * threadIdx.x; e < D * D; e += 4 * NT) {
    f32x4 a = *reinterpret_cast<const f32x4*>(src + e);
    for (int j = 1; j < n_sum; ++j) {
      const f32x4 b = *reinterpret_cast<const f32x4*>(src + size_t(j) * D * D + e);
#pragma unroll
      for (int v = 0; v < 4; ++v) a[v] += b[v];
    }
    if (copy != nullptr) *reinterpret_cast<f32x4*>(copy + e) = a;
    uint2 pk;
    pk.x = pack2(a[0], a[1]);
    pk.y = pack2(a[2], a[3]);
    *reinterpret_cast<uint2*>(dst + (e / D) * SP + e % D) = pk;
  }
}

// O rows of one segment: O_i = s r_i (q_i S), accumulated as O^T = S^T Q^T.  `totals` holds
// n_sum stored matrices per unit at a stride of `slots` matrices; the workgroup of segment 0
// writes their sum to `state` when that is asked for.
template <int D, int C>
__global__ __launch_bounds__(C * 4) void COTTN_SYM(fwd_bidir_apply)(
    const e16_t* __restrict__ Q, const float* __restrict__ s, e16_t* __restrict__ O,
    const float* __restrict__ totals, int slots, int n_sum, float* __restrict__ state, int H, int N,
    int G, int seg_rows, float inv_eps, const int* __restrict__ seq_len, int s_per_unit) {
  using Cfg = BiCfg<D, C>;
  using Stage = TileStage<D, C, Cfg::NT>;
  constexpr int TP = Cfg::TP, SP = Cfg::SP;
  __shared__ __attribute__((aligned(16))) e16_t Qs[Cfg::TILE];   // raw q
  __shared__ __attribute__((aligned(16))) e16_t Sl[Cfg::STATE];  // [d_key][d_value]
  __shared__ float rq[C];

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const e16_t* Qu = Q + ubase;
  e16_t* Ou = O + ubase;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows;
  const int seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));

  Stage qst;
  qst.fetch(Qu, row_begin, row_end);
  stage_summed_matrix<D, Cfg::NT, Cfg::SP>(Sl, totals + size_t(unit) * slots * D * D, n_sum,
                                  (state != nullptr && g == 0) ? state + size_t(unit) * D * D
                                                               : nullptr);

  RowPieces<D> finished;  // output rows of the previous chunk, stored one chunk late
#pragma unroll
  for (int j = 0; j < RowPieces<D>::PER_LANE; ++j) finished.v[j] = uint4{0u, 0u, 0u, 0u};
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    {
      float rqv[Stage::PASSES];
      qst.row_rinv(inv_eps, rqv);
      qst.commit_plain(Qs);
      qst.store_rinv(rq, rqv);
    }
    if (row0 + C < row_end) qst.fetch(Qu, row0 + C, row_end);
    if (row0 > row_begin) store_row_pieces<D>(finished, Ou, row0 - C + 16 * w, row_end, l);
    __syncthreads();
    // oacc[nt][v] = (q S)[query 16w + r][value 16 nt + 4 q4 + v]
    f32x4 oacc[Cfg::DT];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt) oacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    frag8 qf[Cfg::KS], sf[Cfg::KS][Cfg::DT];
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks) {
      qf[ks] = lds_row_frag(Qs + (16 * w + r) * TP + 32 * ks + 8 * q4);
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt)
        sf[ks][nt] = lds_col_frag(Sl, SP, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, 16 * nt, r);
    }
    __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks)
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) oacc[nt] = mma16(sf[ks][nt], qf[ks], oacc[nt]);
    __builtin_amdgcn_sched_barrier(0);
    const float row_factor = scale * rq[16 * w + r];
    wave_lds_sync();  // this wave's reads of its Qs rows precede the staging writes
    gather_rows_transposed<D>(oacc, row_factor, Qs + 16 * w * TP, l, finished);
    __syncthreads();
  }
  if (row_begin < row_end) {
    const int last = row_begin + (row_end - row_begin - 1) / C * C;
    store_row_pieces<D>(finished, Ou, last + 16 * w, row_end, l);
  }
  if (seq_len != nullptr) zero_rows_e16<D>(Ou, row_end, seg_end);  // rows that do not exist
}

// dQ, dK, dV rows of one segment; the first H workgroups also finish ds from the n_ds
// partial sums per (batch, head).  All products are accumulated transposed:
//   dqh^T = S dO^T (over d_value),  dkh^T = G V^T (over d_value),  (k G)^T = G^T k^T (over
//   d_key), then dq_i = s r_i (dqh_i - qh_i (qh_i . dqh_i)), dk_j likewise, dv_j = s r_j (k_j G).
template <int D, int C>
__global__ __launch_bounds__(C * 4) void COTTN_SYM(bwd_bidir_apply)(
    const e16_t* __restrict__ Q, const e16_t* __restrict__ K, const e16_t* __restrict__ V,
    const e16_t* __restrict__ dO, const float* __restrict__ s, e16_t* __restrict__ dQ,
    e16_t* __restrict__ dK, e16_t* __restrict__ dV, const float* __restrict__ s_totals,
    const float* __restrict__ g_totals, int slots, int n_sum, const float* __restrict__ ds_partial,
    int n_ds, float* __restrict__ ds, int B, int H, int N, int G, int seg_rows, float inv_eps,
    const int* __restrict__ seq_len, int s_per_unit) {
  using Cfg = BiCfg<D, C>;
  using Stage = TileStage<D, C, Cfg::NT>;
  constexpr int TP = Cfg::TP, SP = Cfg::SP;
  __shared__ __attribute__((aligned(16))) e16_t Qs[Cfg::TILE];   // raw q
  __shared__ __attribute__((aligned(16))) e16_t Ks[Cfg::TILE];   // raw k
  __shared__ __attribute__((aligned(16))) e16_t Vs[Cfg::TILE];
  __shared__ __attribute__((aligned(16))) e16_t Gs[Cfg::TILE];   // dO
  __shared__ __attribute__((aligned(16))) e16_t Sl[Cfg::STATE];  // Kh^T V,  [d_key][d_value]
  __shared__ __attribute__((aligned(16))) e16_t Gl[Cfg::STATE];  // Qh^T dO, [d_key][d_value]
  __shared__ float rq[C], rk[C];

  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const size_t ubase = size_t(unit) * N * D;
  const e16_t* Qu = Q + ubase;
  const e16_t* Ku = K + ubase;
  const e16_t* Vu = V + ubase;
  const e16_t* Gu = dO + ubase;
  e16_t* dQu = dQ + ubase;
  e16_t* dKu = dK + ubase;
  e16_t* dVu = dV + ubase;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows;
  const int seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));

  Stage qst, kst, vst, gst;
  qst.fetch(Qu, row_begin, row_end);
  kst.fetch(Ku, row_begin, row_end);
  vst.fetch(Vu, row_begin, row_end);
  gst.fetch(Gu, row_begin, row_end);

  // ds[h] = sum of the shares of all batches (ds[b][h], one batch, with a scale per unit)
  if (int(blockIdx.x) < (s_per_unit ? B * H : H) && w == 0) {
    float t = 0.f;
    const int n = s_per_unit ? n_ds : B * n_ds;
    for (int i = l; i < n; i += 64)
      t += s_per_unit ? ds_partial[size_t(blockIdx.x) * n_ds + i]
                      : ds_partial[(size_t(i / n_ds) * H + blockIdx.x) * n_ds + (i % n_ds)];
    t = group_sum<64>(t);
    if (l == 0) ds[blockIdx.x] = t;
  }
  stage_summed_matrix<D, Cfg::NT, Cfg::SP>(Sl, s_totals + size_t(unit) * slots * D * D, n_sum, nullptr);
  stage_summed_matrix<D, Cfg::NT, Cfg::SP>(Gl, g_totals + size_t(unit) * slots * D * D, n_sum, nullptr);

  RowPieces<D> done_q, done_k, done_v;  // rows of the previous chunk, stored one chunk late
#pragma unroll
  for (int j = 0; j < RowPieces<D>::PER_LANE; ++j)
    done_q.v[j] = done_k.v[j] = done_v.v[j] = uint4{0u, 0u, 0u, 0u};
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    {
      float rqv[Stage::PASSES], rkv[Stage::PASSES];
      qst.row_rinv(inv_eps, rqv);
      kst.row_rinv(inv_eps, rkv);
      qst.commit_plain(Qs);
      qst.store_rinv(rq, rqv);
      kst.commit_plain(Ks);
      kst.store_rinv(rk, rkv);
      vst.commit_plain(Vs);
      gst.commit_plain(Gs);
    }
    if (row0 + C < row_end) {
      qst.fetch(Qu, row0 + C, row_end);
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
      gst.fetch(Gu, row0 + C, row_end);
    }
    if (row0 > row_begin) {
      store_row_pieces<D>(done_q, dQu, row0 - C + 16 * w, row_end, l);
      store_row_pieces<D>(done_k, dKu, row0 - C + 16 * w, row_end, l);
      store_row_pieces<D>(done_v, dVu, row0 - C + 16 * w, row_end, l);
    }
    __syncthreads();

    // d*[nt][v] = result[row 16w + r][feature 16 nt + 4 q4 + v]
    f32x4 dq[Cfg::DT], dk[Cfg::DT], dv[Cfg::DT];
#pragma unroll
    for (int nt = 0; nt < Cfg::DT; ++nt) {
      dq[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
      dk[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
      dv[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int ks = 0; ks < Cfg::KS; ++ks) {
      const int off = (16 * w + r) * TP + 32 * ks + 8 * q4;
      const frag8 gf = lds_row_frag(Gs + off), vf = lds_row_frag(Vs + off),
                   kf = lds_row_frag(Ks + off);
      frag8 srow[Cfg::DT], grow[Cfg::DT], gcol[Cfg::DT];
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) {
        const int soff = (16 * nt + r) * SP + 32 * ks + 8 * q4;
        srow[nt] = lds_row_frag(Sl + soff);
        grow[nt] = lds_row_frag(Gl + soff);
        gcol[nt] = lds_col_frag(Gl, SP, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, 16 * nt, r);
      }
      __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
      for (int nt = 0; nt < Cfg::DT; ++nt) {
        dq[nt] = mma16(srow[nt], gf, dq[nt]);   // S dO^T   (over d_value)
        dk[nt] = mma16(grow[nt], vf, dk[nt]);   // G V^T    (over d_value)
        dv[nt] = mma16(gcol[nt], kf, dv[nt]);   // G^T k^T  (over d_key)
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // every tile row is private to its wave here: chain rule on the raw rows, then the
    // results are staged in place (dO rows for dQ, K rows for dK, V rows for dV)
    const float ri = rq[16 * w + r], rj = rk[16 * w + r];
    project_out_row<D, TP, false>(dq, Qs + 16 * w * TP, ri, inv_eps, r, q4);
    project_out_row<D, TP, false>(dk, Ks + 16 * w * TP, rj, inv_eps, r, q4);
    wave_lds_sync();  // own rows of Gs, Ks, Vs were read before the staging writes
    gather_rows_transposed<D>(dq, scale * ri, Gs + 16 * w * TP, l, done_q);
    gather_rows_transposed<D>(dk, scale * rj, Ks + 16 * w * TP, l, done_k);
    gather_rows_transposed<D>(dv, scale * rj, Vs + 16 * w * TP, l, done_v);
    __syncthreads();
  }
  if (row_begin < row_end) {
    const int last = row_begin + (row_end - row_begin - 1) / C * C;
    store_row_pieces<D>(done_q, dQu, last + 16 * w, row_end, l);
    store_row_pieces<D>(done_k, dKu, last + 16 * w, row_end, l);
    store_row_pieces<D>(done_v, dVu, last + 16 * w, row_end, l);
  }
  if (seq_len != nullptr) {  // rows that do not exist
    zero_rows_e16<D>(dQu, row_end, seg_end);
    zero_rows_e16<D>(dKu, row_end, seg_end);
    zero_rows_e16<D>(dVu, row_end, seg_end);
  }
}

SegmentTotalsArgs totals_args(const CausalArgs& a, const void* X, const void* Y, float* dst) {
  SegmentTotalsArgs t{};
  t.X = X; t.Y = Y; t.dst = dst;
  t.units = a.B * a.H; t.N = a.N; t.d = a.d; t.G = a.G; t.n_compute = a.G;
  t.seg_rows = a.seg_rows; t.eps = a.eps; t.stream = a.stream;
  t.seq_len = a.seq_len; t.H = a.H;
  return t;
}

template <int D>
hipError_t run_fwd_bidir(const CausalArgs& a) {
  constexpr int C = 64;
  using Cfg = BiCfg<D, C>;
  const int units = a.B * a.H;
  float* totals = static_cast<float*>(a.workspace);
  hipError_t err = COTTN_SYM(launch_segment_totals)(totals_args(a, a.K, a.V, totals));
  if (err != hipSuccess) return err;
  // few segments: the apply workgroups add the totals up themselves (and write `state`)
  const bool sum_in_apply = a.G <= kMaxSegmentsSummedInScan;
  if (!sum_in_apply) {
    err = launch_bidir_combine(totals, 0, 1, units, a.G, D * D, a.state, nullptr, a.stream);
    if (err != hipSuccess) return err;
  }
  return launch_kernel(COTTN_SYM_STR(fwd_bidir_apply), COTTN_SYM(fwd_bidir_apply)<D, C>, dim3(units * a.G),
                       dim3(Cfg::NT), 0, a.stream, static_cast<const e16_t*>(a.Q), a.s,
                       static_cast<e16_t*>(a.O), totals, a.G, sum_in_apply ? a.G : 1,
                       sum_in_apply ? a.state : nullptr, a.H, a.N, a.G, a.seg_rows, 1.0f / a.eps,
                       a.seq_len, a.s_per_unit);
}

template <int D>
hipError_t run_bwd_bidir(const CausalArgs& a) {
  constexpr int C = 64;
  using Cfg = BiCfg<D, C>;
  const int units = a.B * a.H;
  char* ws = static_cast<char*>(a.workspace);
  float* s_totals = reinterpret_cast<float*>(ws);
  const size_t pair_stride = state_array_bytes(a.B, a.H, D, a.G) / sizeof(float);
  float* g_totals = s_totals + pair_stride;
  float* ds_partial = reinterpret_cast<float*>(ws + 2 * state_array_bytes(a.B, a.H, D, a.G));
  const bool few = a.G <= kMaxSegmentsSummedInScan;
  hipError_t err;
  const float* s_src = s_totals;
  int n_sum = 1, n_ds = 1;
  if (few && a.saved_fwd_states != nullptr) {
    // the forward left the segment totals of Kh^T V behind: only Qh^T dO is reduced here, and
    // the same kernel forms the share <S, G_segment> of ds
    SegmentTotalsArgs t = totals_args(a, a.Q, a.dO, g_totals);
    t.dot_with = a.saved_fwd_states; t.dot_slots = a.G; t.dot_out = ds_partial;
    err = COTTN_SYM(launch_segment_totals)(t);
    if (err != hipSuccess) return err;
    s_src = a.saved_fwd_states;
    n_sum = a.G;
    n_ds = a.G;
  } else {
    err = COTTN_SYM(launch_segment_totals)(totals_args(a, a.K, a.V, s_totals));
    if (err != hipSuccess) return err;
    err = COTTN_SYM(launch_segment_totals)(totals_args(a, a.Q, a.dO, g_totals));
    if (err != hipSuccess) return err;
    err = launch_bidir_combine(s_totals, pair_stride, 2, units, a.G, D * D, nullptr, ds_partial,
                               a.stream);
    if (err != hipSuccess) return err;
    n_ds = D * D / 256;  // the combine kernel's partial sums per (batch, head)
  }
  return launch_kernel(COTTN_SYM_STR(bwd_bidir_apply), COTTN_SYM(bwd_bidir_apply)<D, C>, dim3(units * a.G),
                       dim3(Cfg::NT), 0, a.stream, static_cast<const e16_t*>(a.Q),
                       static_cast<const e16_t*>(a.K), static_cast<const e16_t*>(a.V),
                       static_cast<const e16_t*>(a.dO), a.s, static_cast<e16_t*>(a.dQ),
                       static_cast<e16_t*>(a.dK), static_cast<e16_t*>(a.dV), s_src, g_totals, a.G,
                       n_sum, ds_partial, n_ds, a.ds, a.B, a.H, a.N, a.G, a.seg_rows, 1.0f / a.eps,
                       a.seq_len, a.s_per_unit);
}

}  // namespace

#ifndef COTTN_ELEM_F16  // not specific to the element type: defined once, by the bf16 build
hipError_t launch_bidir_combine(float* totals, size_t pair_stride, int n_pairs, int units, int G,
                                int elems, float* state, float* ds_partial, hipStream_t st) {
  return launch_kernel("bidir_combine", bidir_combine, dim3(unsigned(elems / 256) * units), dim3(256), 0, st,
                       totals, pair_stride, n_pairs, G, elems, state, ds_partial);
}
#endif

hipError_t COTTN_SYM(fwd_bidir)(const CausalArgs& a) {
  switch (a.d) {
    case 32: return run_fwd_bidir<32>(a);
    case 64: return run_fwd_bidir<64>(a);
    case 128: return run_fwd_bidir<128>(a);
    default: return hipErrorInvalidValue;
  }
}

hipError_t COTTN_SYM(bwd_bidir)(const CausalArgs& a) {
  switch (a.d) {
    case 32: return run_bwd_bidir<32>(a);
    case 64: return run_bwd_bidir<64>(a);
    case 128: return run_bwd_bidir<128>(a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cottn
