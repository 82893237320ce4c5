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
//   forward   totals: the segment-totals kernel of the causal forward reduces Kh^T V over one
//             segment of rows per workgroup (split over the sequence because B*H alone may not
//             fill the chip); apply: streams the Q rows and multiplies them with S;
//   backward  first sweep (Q, dO -> dQ): dQ needs only S, which the forward left behind, so
//             the sweep that has to read Q and dO for G = Qh^T dO forms dQ on the way and
//             leaves G's segment totals and the shares of ds (= sum_i qh_i . dqh_i, the same
//             number as <S, G>); second sweep (K, V -> dK, dV) applies G.  Every row of the
//             seven tensors is moved once.  A backward that was not handed the forward's
//             totals reduces Kh^T V first;
//   combine   only with many segments: sums the segment totals per (batch, head) into slot 0;
//             with few, the kernels add the totals up themselves while staging them.
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

// DK, DV: head dimensions of queries / keys and of values / outputs (Sec. 2.1); the matrices
// S = Kh^T V and G = Qh^T dO are DK x DV.
template <int DK, int DV, int C>
struct BiCfg {
  static constexpr int NW = C / 16;
  static constexpr int NT = NW * 64;
  static constexpr int DTK = DK / 16, DTV = DV / 16;
  static constexpr int KSK = DK / 32, KSV = DV / 32;
  static constexpr int TPK = tile_pitch(DK, C), TPV = tile_pitch(DV, C);   // operand tiles
  // the DK x DV matrices are written once per workgroup and then only read, as row fragments
  // too: they take the operand tiles' pitch
  static constexpr int SP = tile_pitch(DV, C);
  static constexpr int TILEK = C * TPK, TILEV = C * TPV;
  static constexpr int STATE = DK * SP;
  // the forward stages finished output rows (DV wide) in the wave's own dead query rows when
  // those are wide enough, else in a tile of their own
  static constexpr bool FWD_OWN_STAGE = lds_pitch(DV) > TPK;
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

// dst (LDS, bf16, row-major [DK][DV] with row pitch SP) <- sum of the first n_sum of the
// [DK][DV] fp32 matrices at src; the fp32 sum also goes to `copy` when that is not null.
template <int DK, int DV, int NT, int SP>
__device__ __forceinline__ void stage_summed_matrix(e16_t* dst, const float* __restrict__ src,
                                                    int n_sum, float* __restrict__ copy) {
  for (int e = 4 * threadIdx.x; e < DK * DV; e += 4 * NT) {
    f32x4 a = *reinterpret_cast<const f32x4*>(src + e);
    for (int j = 1; j < n_sum; ++j) {
      const f32x4 b = *reinterpret_cast<const f32x4*>(src + size_t(j) * DK * DV + e);
#pragma unroll
      for (int v = 0; v < 4; ++v) a[v] += b[v];
    }
    if (copy != nullptr) *reinterpret_cast<f32x4*>(copy + e) = a;
    uint2 pk;
    pk.x = pack2(a[0], a[1]);
    pk.y = pack2(a[2], a[3]);
    *reinterpret_cast<uint2*>(dst + (e / DV) * SP + e % DV) = pk;
  }
}

// O rows of one segment: O_i = s r_i (q_i S), accumulated as O^T = S^T Q^T.  `totals` holds
// n_sum stored matrices per unit at a stride of `slots` matrices; the workgroup of segment 0
// writes their sum to `state` when that is asked for.
template <int DK, int DV, int C>
__global__ __launch_bounds__(C * 4) void COTTN_SYM(fwd_bidir_apply)(
    const e16_t* __restrict__ Q, const float* __restrict__ s, e16_t* __restrict__ O,
    const float* __restrict__ totals, int slots, int n_sum, float* __restrict__ state, int H, int N,
    int G, int seg_rows, float inv_eps, const int* __restrict__ seq_len, int s_per_unit) {
  using Cfg = BiCfg<DK, DV, C>;
  using Stage = TileStage<DK, C, Cfg::NT>;
  constexpr int TP = Cfg::TPK, SP = Cfg::SP;
  __shared__ __attribute__((aligned(16))) e16_t Qs[Cfg::TILEK];  // raw q
  __shared__ __attribute__((aligned(16))) e16_t Sl[Cfg::STATE];  // [d_key][d_value]
  __shared__ __attribute__((aligned(16))) e16_t Os[Cfg::FWD_OWN_STAGE ? Cfg::TILEV : 8];
  __shared__ float rq[C];

  fetch_argument_now(Q, s, O, totals, slots, n_sum, state, H, N, G, seg_rows, inv_eps, seq_len,
                     s_per_unit);
  int unit, g;
  unit_and_segment(blockIdx.x, G, unit, g);
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const e16_t* Qu = Q + size_t(unit) * N * DK;
  e16_t* Ou = O + size_t(unit) * N * DV;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows;
  const int seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));

  Stage qst;
  qst.fetch(Qu, row_begin, row_end);
  stage_summed_matrix<DK, DV, Cfg::NT, Cfg::SP>(Sl, totals + size_t(unit) * slots * DK * DV, n_sum,
                                  (state != nullptr && g == 0) ? state + size_t(unit) * DK * DV
                                                               : nullptr);

  RowPieces<DV> finished;  // output rows of the previous chunk, stored one chunk late
#pragma unroll
  for (int j = 0; j < RowPieces<DV>::PER_LANE; ++j) finished.v[j] = uint4{0u, 0u, 0u, 0u};
  e16_t* stage = Cfg::FWD_OWN_STAGE ? Os + 16 * w * Cfg::TPV : Qs + 16 * w * TP;
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    {
      float rqv[Stage::PASSES];
      qst.row_rinv(inv_eps, rqv);
      qst.commit_plain(Qs);
      qst.store_rinv(rq, rqv);
    }
    if (row0 + C < row_end) qst.fetch(Qu, row0 + C, row_end);
    if (row0 > row_begin) store_row_pieces<DV>(finished, Ou, row0 - C + 16 * w, row_end, l);
    __syncthreads();
    // oacc[nt][v] = (q S)[query 16w + r][value 16 nt + 4 q4 + v]
    f32x4 oacc[Cfg::DTV];
#pragma unroll
    for (int nt = 0; nt < Cfg::DTV; ++nt) oacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    frag8 qf[Cfg::KSK], sf[Cfg::KSK][Cfg::DTV];
#pragma unroll
    for (int ks = 0; ks < Cfg::KSK; ++ks) {
      qf[ks] = lds_row_frag(Qs + (16 * w + r) * TP + 32 * ks + 8 * q4);
#pragma unroll
      for (int nt = 0; nt < Cfg::DTV; ++nt)
        sf[ks][nt] = lds_col_frag(Sl, SP, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, 16 * nt, r);
    }
    __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
    for (int ks = 0; ks < Cfg::KSK; ++ks)
#pragma unroll
      for (int nt = 0; nt < Cfg::DTV; ++nt) oacc[nt] = mma16(sf[ks][nt], qf[ks], oacc[nt]);
    __builtin_amdgcn_sched_barrier(0);
    const float row_factor = scale * rq[16 * w + r];
    wave_lds_sync();  // this wave's reads of its Qs rows precede the staging writes
    gather_rows_transposed<DV>(oacc, row_factor, stage, l, finished);
    __syncthreads();
  }
  if (row_begin < row_end) {
    const int last = row_begin + (row_end - row_begin - 1) / C * C;
    store_row_pieces<DV>(finished, Ou, last + 16 * w, row_end, l);
  }
  if (seq_len != nullptr) zero_rows_e16<DV>(Ou, row_end, seg_end);  // rows that do not exist
}

// Backward, first sweep: dQ rows of one segment and the segment's total of Qh^T dO.  It needs
// only S = Kh^T V, which the forward already reduced, so the rows of Q and dO are read once,
// here, for both dQ and the matrix G that the second sweep applies:
//   dqh^T = S dO^T (over d_value),  dq_i = s r_i (dqh_i - qh_i (qh_i . dqh_i)),
//   G_segment = sum over the rows of qh_i^T dO_i,  ds share = sum of qh_i . dqh_i.
// Q is stored in LDS as qh = r_i q_i: it is contracted over the tokens in G, and the chain
// rule wants the normalised row anyway.  Every wave reads all rows of both tiles (the total
// contracts them over the tokens), so finished dQ rows are staged in a tile of their own.
template <int DK, int DV, int C>
__global__ __launch_bounds__(C * 4) void COTTN_SYM(bwd_bidir_dq)(
    const e16_t* __restrict__ Q, const e16_t* __restrict__ dO, const float* __restrict__ s,
    e16_t* __restrict__ dQ, const float* __restrict__ s_totals, int slots, int n_sum,
    float* __restrict__ g_totals, float* __restrict__ ds_partial, int H, int N, int G,
    int seg_rows, float inv_eps, const int* __restrict__ seq_len, int s_per_unit) {
  using Cfg = BiCfg<DK, DV, C>;
  using RT = AccTiles<DV, DK, Cfg::NW>;   // total of Qh^T dO: value rows, key columns
  using StageK = TileStage<DK, C, Cfg::NT>;
  using StageV = TileStage<DV, C, Cfg::NT>;
  constexpr int TPK = Cfg::TPK, TPV = Cfg::TPV, SP = Cfg::SP;
  __shared__ __attribute__((aligned(16))) e16_t Qs[Cfg::TILEK];   // qh = r_i q_i
  __shared__ __attribute__((aligned(16))) e16_t Gs[Cfg::TILEV];   // dO
  __shared__ __attribute__((aligned(16))) e16_t Os[Cfg::TILEK];   // finished dQ rows
  __shared__ __attribute__((aligned(16))) e16_t Sl[Cfg::STATE];   // Kh^T V, [d_key][d_value]
  __shared__ float rq[C];
  __shared__ float ds_wave[Cfg::NW];

  fetch_argument_now(Q, dO, s, dQ, s_totals, slots, n_sum, g_totals, ds_partial, H, N, G, seg_rows,
                     inv_eps, seq_len, s_per_unit);
  int unit, g;
  unit_and_segment(blockIdx.x, G, unit, g);
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const e16_t* Qu = Q + size_t(unit) * N * DK;
  const e16_t* Gu = dO + size_t(unit) * N * DV;
  e16_t* dQu = dQ + size_t(unit) * N * DK;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows;
  const int seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));

  StageK qst;
  StageV gst;
  qst.fetch(Qu, row_begin, row_end);
  gst.fetch(Gu, row_begin, row_end);
  stage_summed_matrix<DK, DV, Cfg::NT, Cfg::SP>(Sl, s_totals + size_t(unit) * slots * DK * DV, n_sum, nullptr);

  // racc[x][y]: element [v] of lane (r, q4) is G[key 16 ct + r][value 16 rt + 4 q4 + v]
  f32x4 racc[RT::NCT][RT::NRT];
#pragma unroll
  for (int x = 0; x < RT::NCT; ++x)
#pragma unroll
    for (int y = 0; y < RT::NRT; ++y) racc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};
  float ds_lane = 0.f;
  RowPieces<DK> finished;  // dQ rows of the previous chunk, stored one chunk late
#pragma unroll
  for (int j = 0; j < RowPieces<DK>::PER_LANE; ++j) finished.v[j] = uint4{0u, 0u, 0u, 0u};
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    {
      float rqv[StageK::PASSES];
      qst.row_rinv(inv_eps, rqv);
      qst.commit_scaled(Qs, rqv);
      qst.store_rinv(rq, rqv);
      gst.commit_plain(Gs);
    }
    if (row0 + C < row_end) {
      qst.fetch(Qu, row0 + C, row_end);
      gst.fetch(Gu, row0 + C, row_end);
    }
    if (row0 > row_begin) store_row_pieces<DK>(finished, dQu, row0 - C + 16 * w, row_end, l);
    __syncthreads();

    // dq[nt][v] = dqh[row 16w + r][key feature 16 nt + 4 q4 + v]
    f32x4 dq[Cfg::DTK];
#pragma unroll
    for (int nt = 0; nt < Cfg::DTK; ++nt) dq[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < Cfg::KSV; ++ks) {
      const frag8 gf = lds_row_frag(Gs + (16 * w + r) * TPV + 32 * ks + 8 * q4);
      frag8 srow[Cfg::DTK];
#pragma unroll
      for (int nt = 0; nt < Cfg::DTK; ++nt)
        srow[nt] = lds_row_frag(Sl + (16 * nt + r) * SP + 32 * ks + 8 * q4);
      __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
      for (int nt = 0; nt < Cfg::DTK; ++nt) dq[nt] = mma16(srow[nt], gf, dq[nt]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // G^T += dO^T qh over the chunk's tokens, 32 at a time (rows beyond the sequence are zero)
    if (RT::active(w)) {
#pragma unroll
      for (int p = 0; p < C / 32; ++p) {
        const int t0 = 32 * p + 4 * q4, t1 = 32 * p + 16 + 4 * q4;
        frag8 qcol[RT::NCT], grow[RT::NRT];
#pragma unroll
        for (int x = 0; x < RT::NCT; ++x)
          qcol[x] = lds_col_frag(Qs, TPK, t0, t1, 16 * RT::col_tile(w, x), r);
#pragma unroll
        for (int y = 0; y < RT::NRT; ++y)
          grow[y] = lds_col_frag(Gs, TPV, t0, t1, 16 * RT::row_tile(w, y), r);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int y = 0; y < RT::NRT; ++y)
#pragma unroll
          for (int x = 0; x < RT::NCT; ++x) racc[x][y] = mma16(grow[y], qcol[x], racc[x][y]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    const float ri = rq[16 * w + r];
    const float rho = project_out_row<DK, TPK, true>(dq, Qs + 16 * w * TPK, ri, inv_eps, r, q4);
    if (q4 == 0) ds_lane += rho;
    gather_rows_transposed<DK>(dq, scale * ri, Os + 16 * w * TPK, l, finished);
    __syncthreads();
  }
  if (row_begin < row_end) {
    const int last = row_begin + (row_end - row_begin - 1) / C * C;
    store_row_pieces<DK>(finished, dQu, last + 16 * w, row_end, l);
  }
  if (seq_len != nullptr) zero_rows_e16<DK>(dQu, row_end, seg_end);  // rows that do not exist

  if (RT::active(w)) {
    float* out = g_totals + (size_t(unit) * slots + g) * DK * DV;
#pragma unroll
    for (int x = 0; x < RT::NCT; ++x)
#pragma unroll
      for (int y = 0; y < RT::NRT; ++y)
        store_state_words(out + (16 * RT::col_tile(w, x) + r) * DV + 16 * RT::row_tile(w, y) + 4 * q4,
                          racc[x][y]);
  }
  // the segment's share of ds: lanes of the first lane row hold the row sums
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

// Backward, second sweep: dK and dV rows of one segment from G = Qh^T dO (the sum of the n_sum
// stored matrices at g_totals); the first H workgroups also finish ds from the n_ds partial
// sums per (batch, head) that the first sweep left.  Accumulated transposed:
//   dkh^T = G V^T (over d_value),  (k G)^T = G^T k^T (over d_key),
//   dk_j = s r_j (dkh_j - kh_j (kh_j . dkh_j)),  dv_j = s r_j (k_j G).
template <int DK, int DV, int C>
__global__ __launch_bounds__(C * 4) void COTTN_SYM(bwd_bidir_dkdv)(
    const e16_t* __restrict__ K, const e16_t* __restrict__ V, const float* __restrict__ s,
    e16_t* __restrict__ dK, e16_t* __restrict__ dV, const float* __restrict__ g_totals, int slots,
    int n_sum, const float* __restrict__ ds_partial, int n_ds, float* __restrict__ ds, int B, int H,
    int N, int G, int seg_rows, float inv_eps, const int* __restrict__ seq_len, int s_per_unit) {
  using Cfg = BiCfg<DK, DV, C>;
  using StageK = TileStage<DK, C, Cfg::NT>;
  using StageV = TileStage<DV, C, Cfg::NT>;
  constexpr int TPK = Cfg::TPK, TPV = Cfg::TPV, SP = Cfg::SP;
  __shared__ __attribute__((aligned(16))) e16_t Ks[Cfg::TILEK];   // raw k
  __shared__ __attribute__((aligned(16))) e16_t Vs[Cfg::TILEV];
  __shared__ __attribute__((aligned(16))) e16_t Gl[Cfg::STATE];  // Qh^T dO, [d_key][d_value]
  __shared__ float rk[C];

  fetch_argument_now(K, V, s, dK, dV, g_totals, slots, n_sum, ds_partial, n_ds, ds, B, H, N, G,
                     seg_rows, inv_eps, seq_len, s_per_unit);
  int unit, g;
  unit_and_segment(blockIdx.x, G, unit, g);
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const e16_t* Ku = K + size_t(unit) * N * DK;
  const e16_t* Vu = V + size_t(unit) * N * DV;
  e16_t* dKu = dK + size_t(unit) * N * DK;
  e16_t* dVu = dV + size_t(unit) * N * DV;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows;
  const int seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));

  StageK kst;
  StageV vst;
  kst.fetch(Ku, row_begin, row_end);
  vst.fetch(Vu, row_begin, row_end);

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
  stage_summed_matrix<DK, DV, Cfg::NT, Cfg::SP>(Gl, g_totals + size_t(unit) * slots * DK * DV, n_sum, nullptr);

  RowPieces<DK> done_k;  // rows of the previous chunk, stored one chunk late
  RowPieces<DV> done_v;
#pragma unroll
  for (int j = 0; j < RowPieces<DK>::PER_LANE; ++j) done_k.v[j] = uint4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < RowPieces<DV>::PER_LANE; ++j) done_v.v[j] = uint4{0u, 0u, 0u, 0u};
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    {
      float rkv[StageK::PASSES];
      kst.row_rinv(inv_eps, rkv);
      kst.commit_plain(Ks);
      kst.store_rinv(rk, rkv);
      vst.commit_plain(Vs);
    }
    if (row0 + C < row_end) {
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
    }
    if (row0 > row_begin) {
      store_row_pieces<DK>(done_k, dKu, row0 - C + 16 * w, row_end, l);
      store_row_pieces<DV>(done_v, dVu, row0 - C + 16 * w, row_end, l);
    }
    __syncthreads();

    // d*[nt][v] = result[row 16w + r][feature 16 nt + 4 q4 + v]
    f32x4 dk[Cfg::DTK], dv[Cfg::DTV];
#pragma unroll
    for (int nt = 0; nt < Cfg::DTK; ++nt) dk[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int nt = 0; nt < Cfg::DTV; ++nt) dv[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // G V^T contracts over d_value (row fragments of Gl along its rows)
#pragma unroll
    for (int ks = 0; ks < Cfg::KSV; ++ks) {
      const frag8 vf = lds_row_frag(Vs + (16 * w + r) * TPV + 32 * ks + 8 * q4);
      frag8 grow[Cfg::DTK];
#pragma unroll
      for (int nt = 0; nt < Cfg::DTK; ++nt)
        grow[nt] = lds_row_frag(Gl + (16 * nt + r) * SP + 32 * ks + 8 * q4);
      __builtin_amdgcn_sched_barrier(0);  // all LDS reads are issued before the first MFMA
#pragma unroll
      for (int nt = 0; nt < Cfg::DTK; ++nt) dk[nt] = mma16(grow[nt], vf, dk[nt]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // G^T k^T contracts over d_key (fragments down the rows of Gl)
#pragma unroll
    for (int ks = 0; ks < Cfg::KSK; ++ks) {
      const frag8 kf = lds_row_frag(Ks + (16 * w + r) * TPK + 32 * ks + 8 * q4);
      frag8 gcol[Cfg::DTV];
#pragma unroll
      for (int nt = 0; nt < Cfg::DTV; ++nt)
        gcol[nt] = lds_col_frag(Gl, SP, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, 16 * nt, r);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int nt = 0; nt < Cfg::DTV; ++nt) dv[nt] = mma16(gcol[nt], kf, dv[nt]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // every tile row is private to its wave here: chain rule on the raw rows, then the
    // results are staged in place (K rows for dK, V rows for dV)
    const float rj = rk[16 * w + r];
    project_out_row<DK, TPK, false>(dk, Ks + 16 * w * TPK, rj, inv_eps, r, q4);
    wave_lds_sync();  // own rows of Ks, Vs were read before the staging writes
    gather_rows_transposed<DK>(dk, scale * rj, Ks + 16 * w * TPK, l, done_k);
    gather_rows_transposed<DV>(dv, scale * rj, Vs + 16 * w * TPV, l, done_v);
    __syncthreads();
  }
  if (row_begin < row_end) {
    const int last = row_begin + (row_end - row_begin - 1) / C * C;
    store_row_pieces<DK>(done_k, dKu, last + 16 * w, row_end, l);
    store_row_pieces<DV>(done_v, dVu, last + 16 * w, row_end, l);
  }
  if (seq_len != nullptr) {  // rows that do not exist
    zero_rows_e16<DK>(dKu, row_end, seg_end);
    zero_rows_e16<DV>(dVu, row_end, seg_end);
  }
}

SegmentTotalsArgs totals_args(const CausalArgs& a, const void* X, const void* Y, float* dst) {
  SegmentTotalsArgs t{};
  t.X = X; t.Y = Y; t.dst = dst;
  t.units = a.B * a.H; t.N = a.N; t.dk = a.dk; t.dv = a.dv; t.G = a.G; t.n_compute = a.G;
  t.seg_rows = a.seg_rows; t.eps = a.eps; t.stream = a.stream;
  t.seq_len = a.seq_len; t.H = a.H;
  return t;
}

template <int DK, int DV>
hipError_t run_fwd_bidir(const CausalArgs& a) {
  constexpr int C = 64;
  using Cfg = BiCfg<DK, DV, C>;
  const int units = a.B * a.H;
  float* totals = static_cast<float*>(a.workspace);
  hipError_t err = COTTN_SYM(launch_segment_totals)(totals_args(a, a.K, a.V, totals));
  if (err != hipSuccess) return err;
  // few segments: the apply workgroups add the totals up themselves (and write `state`)
  const bool sum_in_apply = a.G <= kMaxSegmentsSummedInScan;
  if (!sum_in_apply) {
    err = launch_bidir_combine(totals, 0, 1, units, a.G, DK * DV, a.state, nullptr, a.stream);
    if (err != hipSuccess) return err;
  }
  return launch_kernel(COTTN_SYM_STR(fwd_bidir_apply), COTTN_SYM(fwd_bidir_apply)<DK, DV, C>, dim3(units * a.G),
                       dim3(Cfg::NT), 0, a.stream, static_cast<const e16_t*>(a.Q), a.s,
                       static_cast<e16_t*>(a.O), totals, a.G, sum_in_apply ? a.G : 1,
                       sum_in_apply ? a.state : nullptr, a.H, a.N, a.G, a.seg_rows, 1.0f / a.eps,
                       a.seq_len, a.s_per_unit);
}

template <int DK, int DV>
hipError_t run_bwd_bidir(const CausalArgs& a) {
  constexpr int C = 64;
  using Cfg = BiCfg<DK, DV, C>;
  const int units = a.B * a.H;
  char* ws = static_cast<char*>(a.workspace);
  float* s_totals = reinterpret_cast<float*>(ws);
  const size_t pair_stride = state_array_bytes(a.B, a.H, DK, DV, a.G) / sizeof(float);
  float* g_totals = s_totals + pair_stride;
  float* ds_partial = reinterpret_cast<float*>(ws + 2 * state_array_bytes(a.B, a.H, DK, DV, a.G));
  // few segments: the sweeps add the segment totals up themselves while staging them; many:
  // the combine kernel leaves the sum in slot 0
  const bool few = a.G <= kMaxSegmentsSummedInScan;
  hipError_t err;
  // S = Kh^T V: the totals the forward left behind (slot 0 is their sum already when the
  // forward ran the combine kernel), or reduced here
  const float* s_src = a.saved_fwd_states;
  if (s_src == nullptr) {
    err = COTTN_SYM(launch_segment_totals)(totals_args(a, a.K, a.V, s_totals));
    if (err != hipSuccess) return err;
    if (!few) {
      err = launch_bidir_combine(s_totals, 0, 1, units, a.G, DK * DV, nullptr, nullptr, a.stream);
      if (err != hipSuccess) return err;
    }
    s_src = s_totals;
  }
  err = launch_kernel(COTTN_SYM_STR(bwd_bidir_dq), COTTN_SYM(bwd_bidir_dq)<DK, DV, C>, dim3(units * a.G),
                      dim3(Cfg::NT), 0, a.stream, static_cast<const e16_t*>(a.Q),
                      static_cast<const e16_t*>(a.dO), a.s, static_cast<e16_t*>(a.dQ), s_src, a.G,
                      few ? a.G : 1, g_totals, ds_partial, a.H, a.N, a.G, a.seg_rows, 1.0f / a.eps,
                      a.seq_len, a.s_per_unit);
  if (err != hipSuccess) return err;
  if (!few) {
    err = launch_bidir_combine(g_totals, 0, 1, units, a.G, DK * DV, nullptr, nullptr, a.stream);
    if (err != hipSuccess) return err;
  }
  return launch_kernel(COTTN_SYM_STR(bwd_bidir_dkdv), COTTN_SYM(bwd_bidir_dkdv)<DK, DV, C>, dim3(units * a.G),
                       dim3(Cfg::NT), 0, a.stream, static_cast<const e16_t*>(a.K),
                       static_cast<const e16_t*>(a.V), a.s, static_cast<e16_t*>(a.dK),
                       static_cast<e16_t*>(a.dV), g_totals, a.G, few ? a.G : 1, ds_partial, a.G, a.ds,
                       a.B, a.H, a.N, a.G, a.seg_rows, 1.0f / a.eps, a.seq_len, a.s_per_unit);
}

}  // namespace

#ifndef COTTN_ELEM_F16  // not specific to the element type: defined once, by the bf16 build
hipError_t launch_bidir_combine(float* totals, size_t pair_stride, int n_pairs, int units, int G,
                                int elems, float* state, float* ds_partial, hipStream_t st) {
  return launch_kernel("bidir_combine", bidir_combine, dim3(unsigned(elems / 256) * units), dim3(256), 0, st,
                       totals, pair_stride, n_pairs, G, elems, state, ds_partial);
}
#endif

#define COTTN_FOR_EACH_DK_DV(CALL)                                                              \
  switch (a.dk * 1000 + a.dv) {                                                                 \
    case 32032: return CALL<32, 32>(a);                                                         \
    case 32064: return CALL<32, 64>(a);                                                         \
    case 32128: return CALL<32, 128>(a);                                                        \
    case 64032: return CALL<64, 32>(a);                                                         \
    case 64064: return CALL<64, 64>(a);                                                         \
    case 64128: return CALL<64, 128>(a);                                                        \
    case 128032: return CALL<128, 32>(a);                                                       \
    case 128064: return CALL<128, 64>(a);                                                       \
    case 128128: return CALL<128, 128>(a);                                                      \
    default: return hipErrorInvalidValue;                                                       \
  }

hipError_t COTTN_SYM(fwd_bidir)(const CausalArgs& a) { COTTN_FOR_EACH_DK_DV(run_fwd_bidir) }

hipError_t COTTN_SYM(bwd_bidir)(const CausalArgs& a) { COTTN_FOR_EACH_DK_DV(run_bwd_bidir) }

}  // namespace cottn
