// Causal cosine attention backward, 16-bit storage / 16-bit MFMA / fp32 accumulation (gfx950).
// Written for a 16-bit element type: this file builds the bfloat16 kernels, and the IEEE half
// ones when it is included with COTTN_ELEM_F16 defined.
//
// Sec. 4 gives, for the normalised operands Qh, Kh (A = dO V^T, P = Qh Kh^T, M the
// lower-triangular mask),
//     dQh = (A (.) M) Kh,    dKh = (A (.) M)^T Qh,    dV = (P (.) M)^T dO,
// and notes that dQh is a cumulative sum running forward in time while dKh and dV use one
// running backward.  With S_t = sum_{j<=t} kh_j^T v_j and R_t = sum_{i>=t} qh_i^T dO_i:
//     dqh_t = s dO_t S_t^T,    dkh_t = s v_t R_t^T,    dv_t = s kh_t R_t.
// Both sums are regrouped exactly into chunks of C rows inside G segments per (batch, head):
//   forward-time states   per-segment totals of Kh^T V (d_key x d_value, stored tile by tile
//             like all states that only these kernels exchange): taken over from the
//             forward call when it hands its workspace on, else rebuilt by the forward's
//             totals kernel; with many segments a carry kernel turns totals into prefixes
//             (and the reverse-time totals into suffixes), with few the scans add them up;
//   dQ scan   forward-time: dQ of a segment, chunk by chunk, first to last; it has Q and dO
//             in LDS anyway and leaves the segment's reverse-time total Qh^T dO behind;
//   dK/dV scan  reverse-time: dK and dV of a segment, chunk by chunk, last to first (so it
//             starts on the rows the dQ scan read last, which are still in the XCD's L2);
//             its first workgroups also add up ds from the dQ scan's partial sums
//             (a separate small kernel does that for the fp32 path).
//
// Normalisation factors r_i = 1/max(|q_i|, eps), r_j = 1/max(|k_j|, eps) are not applied to
// Q and K element-wise where a row factor does the same:
//   dQ pass    K is contracted over the token index everywhere and is stored as kh = r_j k_j;
//              V stays raw; Q is only needed normalised (for the chain rule below and for
//              the reverse-time total) and is stored as qh;
//              dqh_i = sum_j A_ij kh_j + dO_i S^T,  S = sum kh_j^T v_j;
//   dK/dV pass Q is rescaled to r_i q_i (it is contracted over the token index in the
//              reverse state R = sum (r_i q_i)^T dO_i); K and V stay raw;
//              dv_j = s r_j [ sum_i ((r_i q_i).k_j) dO_i + k_j R ],
//              dkh_j = sum_i A_ij (r_i q_i) + v_j R^T.
// The chain rule through x/max(||x||, eps), with t = x . dxh on the raw row:
//     dx = s r (dxh - x r^2 t) = s r (dxh - xh (xh . dxh))   (rows at or below eps: dx = s r dxh),
// and ds_h = sum over rows of qh_i . dqh_i before scaling by s.
//
// Inside a chunk the masked A and P tiles are produced directly in the register layout the
// next product needs as an operand, so they never pass through LDS; operands contracted
// over the token index are read from the row-major LDS tiles with the transposing LDS read,
// and the fragments read for the intra-chunk products are reused by the state updates.
// Results are accumulated transposed (a lane holds 4 consecutive columns of one result row),
// which makes every row factor a per-lane scalar and the staging writes 8 bytes wide.
// Scheduling follows the forward file: all LDS reads of a group of MFMAs are issued first,
// and the next chunk's tiles are prefetched into registers.
#include "device_common.h"
#include "launch.h"
#include "tile_io.h"
#include "workspace.h"

namespace cottn {
namespace {

// DK, DV: the head dimensions of the keys / queries and of the values / outputs (Sec. 2.1:
// d_H_key and d_H_value); Q, K, dQ, dK rows are DK wide, V, dO, dV rows DV wide, and both
// running states (Kh^T V forward in time, Qh^T dO backward in time) are DK x DV.
template <int DK, int DV, int C>
struct BwdCfg {
  static constexpr int NW = C / 16;
  static constexpr int NT = NW * 64;
  static constexpr int DTK = DK / 16, DTV = DV / 16;
  static constexpr int KSK = DK / 32, KSV = DV / 32;
  static constexpr int NP = C / 32;
  static constexpr int TPK = tile_pitch(DK, C), TPV = tile_pitch(DV, C);   // operand tiles
  static constexpr int SPK = lds_pitch(DK), SPV = lds_pitch(DV);   // state copies
  static constexpr int TILEK = C * TPK, TILEV = C * TPV;
  // the bf16 copy of the running state, [d_key][d_value] in both scans
  static constexpr int STATE = DK * SPV;
  static constexpr int LDS_BYTES = 2 * (2 * TILEK + 2 * TILEV + STATE) + 4 * C + 64;
  static constexpr int WG_PER_CU = (160 * 1024) / LDS_BYTES;
  // the dQ kernel adds a staging tile when that does not lower the workgroups per compute
  // unit, and must when the finished rows (DK wide) do not fit the rows of the dO tile
  static constexpr bool DQ_OWN_STAGE =
      lds_pitch(DK) > TPV ||
      (LDS_BYTES + 2 * TILEK <= 160 * 1024 && (160 * 1024) / (LDS_BYTES + 2 * TILEK) == WG_PER_CU);
  static constexpr int WAVES_RAW = (WG_PER_CU >= 2 ? 2 : 1) * NW / 4;
  // never budget registers for more than two waves per SIMD unless one workgroup alone needs
  // it: spilling costs more than the second workgroup of a large chunk gains
  // (DK = 128 with DV = 64: the dQ scan's two states and its result need more than the 256
  // registers that two waves per SIMD leave each wave)
  static constexpr int WAVES_PER_EU =
      (DK == 128 && DV == 64) ? 1 : NW / 4 > 2 ? NW / 4 : (WAVES_RAW > 2 ? 2 : WAVES_RAW);
};

// pack a masked accumulator tile into half of an operand fragment
__device__ __forceinline__ void put_half(frag8& frag, int half, f32x4 acc, bool k0, bool k1,
                                         bool k2, bool k3) {
  u32x4 words = __builtin_bit_cast(u32x4, frag);
  words[2 * half + 0] = pack2(k0 ? acc[0] : 0.f, k1 ? acc[1] : 0.f);
  words[2 * half + 1] = pack2(k2 ? acc[2] : 0.f, k3 ? acc[3] : 0.f);
  frag = __builtin_bit_cast(frag8, words);
}

// ---------------------------------------------------------------------------------------
// Kernel 2: blockIdx.y == 0: slot g <- sum of fwd totals of segments < g;
//           blockIdx.y == 1: slot g <- sum of rev totals of segments > g.
// Totals that were never computed (fwd slot G-1, rev slot 0) are not read; a null array is
// skipped.
__global__ __launch_bounds__(256) void bwd_state_carry(float* __restrict__ fwd_tot,
                                                       float* __restrict__ rev_tot, int G,
                                                       int elems_per_state, long total) {
  const long idx = (long(blockIdx.x) * 256 + threadIdx.x) * 4;  // 4 elements per thread
  float* tot = blockIdx.y == 0 ? fwd_tot : rev_tot;
  if (idx >= total || tot == nullptr) return;
  const long unit = idx / elems_per_state, e = idx % elems_per_state;
  exclusive_running_sum(tot + unit * G * elems_per_state + e, G, size_t(elems_per_state),
                        blockIdx.y == 1);
}

// ---------------------------------------------------------------------------------------
// Kernel 3: dQ of one segment, chunks in forward order.  Wave w owns query rows 16w..16w+15.
// The running state S ([d_key][d_value]) sits in accumulators with the keys along the lanes:
// element [v] of lane (r, q4) of tile (key tile y, value tile x) is
// S[16 rt + r][16 ct + 4 q4 + v], the orientation the forward scan and the totals kernel use
// (so the stored states are read tile by tile, one 1 KB instruction per tile).  A lane holds 4
// consecutive values of one key row and publishes them with one 8-byte write to the row-major
// LDS copy St[d_key][d_value]; the update's key-side operand is the K fragment already read
// for the intra-chunk product.
template <int DK, int DV, int C>
__global__ __launch_bounds__(C * 4, (BwdCfg<DK, DV, C>::WAVES_PER_EU)) void COTTN_SYM(bwd_dq_scan)(
    const e16_t* __restrict__ Q, const e16_t* __restrict__ K, const e16_t* __restrict__ V,
    const e16_t* __restrict__ dO, const float* __restrict__ s, e16_t* __restrict__ dQ,
    const float* __restrict__ fwd_states, float* __restrict__ rev_totals,
    float* __restrict__ ds_partial, int H, int N, int G, int seg_rows, float inv_eps,
    int sum_totals, const int* __restrict__ seq_len, int s_per_unit,
    const float* __restrict__ state_in) {
  using Cfg = BwdCfg<DK, DV, C>;
  using AT = AccTiles<DK, DV, Cfg::NW>;   // forward-time state: key rows, value columns
  using RT = AccTiles<DV, DK, Cfg::NW>;   // reverse-time total: value rows, key columns
  using StageK = TileStage<DK, C, Cfg::NT>;
  using StageV = TileStage<DV, C, Cfg::NT>;
  constexpr int TPK = Cfg::TPK, TPV = Cfg::TPV, SP = Cfg::SPV;
  __shared__ __attribute__((aligned(16))) e16_t Qs[Cfg::TILEK];   // qh = r_i q_i
  __shared__ __attribute__((aligned(16))) e16_t Ks[Cfg::TILEK];   // kh = r_j k_j
  __shared__ __attribute__((aligned(16))) e16_t Vs[Cfg::TILEV];   // raw v
  __shared__ __attribute__((aligned(16))) e16_t Gs[Cfg::TILEV];   // dO
  __shared__ __attribute__((aligned(16))) e16_t St[DK * Cfg::SPV];  // state, [d_key][d_value]
  // Every wave reads all rows of all four tiles until the end of a chunk (the reverse total
  // contracts Qs and Gs over the tokens), so finished dQ rows are staged in a tile of their
  // own when LDS has room for one; otherwise behind a barrier in the dead dO tile.
  __shared__ __attribute__((aligned(16))) e16_t Os[Cfg::DQ_OWN_STAGE ? Cfg::TILEK : 8];
  __shared__ float rq[C];
  __shared__ float ds_wave[Cfg::NW];

  fetch_argument_now(Q, K, V, dO, s, dQ, fwd_states, rev_totals, ds_partial, H, N, G, seg_rows,
                     inv_eps, sum_totals, seq_len, s_per_unit, state_in);
  int unit, g;
  unit_and_segment(blockIdx.x, G, unit, g);
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const e16_t* Qu = Q + size_t(unit) * N * DK;
  const e16_t* Ku = K + size_t(unit) * N * DK;
  const e16_t* Vu = V + size_t(unit) * N * DV;
  const e16_t* Gu = dO + size_t(unit) * N * DV;
  e16_t* dQu = dQ + size_t(unit) * N * DK;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows;
  const int seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));

  // fwd_states holds the carried prefixes (slot g = state at the start of segment g) or, with
  // sum_totals set, the raw segment totals, which this workgroup then adds up itself
  f32x4 sacc[AT::NCT][AT::NRT];
  // By-product for the dK/dV kernel: this segment's total of qh^T dO (segments after the
  // first; earlier segments need it), accumulated in that kernel's layout: element [v] of
  // lane (r, q4) of tile (y, x) is R[key 16 ct + r][value 16 rt + 4 q4 + v].
  f32x4 racc[RT::NCT][RT::NRT];
  const bool with_rev = rev_totals != nullptr && g > 0;
#pragma unroll
  for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
    for (int y = 0; y < AT::NRT; ++y) sacc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int x = 0; x < RT::NCT; ++x)
#pragma unroll
    for (int y = 0; y < RT::NRT; ++y) racc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};
  // the first chunk's rows and the stored states are all requested before anything waits
  float ds_lane = 0.f;
  StageK qst, kst;
  StageV vst, gst;
  qst.fetch(Qu, row_begin, row_end);
  kst.fetch(Ku, row_begin, row_end);
  vst.fetch(Vu, row_begin, row_end);
  gst.fetch(Gu, row_begin, row_end);
  if (fwd_states != nullptr && g > 0 && AT::active(w)) {
    const float* src = fwd_states + size_t(unit) * G * DK * DV;
    add_stored_states<AT::STATE_BATCH>(
        sacc, sum_totals ? 0 : g, sum_totals ? g - 1 : g, [&](int gp, int x, int y) {
          return *reinterpret_cast<const f32x4*>(
              src + size_t(gp) * DK * DV +
              tiled_state_offset(AT::row_tile(w, y), AT::col_tile(w, x), DV / 16, l));
        });
  }
  // the state of the rows before this piece of the sequence belongs to every segment's start
  if (state_in != nullptr && AT::active(w)) {
    const float* src = state_in + size_t(unit) * DK * DV;
#pragma unroll
    for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
      for (int y = 0; y < AT::NRT; ++y)
        sacc[x][y] += *reinterpret_cast<const f32x4*>(src + (16 * AT::row_tile(w, y) + r) * DV +
                                                      16 * AT::col_tile(w, x) + 4 * q4);
  }

  RowPieces<DK> finished;  // dQ rows of the previous chunk, stored one chunk late
#pragma unroll
  for (int j = 0; j < RowPieces<DK>::PER_LANE; ++j) finished.v[j] = uint4{0u, 0u, 0u, 0u};
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    if (AT::active(w)) {
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y) {
          uint2 pk;
          pk.x = pack2(sacc[x][y][0], sacc[x][y][1]);
          pk.y = pack2(sacc[x][y][2], sacc[x][y][3]);
          *reinterpret_cast<uint2*>(St + (16 * AT::row_tile(w, y) + r) * SP +
                                    16 * AT::col_tile(w, x) + 4 * q4) = pk;
        }
    }
    {
      float rqv[StageK::PASSES], rkv[StageK::PASSES];
      qst.row_rinv(inv_eps, rqv);
      kst.row_rinv(inv_eps, rkv);
      qst.commit_scaled(Qs, rqv);
      qst.store_rinv(rq, rqv);
      kst.commit_scaled(Ks, rkv);
      vst.commit_plain(Vs);
      gst.commit_plain(Gs);
    }
    if (row0 + C < row_end) {
      qst.fetch(Qu, row0 + C, row_end);
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
      gst.fetch(Gu, row0 + C, row_end);
    }
    if (row0 > row_begin) store_row_pieces<DK>(finished, dQu, row0 - C + 16 * w, row_end, l);
    __syncthreads();

    // earlier chunks: dqh^T += S dO^T (contraction over d_value = along the rows of St)
    frag8 gf[Cfg::KSV];  // dO rows of this wave: column-side operand of every product
#pragma unroll
    for (int ks = 0; ks < Cfg::KSV; ++ks)
      gf[ks] = lds_row_frag(Gs + (16 * w + r) * TPV + 32 * ks + 8 * q4);
    // dq[nt][v] = dqh[query 16w + r][key feature 16 nt + 4 q4 + v]
    f32x4 dq[Cfg::DTK];
#pragma unroll
    for (int nt = 0; nt < Cfg::DTK; ++nt) dq[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < Cfg::KSV; ++ks) {
      frag8 sf[Cfg::DTK];
#pragma unroll
      for (int nt = 0; nt < Cfg::DTK; ++nt)
        sf[nt] = lds_row_frag(St + (16 * nt + r) * SP + 32 * ks + 8 * q4);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int nt = 0; nt < Cfg::DTK; ++nt) dq[nt] = mma16(sf[nt], gf[ks], dq[nt]);
      __builtin_amdgcn_sched_barrier(0);
    }

    // this chunk: dqh^T += Kh^T (A (.) M)^T with A^T = V dO^T, and the state update,
    // 32 tokens at a time
#pragma unroll
    for (int p = 0; p < Cfg::NP; ++p) {
      const bool diag_or_below = 2 * p <= w;
      const int t0 = 32 * p + 4 * q4, t1 = 32 * p + 16 + 4 * q4;  // token order of the A slots
      frag8 kc[Cfg::DTK], vcol[AT::NCT], krow[AT::NRT], vr[2][Cfg::KSV];
      frag8 qcol[RT::NCT], grow[RT::NRT];
#pragma unroll
      for (int nt = 0; nt < Cfg::DTK; ++nt) kc[nt] = lds_col_frag(Ks, TPK, t0, t1, 16 * nt, r);
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
        vcol[x] = lds_col_frag(Vs, TPV, t0, t1, 16 * AT::col_tile(w, x), r);
      if (AT::WPC != 1) {
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
          krow[y] = lds_col_frag(Ks, TPK, t0, t1, 16 * AT::row_tile(w, y), r);
      }
      if (with_rev && RT::active(w)) {
#pragma unroll
        for (int x = 0; x < RT::NCT; ++x)
          qcol[x] = lds_col_frag(Qs, TPK, t0, t1, 16 * RT::col_tile(w, x), r);
#pragma unroll
        for (int y = 0; y < RT::NRT; ++y)
          grow[y] = lds_col_frag(Gs, TPV, t0, t1, 16 * RT::row_tile(w, y), r);
      }
      if (diag_or_below) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
          for (int ks = 0; ks < Cfg::KSV; ++ks)
            vr[half][ks] = lds_row_frag(Vs + (16 * (2 * p + half) + r) * TPV + 32 * ks + 8 * q4);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (diag_or_below) {
        frag8 af;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int jt = 2 * p + half;
          f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < Cfg::KSV; ++ks) t = mma16(vr[half][ks], gf[ks], t);
          // t[v] = dO_(16w + r) . v_(16jt + 4 q4 + v); keep key <= query
          const bool full = jt < w, diag = jt == w;
          put_half(af, half, t, full || (diag && 4 * q4 + 0 <= r), full || (diag && 4 * q4 + 1 <= r),
                   full || (diag && 4 * q4 + 2 <= r), full || (diag && 4 * q4 + 3 <= r));
        }
#pragma unroll
        for (int nt = 0; nt < Cfg::DTK; ++nt) dq[nt] = mma16(kc[nt], af, dq[nt]);
      }
      // state update: S += kh^T v over these 32 tokens
      if (AT::active(w)) {
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
#pragma unroll
          for (int x = 0; x < AT::NCT; ++x)
            sacc[x][y] = mma16(vcol[x], AT::WPC == 1 ? kc[y] : krow[y], sacc[x][y]);
      }
      // reverse total: R^T += dO^T qh over the same tokens
      if (with_rev && RT::active(w)) {
#pragma unroll
        for (int y = 0; y < RT::NRT; ++y)
#pragma unroll
          for (int x = 0; x < RT::NCT; ++x) racc[x][y] = mma16(grow[y], qcol[x], racc[x][y]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // epilogue: normalisation chain rule on the rows (Qs holds qh), then s r_i and the store
    const float ri = rq[16 * w + r];
    const float rho = project_out_row<DK, TPK, true>(dq, Qs + 16 * w * TPK, ri, inv_eps, r, q4);
    if (q4 == 0) ds_lane += rho;
    if (Cfg::DQ_OWN_STAGE) {
      gather_rows_transposed<DK>(dq, scale * ri, Os + 16 * w * TPK, l, finished);
    } else {
      __syncthreads();  // every wave is done with the dO tile
      gather_rows_transposed<DK>(dq, scale * ri, Gs + 16 * w * TPV, l, finished);
    }
    __syncthreads();
  }
  if (row_begin < row_end) {
    const int last = row_begin + (row_end - row_begin - 1) / C * C;
    store_row_pieces<DK>(finished, dQu, last + 16 * w, row_end, l);
  }

  if (seq_len != nullptr) zero_rows_e16<DK>(dQu, row_end, seg_end);  // rows that do not exist

  if (with_rev && RT::active(w)) {
    float* out = rev_totals + (size_t(unit) * G + g) * DK * DV;
#pragma unroll
    for (int x = 0; x < RT::NCT; ++x)
#pragma unroll
      for (int y = 0; y < RT::NRT; ++y)
        store_state_words(out + tiled_state_offset(RT::col_tile(w, x), RT::row_tile(w, y), DV / 16, l),
                          racc[x][y]);
  }

  // per-workgroup partial of ds: lanes of the first lane row hold the row sums
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
template <int DK, int DV, int C>
__global__ __launch_bounds__(C * 4, (BwdCfg<DK, DV, C>::WAVES_PER_EU)) void COTTN_SYM(bwd_dkdv_scan)(
    const e16_t* __restrict__ Q, const e16_t* __restrict__ K, const e16_t* __restrict__ V,
    const e16_t* __restrict__ dO, const float* __restrict__ s, e16_t* __restrict__ dK,
    e16_t* __restrict__ dV, const float* __restrict__ rev_states,
    const float* __restrict__ ds_partial, float* __restrict__ ds, int B, int H, int N, int G,
    int seg_rows, float inv_eps, int sum_totals, const int* __restrict__ seq_len, int s_per_unit,
    const float* __restrict__ rev_in, float* __restrict__ rev_out) {
  using Cfg = BwdCfg<DK, DV, C>;
  using AT = AccTiles<DV, DK, Cfg::NW>;   // value rows, key columns (the state is held transposed)
  using StageK = TileStage<DK, C, Cfg::NT>;
  using StageV = TileStage<DV, C, Cfg::NT>;
  constexpr int TPK = Cfg::TPK, TPV = Cfg::TPV, SP = Cfg::SPV;
  __shared__ __attribute__((aligned(16))) e16_t Qs[Cfg::TILEK];   // r_i q_i
  __shared__ __attribute__((aligned(16))) e16_t Ks[Cfg::TILEK];   // raw k
  __shared__ __attribute__((aligned(16))) e16_t Vs[Cfg::TILEV];   // raw v
  __shared__ __attribute__((aligned(16))) e16_t Gs[Cfg::TILEV];   // dO
  __shared__ __attribute__((aligned(16))) e16_t Rl[DK * Cfg::SPV];  // reverse state, [d_key][d_value]
  __shared__ float rk[C];

  fetch_argument_now(Q, K, V, dO, s, dK, dV, rev_states, ds_partial, ds, B, H, N, G, seg_rows,
                     inv_eps, sum_totals, seq_len, s_per_unit, rev_in, rev_out);
  int unit, g;
  unit_and_segment(blockIdx.x, G, unit, g);
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const e16_t* Qu = Q + size_t(unit) * N * DK;
  const e16_t* Ku = K + size_t(unit) * N * DK;
  const e16_t* Vu = V + size_t(unit) * N * DV;
  const e16_t* Gu = dO + size_t(unit) * N * DV;
  e16_t* dKu = dK + size_t(unit) * N * DK;
  e16_t* dVu = dV + size_t(unit) * N * DV;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows;
  const int seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));
  const int n_chunks = (row_end - row_begin + C - 1) / C;

  // the first H workgroups also finish ds: ds[h] = sum over batches and segments of the
  // partial sums the dQ kernel left behind (with a scale per (batch, head): the first B*H
  // workgroups, ds[b][h] = sum over the segments)
  if (int(blockIdx.x) < (s_per_unit ? B * H : H) && w == 0) {
    float t = 0.f;
    const int n = s_per_unit ? G : B * G;
    for (int i = l; i < n; i += 64)
      t += s_per_unit ? ds_partial[size_t(blockIdx.x) * G + i]
                      : ds_partial[(size_t(i / G) * H + blockIdx.x) * G + (i % G)];
    t = group_sum<64>(t);
    if (l == 0) ds[blockIdx.x] = t;
  }

  // rev_states holds the carried suffixes (slot g = reverse state at the end of segment g)
  // or, with sum_totals set, the raw segment totals of the later segments to be added up here
  f32x4 racc[AT::NCT][AT::NRT];
#pragma unroll
  for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
    for (int y = 0; y < AT::NRT; ++y) racc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};
  // the last chunk's rows and the stored states are all requested before anything waits
  StageK qst, kst;
  StageV vst, gst;
  if (n_chunks > 0) {  // (a segment of a padded batch can be empty)
    const int first = row_begin + (n_chunks - 1) * C;
    qst.fetch(Qu, first, row_end);
    kst.fetch(Ku, first, row_end);
    vst.fetch(Vu, first, row_end);
    gst.fetch(Gu, first, row_end);
  }
  if (rev_states != nullptr && g < G - 1 && AT::active(w)) {
    const float* src = rev_states + size_t(unit) * G * DK * DV;
    add_stored_states<AT::STATE_BATCH>(
        racc, sum_totals ? g + 1 : g, sum_totals ? G - 1 : g, [&](int gp, int x, int y) {
          return *reinterpret_cast<const f32x4*>(
              src + size_t(gp) * DK * DV +
              tiled_state_offset(AT::col_tile(w, x), AT::row_tile(w, y), DV / 16, l));
        });
  }
  // the reverse state of the rows after this piece of the sequence belongs to every segment
  if (rev_in != nullptr && AT::active(w)) {
    const float* src = rev_in + size_t(unit) * DK * DV;
#pragma unroll
    for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
      for (int y = 0; y < AT::NRT; ++y)
        racc[x][y] += *reinterpret_cast<const f32x4*>(src + (16 * AT::col_tile(w, x) + r) * DV +
                                                      16 * AT::row_tile(w, y) + 4 * q4);
  }

  RowPieces<DK> done_k;  // dK and dV rows of the previous chunk, stored one chunk late
  RowPieces<DV> done_v;
#pragma unroll
  for (int j = 0; j < RowPieces<DK>::PER_LANE; ++j) done_k.v[j] = uint4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < RowPieces<DV>::PER_LANE; ++j) done_v.v[j] = uint4{0u, 0u, 0u, 0u};
  for (int c = n_chunks - 1; c >= 0; --c) {
    const int row0 = row_begin + c * C;
    if (AT::active(w)) {
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y) {
          uint2 pk;
          pk.x = pack2(racc[x][y][0], racc[x][y][1]);
          pk.y = pack2(racc[x][y][2], racc[x][y][3]);
          *reinterpret_cast<uint2*>(Rl + (16 * AT::col_tile(w, x) + r) * SP +
                                    16 * AT::row_tile(w, y) + 4 * q4) = pk;
        }
    }
    {
      float rqv[StageK::PASSES], rkv[StageK::PASSES];
      qst.row_rinv(inv_eps, rqv);
      kst.row_rinv(inv_eps, rkv);
      qst.commit_scaled(Qs, rqv);
      kst.commit_plain(Ks);
      kst.store_rinv(rk, rkv);
      vst.commit_plain(Vs);
      gst.commit_plain(Gs);
    }
    if (c > 0) {
      qst.fetch(Qu, row0 - C, row_end);
      kst.fetch(Ku, row0 - C, row_end);
      vst.fetch(Vu, row0 - C, row_end);
      gst.fetch(Gu, row0 - C, row_end);
    }
    if (c < n_chunks - 1) {
      store_row_pieces<DK>(done_k, dKu, row0 + C + 16 * w, row_end, l);
      store_row_pieces<DV>(done_v, dVu, row0 + C + 16 * w, row_end, l);
    }
    __syncthreads();

    frag8 kf[Cfg::KSK], vf[Cfg::KSV];  // this wave's key rows and value rows (column side)
#pragma unroll
    for (int ks = 0; ks < Cfg::KSK; ++ks)
      kf[ks] = lds_row_frag(Ks + (16 * w + r) * TPK + 32 * ks + 8 * q4);
#pragma unroll
    for (int ks = 0; ks < Cfg::KSV; ++ks)
      vf[ks] = lds_row_frag(Vs + (16 * w + r) * TPV + 32 * ks + 8 * q4);
    // dk[nt][v] = dkh[key 16w + r][feature 16 nt + 4 q4 + v]; dv likewise before s r_j
    f32x4 dk[Cfg::DTK], dv[Cfg::DTV];
#pragma unroll
    for (int nt = 0; nt < Cfg::DTK; ++nt) dk[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int nt = 0; nt < Cfg::DTV; ++nt) dv[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // later chunks: dv^T += R^T k^T (over d_key), dkh^T += R v^T (over d_value)
    constexpr int KS_BOTH = Cfg::KSK < Cfg::KSV ? Cfg::KSK : Cfg::KSV;
#pragma unroll
    for (int ks = 0; ks < (Cfg::KSK > Cfg::KSV ? Cfg::KSK : Cfg::KSV); ++ks) {
      frag8 rcol[Cfg::DTV], rrow[Cfg::DTK];
      if (ks < Cfg::KSK) {
#pragma unroll
        for (int nt = 0; nt < Cfg::DTV; ++nt)
          rcol[nt] = lds_col_frag(Rl, SP, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, 16 * nt, r);
      }
      if (ks < Cfg::KSV) {
#pragma unroll
        for (int nt = 0; nt < Cfg::DTK; ++nt)
          rrow[nt] = lds_row_frag(Rl + (16 * nt + r) * SP + 32 * ks + 8 * q4);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (ks < KS_BOTH && Cfg::DTK == Cfg::DTV) {
#pragma unroll
        for (int nt = 0; nt < Cfg::DTK; ++nt) {
          dv[nt] = mma16(rcol[nt], kf[ks], dv[nt]);
          dk[nt] = mma16(rrow[nt], vf[ks], dk[nt]);
        }
      } else {
        if (ks < Cfg::KSK) {
#pragma unroll
          for (int nt = 0; nt < Cfg::DTV; ++nt) dv[nt] = mma16(rcol[nt], kf[ks], dv[nt]);
        }
        if (ks < Cfg::KSV) {
#pragma unroll
          for (int nt = 0; nt < Cfg::DTK; ++nt) dk[nt] = mma16(rrow[nt], vf[ks], dk[nt]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // this chunk: query tiles it >= w two at a time, and the reverse state update
#pragma unroll
    for (int p = 0; p < Cfg::NP; ++p) {
      const bool diag_or_above = 2 * p + 1 >= w;
      const int t0 = 32 * p + 4 * q4, t1 = 32 * p + 16 + 4 * q4;  // token order of the slots
      frag8 gc[Cfg::DTV], qcol[AT::NCT], grow[AT::NRT];
#pragma unroll
      for (int nt = 0; nt < Cfg::DTV; ++nt) gc[nt] = lds_col_frag(Gs, TPV, t0, t1, 16 * nt, r);
#pragma unroll
      for (int x = 0; x < AT::NCT; ++x)
        qcol[x] = lds_col_frag(Qs, TPK, t0, t1, 16 * AT::col_tile(w, x), r);
      if (AT::WPC != 1) {
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
          grow[y] = lds_col_frag(Gs, TPV, t0, t1, 16 * AT::row_tile(w, y), r);
      }
      __builtin_amdgcn_sched_barrier(0);
      // reverse state update: R^T += dO^T (r q) over these 32 tokens
      if (AT::active(w)) {
#pragma unroll
        for (int y = 0; y < AT::NRT; ++y)
#pragma unroll
          for (int x = 0; x < AT::NCT; ++x)
            racc[x][y] = mma16(AT::WPC == 1 ? gc[y] : grow[y], qcol[x], racc[x][y]);
      }
      if (diag_or_above) {
        frag8 qr[2][Cfg::KSK], gr[2][Cfg::KSV], qc[Cfg::DTK];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
          for (int ks = 0; ks < Cfg::KSK; ++ks)
            qr[half][ks] = lds_row_frag(Qs + (16 * (2 * p + half) + r) * TPK + 32 * ks + 8 * q4);
#pragma unroll
          for (int ks = 0; ks < Cfg::KSV; ++ks)
            gr[half][ks] = lds_row_frag(Gs + (16 * (2 * p + half) + r) * TPV + 32 * ks + 8 * q4);
        }
#pragma unroll
        for (int nt = 0; nt < Cfg::DTK; ++nt) qc[nt] = lds_col_frag(Qs, TPK, t0, t1, 16 * nt, r);
        __builtin_amdgcn_sched_barrier(0);
        frag8 pf, af;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int it = 2 * p + half;
          f32x4 tp = {0.f, 0.f, 0.f, 0.f}, ta = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < Cfg::KSK; ++ks) tp = mma16(qr[half][ks], kf[ks], tp);
#pragma unroll
          for (int ks = 0; ks < Cfg::KSV; ++ks) ta = mma16(gr[half][ks], vf[ks], ta);
          // t*[v]: query 16 it + 4 q4 + v, key 16 w + r; keep key <= query
          const bool full = it > w, diag = it == w;
          const bool k0 = full || (diag && r <= 4 * q4 + 0), k1 = full || (diag && r <= 4 * q4 + 1),
                     k2 = full || (diag && r <= 4 * q4 + 2), k3 = full || (diag && r <= 4 * q4 + 3);
          put_half(pf, half, tp, k0, k1, k2, k3);
          put_half(af, half, ta, k0, k1, k2, k3);
        }
#pragma unroll
        for (int nt = 0; nt < Cfg::DTV; ++nt) dv[nt] = mma16(gc[nt], pf, dv[nt]);
#pragma unroll
        for (int nt = 0; nt < Cfg::DTK; ++nt) dk[nt] = mma16(qc[nt], af, dk[nt]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // epilogue: dv_j = s r_j dv; dk_j through the normalisation chain rule; both staged in
    // this wave's own (dead) rows of Vs and Ks
    const float rj = rk[16 * w + r];
    project_out_row<DK, TPK, false>(dk, Ks + 16 * w * TPK, rj, inv_eps, r, q4);
    wave_lds_sync();  // own Ks / Vs rows (kf, vf, raw k) were read before the staging writes
    gather_rows_transposed<DK>(dk, scale * rj, Ks + 16 * w * TPK, l, done_k);
    gather_rows_transposed<DV>(dv, scale * rj, Vs + 16 * w * TPV, l, done_v);
    __syncthreads();
  }
  if (n_chunks > 0) {
    store_row_pieces<DK>(done_k, dKu, row_begin + 16 * w, row_end, l);
    store_row_pieces<DV>(done_v, dVu, row_begin + 16 * w, row_end, l);
  }
  if (seq_len != nullptr) {  // rows that do not exist
    zero_rows_e16<DK>(dKu, row_end, seg_end);
    zero_rows_e16<DV>(dVu, row_end, seg_end);
  }
  // the first segment ends with the reverse state of the whole piece and what followed it
  if (rev_out != nullptr && g == 0 && AT::active(w)) {
    float* out = rev_out + size_t(unit) * DK * DV;
#pragma unroll
    for (int x = 0; x < AT::NCT; ++x)
#pragma unroll
      for (int y = 0; y < AT::NRT; ++y)
        *reinterpret_cast<f32x4*>(out + (16 * AT::col_tile(w, x) + r) * DV +
                                  16 * AT::row_tile(w, y) + 4 * q4) = racc[x][y];
  }
}

// ---------------------------------------------------------------------------------------
// Kernel 5: ds[h] = sum over batches b and segments g of partial[(b H + h) G + g].
__global__ __launch_bounds__(256) void bwd_reduce_ds(const float* __restrict__ partial,
                                                     float* __restrict__ ds, int B, int H, int G,
                                                     int per_unit) {
  __shared__ float red[256];
  const int h = blockIdx.x;  // head, or (batch, head) with per_unit
  float acc = 0.f;
  const long n = per_unit ? G : long(B) * G;
  for (long i = threadIdx.x; i < n; i += 256) {
    const long b = i / G, g = i % G;
    acc += per_unit ? partial[long(h) * G + i] : partial[(b * H + h) * G + g];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int stride = 128; stride > 0; stride >>= 1) {
    if (int(threadIdx.x) < stride) red[threadIdx.x] += red[threadIdx.x + stride];
    __syncthreads();
  }
  if (threadIdx.x == 0) ds[h] = red[0];
}

template <int DK, int DV, int C>
hipError_t run_bwd_causal(const CausalArgs& a) {
  using Cfg = BwdCfg<DK, DV, C>;
  const int units = a.B * a.H;
  const e16_t* Q = static_cast<const e16_t*>(a.Q);
  const e16_t* K = static_cast<const e16_t*>(a.K);
  const e16_t* V = static_cast<const e16_t*>(a.V);
  const e16_t* dO = static_cast<const e16_t*>(a.dO);
  char* ws = static_cast<char*>(a.workspace);
  const float* fwd_states = nullptr;
  float* rev_states = nullptr;
  const dim3 grid(units * a.G), block(Cfg::NT);
  const float inv_eps = 1.0f / a.eps;
  // few segments: no carry launches, the scan workgroups add up the totals they need
  const bool sum_in_scan = a.G <= kMaxSegmentsSummedInScan;
  hipError_t err;
  if (a.G > 1) {
    // Forward-time states: taken over from the forward call when it left them behind (raw
    // totals or carried prefixes, by the same rule as here), else recomputed from K and V.
    float* own_fwd = reinterpret_cast<float*>(ws);
    rev_states = reinterpret_cast<float*>(ws + state_array_bytes(a.B, a.H, DK, DV, a.G));
    ws += 2 * state_array_bytes(a.B, a.H, DK, DV, a.G);
    if (a.saved_fwd_states != nullptr) {
      fwd_states = a.saved_fwd_states;
    } else {
      err = COTTN_SYM(launch_fwd_segment_totals)(a, own_fwd);
      if (err != hipSuccess) return err;
      if (!sum_in_scan) {
        err = launch_bwd_state_carry(own_fwd, nullptr, units, a.G, DK * DV, a.stream);
        if (err != hipSuccess) return err;
      }
      fwd_states = own_fwd;
    }
  }
  float* ds_partial = reinterpret_cast<float*>(ws);
  // the dQ scan leaves the reverse-time segment totals (of qh^T dO) behind for the dK/dV scan
  err = launch_kernel(COTTN_SYM_STR(bwd_dq_scan), COTTN_SYM(bwd_dq_scan)<DK, DV, C>, grid, block, 0, a.stream, Q, K, V,
                      dO, a.s, static_cast<e16_t*>(a.dQ), fwd_states, rev_states, ds_partial, a.H,
                      a.N, a.G, a.seg_rows, inv_eps, sum_in_scan ? 1 : 0, a.seq_len, a.s_per_unit,
                      a.state_in);
  if (err != hipSuccess) return err;
  if (a.G > 1 && !sum_in_scan) {
    err = launch_bwd_state_carry(nullptr, rev_states, units, a.G, DK * DV, a.stream);
    if (err != hipSuccess) return err;
  }
  // the dK/dV kernel also reduces the ds partial sums written by the dQ kernel
  return launch_kernel(COTTN_SYM_STR(bwd_dkdv_scan), COTTN_SYM(bwd_dkdv_scan)<DK, DV, C>, grid, block, 0, a.stream, Q,
                       K, V, dO, a.s, static_cast<e16_t*>(a.dK), static_cast<e16_t*>(a.dV),
                       rev_states, ds_partial, a.ds, a.B, a.H, a.N, a.G, a.seg_rows, inv_eps,
                       sum_in_scan ? 1 : 0, a.seq_len, a.s_per_unit, a.rev_state_in,
                       a.rev_state_out);
}

}  // namespace

#ifndef COTTN_ELEM_F16  // not specific to the element type: defined once, by the bf16 build
hipError_t launch_bwd_state_carry(float* fwd_tot, float* rev_tot, int units, int G, int elems,
                                  hipStream_t st) {
  const long total = long(units) * elems;
  return launch_kernel("bwd_state_carry", bwd_state_carry, dim3(unsigned((total / 4 + 255) / 256), 2),
                       dim3(256), 0, st, fwd_tot, rev_tot, G, elems, total);
}

hipError_t launch_reduce_ds(const float* partial, float* ds, int B, int H, int G, int per_unit,
                            hipStream_t st) {
  return launch_kernel("bwd_reduce_ds", bwd_reduce_ds, dim3(per_unit ? B * H : H), dim3(256), 0, st,
                       partial, ds, B, H, G, per_unit);
}
#endif

hipError_t COTTN_SYM(bwd_causal)(const CausalArgs& a) {
  // d_key != d_value: chunks of 64 rows
  switch ((a.dk * 1000 + a.dv) * 1000 + a.C) {
    case 32032064: return run_bwd_causal<32, 32, 64>(a);
    case 32032128: return run_bwd_causal<32, 32, 128>(a);
    case 32032256: return run_bwd_causal<32, 32, 256>(a);
    case 64064064: return run_bwd_causal<64, 64, 64>(a);
    case 64064128: return run_bwd_causal<64, 64, 128>(a);
    case 64064256: return run_bwd_causal<64, 64, 256>(a);
    case 128128064: return run_bwd_causal<128, 128, 64>(a);
    case 32064064: return run_bwd_causal<32, 64, 64>(a);
    case 32128064: return run_bwd_causal<32, 128, 64>(a);
    case 64032064: return run_bwd_causal<64, 32, 64>(a);
    case 64128064: return run_bwd_causal<64, 128, 64>(a);
    case 128032064: return run_bwd_causal<128, 32, 64>(a);
    case 128064064: return run_bwd_causal<128, 64, 64>(a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cottn
