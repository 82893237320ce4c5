// Causal cosine attention forward, 16-bit storage / 16-bit MFMA / fp32 accumulation (gfx950).
// Written for a 16-bit element type: this file builds the bfloat16 kernels, and the IEEE half
// ones when it is included with COTTN_ELEM_F16 defined.
//
// Sec. 4 eq. attn_2 writes the causal output as an inclusive cumulative sum over the sequence
// of the outer products kh_j^T v_j, contracted with qh_i.  Regrouping that sum exactly:
//   * the sequence of one (batch, head) is cut into G segments, each a whole number of chunks
//     of C rows;
//   * kernel 1 (segment totals) reduces kh^T v over every segment but the last;
//   * kernel 2 (carry, only with many segments; with few the scan adds the totals up itself)
//     turns the totals into exclusive prefixes: the state at each segment start;
//   * kernel 3 (scan) walks the chunks of its segment with the d x d state in fp32
//     accumulators:  O_c = s_h [ (Qh_c Kh_c^T (.) M) V_c + Qh_c S ],  S += Kh_c^T V_c,
//     where the first term is eq. attn_1 restricted to the chunk.
// With G = 1 only the scan kernel runs; with one chunk per segment this is the fully
// chunk-parallel form.
//
// Normalisation (Sec. 3.2): with r_i = 1/max(|q_i|,eps) and kh_j = k_j / max(|k_j|,eps),
//     O_i = s_h r_i [ sum_{j<=i} (q_i . kh_j) v_j + q_i S ],   S = sum_j kh_j^T v_j,
// so the raw Q rows are an MFMA operand and r_i multiplies the finished output row, while K,
// which is contracted over the token index in S, is rescaled to kh on its way into LDS.
//
// Work split inside the scan workgroup (C/16 waves): wave w owns query rows 16w..16w+15 of
// the chunk for the output, and a fixed set of 16x16 tiles of the state for the update.
// Tiles sit row-major in LDS; operands whose contraction index is the token are read with
// the transposing LDS read, so no transposed copy is kept.  The masked similarity tile is
// produced as P^T = K Q^T, whose accumulator layout is the operand layout the following
// product needs (with the token slots permuted the same way on the V side), so P never
// touches LDS; the V fragments read for P V are reused by the state update.  Outputs are
// accumulated transposed (O^T = V^T P^T + S^T Q^T) so that a lane ends up with 4 consecutive
// columns of one output row: one row factor per lane and 8-byte staging writes.
//
// Scheduling: the kernels wait for memory and for their own latencies, not for the MFMA
// units, so every group of MFMAs is preceded by all of its LDS reads, issued back to back into
// distinct registers (a scheduling barrier keeps the compiler from sinking a read next to its
// use), the next chunk's tiles are prefetched into registers while the current one is
// computed, and finished output rows are stored one chunk late, non-temporally.  An XCD's L2
// keeps its contents between launches and workgroups are dealt to the XCDs by index, so the
// totals kernel and the scan number their workgroups alike: the scan finds its K, V rows in L2.
#include "device_common.h"
#include "launch.h"
#include "tile_io.h"

namespace cottn {
namespace {

// DK, DV: the head dimensions of the keys / queries and of the values / outputs (Sec. 2.1:
// d_H_key and d_H_value); the state Kh^T V is DK x DV.
template <int DK, int DV, int C>
struct FwdCfg {
  static constexpr int NW = C / 16;
  static constexpr int NT = NW * 64;
  static constexpr int DTK = DK / 16, DTV = DV / 16;
  static constexpr int KSK = DK / 32;   // k steps of a contraction over the key features
  static constexpr int NP = C / 32;     // pairs of 16-token tiles in a chunk
  static constexpr int TPK = tile_pitch(DK, C), TPV = tile_pitch(DV, C);   // operand tiles
  static constexpr int SP = lds_pitch(DV);   // state copy [d_key][d_value]
  static constexpr int TILEK = C * TPK, TILEV = C * TPV;   // elements of one LDS tile
  static constexpr int STATE = DK * SP;          // elements of the bf16 state copy
  // finished output rows (DV wide) are staged in the wave's own dead query rows when those are
  // wide enough, else in a tile of their own
  static constexpr bool OWN_STAGE = lds_pitch(DV) > TPK;
  static constexpr int LDS_BYTES = 2 * (2 * TILEK + TILEV + STATE + (OWN_STAGE ? TILEV : 0)) + 4 * C;
  static constexpr int WG_PER_CU = (160 * 1024) / LDS_BYTES;
  // waves per SIMD the register allocation is capped for (two workgroups per compute unit
  // when LDS allows, never more than the hardware needs for one workgroup)
  static constexpr int WAVES_RAW = (WG_PER_CU >= 2 ? 2 : 1) * NW / 4;
  // never budget registers for more than two waves per SIMD unless one workgroup alone needs
  // it: spilling costs more than the second workgroup of a large chunk gains
  static constexpr int WAVES_PER_EU = NW / 4 > 2 ? NW / 4 : (WAVES_RAW > 2 ? 2 : WAVES_RAW);
  // with CS waves per row group: one workgroup alone has NW * CS / 4 waves per SIMD; two
  // workgroups per compute unit when the LDS (one more tile for staging) allows
  template <int CS>
  static constexpr int waves_per_eu() {
    if (CS == 1) return WAVES_PER_EU;
    const int own = NW * CS / 4;
    const int wg = (160 * 1024) / (LDS_BYTES + 2 * TILEV) >= 2 ? 2 : 1;
    return own * wg > 4 ? (own > 4 ? own : 4) : own * wg;
  }
};

// Waves per 16-row group in the scan kernel (see the kernel), chosen per shape by measurement:
// two at d = 128, where one workgroup fills the LDS of a compute unit and four waves are too
// few to cover latencies (+6 % on a 2048-token prefill of 4096 heads); at d = 64 and 32 the
// two variants time the same and the smaller workgroup is kept.
template <int DK, int DV, int C> struct FwdSplit { static constexpr int CS = 1; };
template <> struct FwdSplit<128, 128, 64> { static constexpr int CS = 2; };

// ---------------------------------------------------------------------------------------
// Kernel 1: T[unit][g] = sum over the rows of segment g of kh^T v   (fp32, d_key x d_value;
// K rows are DK wide, V rows DV wide)
// grid = units * n_slots workgroups, workgroup (unit, g) as in the scan kernels: workgroups are
// dealt to the XCDs by their index, and what this kernel reads stays in that XCD's L2 for the
// scan workgroup of the same (unit, g) in the next launch.  Segment g of a unit writes slot g
// of the unit's n_slots slots; segments at or beyond n_compute have no total to form and
// leave at once (the causal forward needs all segments but the last).  The bidirectional
// path uses it for Kh^T V (row-major slots, TILED = false; the causal scans read theirs tile
// by tile, TILED = true).
template <int DK, int DV, int C, bool TILED>
__global__ __launch_bounds__(C * 4) void COTTN_SYM(fwd_segment_state)(
    const e16_t* __restrict__ K, const e16_t* __restrict__ V, float* __restrict__ seg_state,
    int N, int n_slots, int n_compute, int seg_rows, float inv_eps,
    const int* __restrict__ seq_len, int H) {
  using Cfg = FwdCfg<DK, DV, C>;
  using ST = AccTiles<DK, DV, Cfg::NW>;   // key rows, value columns
  using StageK = TileStage<DK, C, Cfg::NT>;
  using StageV = TileStage<DV, C, Cfg::NT>;
  __shared__ __attribute__((aligned(16))) e16_t Ks[Cfg::TILEK];
  __shared__ __attribute__((aligned(16))) e16_t Vs[Cfg::TILEV];

  fetch_argument_now(K, V, seg_state, N, n_slots, n_compute, seg_rows, inv_eps, seq_len, H);
  int unit, g;
  unit_and_segment(blockIdx.x, n_slots, unit, g);
  if (g >= n_compute) return;
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const e16_t* Ku = K + size_t(unit) * N * DK;
  const e16_t* Vu = V + size_t(unit) * N * DV;
  const int row_begin = g * seg_rows;
  const int row_end = min(valid_rows(seq_len, unit, H, N), row_begin + seg_rows);

  // acc[x][y] = S tile (key tile row_tile(y), value tile col_tile(x)), held with the keys
  // along the lanes: element [v] of lane (r, q4) is S[16 kt + r][16 vt + 4 q4 + v], the
  // orientation the forward and the dQ scan keep their running state in
  f32x4 acc[ST::NCT][ST::NRT];
#pragma unroll
  for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
    for (int y = 0; y < ST::NRT; ++y) acc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};

  StageK kst;
  StageV vst;
  kst.fetch(Ku, row_begin, row_end);
  vst.fetch(Vu, row_begin, row_end);
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    float rk[StageK::PASSES];
    kst.row_rinv(inv_eps, rk);
    __syncthreads();  // previous chunk's reads of Ks/Vs are done
    kst.commit_scaled(Ks, rk);
    vst.commit_plain(Vs);
    if (row0 + C < row_end) {
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
    }
    __syncthreads();
    if (ST::active(w)) {
#pragma unroll
      for (int p = 0; p < Cfg::NP; ++p) {
        const int k0 = 32 * p + 8 * q4;
        frag8 bv[ST::NCT], ak[ST::NRT];
#pragma unroll
        for (int x = 0; x < ST::NCT; ++x)
          bv[x] = lds_col_frag(Vs, Cfg::TPV, k0, k0 + 4, 16 * ST::col_tile(w, x), r);
#pragma unroll
        for (int y = 0; y < ST::NRT; ++y)
          ak[y] = lds_col_frag(Ks, Cfg::TPK, k0, k0 + 4, 16 * ST::row_tile(w, y), r);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int y = 0; y < ST::NRT; ++y)
#pragma unroll
          for (int x = 0; x < ST::NCT; ++x) acc[x][y] = mma16(bv[x], ak[y], acc[x][y]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  if (ST::active(w)) {
    float* out = seg_state + (size_t(unit) * n_slots + g) * DK * DV;
#pragma unroll
    for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
      for (int y = 0; y < ST::NRT; ++y)
        store_state_words(out + (TILED ? tiled_state_offset(ST::row_tile(w, y), ST::col_tile(w, x), DV / 16, l)
                                       : (16 * ST::row_tile(w, y) + r) * DV + 16 * ST::col_tile(w, x) + 4 * q4),
                          acc[x][y]);
  }
}

// ---------------------------------------------------------------------------------------
// Kernel 2: in place, per (unit, element): slot g <- sum of slots < g (exclusive prefix
// along the segment axis); slot n_slots-1 never held a total and only receives its prefix.
__global__ __launch_bounds__(256) void fwd_state_carry(float* __restrict__ seg_state, int n_slots,
                                                       int elems_per_state, long total) {
  const long idx = (long(blockIdx.x) * 256 + threadIdx.x) * 4;  // 4 elements per thread
  if (idx >= total) return;
  const long unit = idx / elems_per_state, e = idx % elems_per_state;
  exclusive_running_sum(seg_state + unit * n_slots * elems_per_state + e, n_slots,
                        size_t(elems_per_state), false);
}

// ---------------------------------------------------------------------------------------
// Kernel 3: the chunk scan of one segment.
// The running state is held TRANSPOSED in the accumulators: tile (y, x) of the wave covers
// value rows 16*row_tile(y).. and key columns 16*col_tile(x)..; element [v] of lane (r, q4)
// is S[key 16ct + r][value 16rt + 4 q4 + v].  That way a lane holds 4 consecutive values
// of one key row, which it publishes to the row-major LDS copy Sl[key][value] with one
// 8-byte write, and the update's row-side operand is the V fragment already read for P V.
//
// CS = 2 puts two waves on every 16-row group: both form the masked similarity tile of the
// group, each accumulates one half of the output columns and owns the state tiles whose
// value side is that half.  Per-wave work and registers shrink; the workgroup has twice the
// waves to cover latencies with.
template <int DK, int DV, int C, int CS>
__global__ __launch_bounds__(C * 4 * CS, (FwdCfg<DK, DV, C>::template waves_per_eu<CS>())) void COTTN_SYM(fwd_causal_scan)(
    const e16_t* __restrict__ Q, const e16_t* __restrict__ K, const e16_t* __restrict__ V,
    const float* __restrict__ s, e16_t* __restrict__ O, float* __restrict__ state_out,
    const float* __restrict__ seg_states, const float* __restrict__ state_in, int H, int N, int G,
    int seg_rows, float inv_eps, int sum_totals, const int* __restrict__ seq_len, int s_per_unit,
    int stream_q) {
  using Cfg = FwdCfg<DK, DV, C>;
  constexpr int RG = C / 16;           // row groups of a chunk
  constexpr int NOT = Cfg::DTV / CS;   // output column tiles per wave
  using ST = SplitTiles<DV, DK, RG, CS>;   // value rows, key columns (the state is held transposed)
  using StageK = TileStage<DK, C, Cfg::NT * CS>;
  using StageV = TileStage<DV, C, Cfg::NT * CS>;
  constexpr int TPK = Cfg::TPK, TPV = Cfg::TPV, SP = Cfg::SP;
  constexpr bool OWN_STAGE = CS > 1 || Cfg::OWN_STAGE;
  __shared__ __attribute__((aligned(16))) e16_t Qs[Cfg::TILEK];   // raw q rows
  __shared__ __attribute__((aligned(16))) e16_t Ks[Cfg::TILEK];   // kh = r_j k_j
  __shared__ __attribute__((aligned(16))) e16_t Vs[Cfg::TILEV];   // raw v rows
  __shared__ __attribute__((aligned(16))) e16_t Sl[Cfg::STATE];   // state, [d_key][d_value]
  // with two waves on a row group the q rows stay live in the other wave, and with outputs
  // wider than the queries they do not fit the q rows: own staging tile
  __shared__ __attribute__((aligned(16))) e16_t Os[OWN_STAGE ? Cfg::TILEV : 8];
  __shared__ float rq[C];
  fetch_argument_now(Q, K, V, s, O, state_out, seg_states, state_in, H, N, G, seg_rows, inv_eps,
                     sum_totals, seq_len, s_per_unit, stream_q);
  int unit, g;
  unit_and_segment(blockIdx.x, G, unit, g);
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid / 64), l = tid % 64,
            r = l % 16, q4 = l / 16;
  const int rg = w % RG, cp = w / RG;  // row group, column part
  const e16_t* Qu = Q + size_t(unit) * N * DK;
  const e16_t* Ku = K + size_t(unit) * N * DK;
  const e16_t* Vu = V + size_t(unit) * N * DV;
  e16_t* Ou = O + size_t(unit) * N * DV;
  const float scale = unit_scale(s, unit, H, s_per_unit);
  const int row_begin = g * seg_rows;
  const int seg_end = min(N, row_begin + seg_rows);
  const int row_end = max(row_begin, min(valid_rows(seq_len, unit, H, N), seg_end));

  // running state in fp32 accumulators, seeded with the segment's prefix ([d_key][d_value])
  // seg_states holds either the carried prefixes (slot g = state at the start of segment g)
  // or, with sum_totals set, the raw segment totals: then the workgroup adds up the totals of
  // the segments before its own (few segments: cheaper than a separate carry launch).
  f32x4 sacc[ST::NCT][ST::NRT];
#pragma unroll
  for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
    for (int y = 0; y < ST::NRT; ++y) sacc[x][y] = f32x4{0.f, 0.f, 0.f, 0.f};
  // the first chunk's rows and the stored states are all requested before anything waits
  StageK qst, kst;
  StageV vst;
  qst.fetch(Qu, row_begin, row_end, stream_q != 0);
  kst.fetch(Ku, row_begin, row_end);
  vst.fetch(Vu, row_begin, row_end);
  // the state the sequence starts from (chunked prefill) belongs to every segment's start state
  f32x4 start[ST::NCT][ST::NRT];
  if (state_in != nullptr && ST::active(rg, cp)) {
    const float* src = state_in + size_t(unit) * DK * DV;
#pragma unroll
    for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
      for (int y = 0; y < ST::NRT; ++y)
        start[x][y] = *reinterpret_cast<const f32x4*>(src + (16 * ST::col_tile(rg, cp, x) + r) * DV +
                                                      16 * ST::row_tile(rg, cp, y) + 4 * q4);
  }
  if (seg_states != nullptr && g > 0 && ST::active(rg, cp)) {
    const float* src = seg_states + size_t(unit) * G * DK * DV + 4 * l;
    add_stored_states<ST::STATE_BATCH>(
        sacc, sum_totals ? 0 : g, sum_totals ? g - 1 : g, [&](int gp, int x, int y) {
          return *reinterpret_cast<const f32x4*>(
              src + size_t(gp) * DK * DV +
              tiled_state_offset(ST::col_tile(rg, cp, x), ST::row_tile(rg, cp, y), DV / 16, 0));
        });
  }

  if (state_in != nullptr && ST::active(rg, cp)) {
#pragma unroll
    for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
      for (int y = 0; y < ST::NRT; ++y)
#pragma unroll
        for (int v = 0; v < 4; ++v) sacc[x][y][v] += start[x][y][v];
  }

  RowPieces<DV, NOT> finished;  // output rows of the previous chunk, stored one chunk late
#pragma unroll
  for (int j = 0; j < RowPieces<DV, NOT>::PER_LANE; ++j) finished.v[j] = uint4{0u, 0u, 0u, 0u};
  e16_t* stage = OWN_STAGE ? Os + 16 * rg * TPV : Qs + 16 * rg * TPK;
  const int col0 = 16 * NOT * cp;  // first output column of this wave
  for (int row0 = row_begin; row0 < row_end; row0 += C) {
    // ---- publish the state (bf16) and this chunk's tiles
    if (ST::active(rg, cp)) {
#pragma unroll
      for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
        for (int y = 0; y < ST::NRT; ++y) {
          uint2 pk;
          pk.x = pack2(sacc[x][y][0], sacc[x][y][1]);
          pk.y = pack2(sacc[x][y][2], sacc[x][y][3]);
          *reinterpret_cast<uint2*>(Sl + (16 * ST::col_tile(rg, cp, x) + r) * SP +
                                    16 * ST::row_tile(rg, cp, y) + 4 * q4) = pk;
        }
    }
    {
      float rk[StageK::PASSES], rqv[StageK::PASSES];
      qst.row_rinv(inv_eps, rqv);
      kst.row_rinv(inv_eps, rk);
      qst.commit_plain(Qs);
      qst.store_rinv(rq, rqv);
      kst.commit_scaled(Ks, rk);
      vst.commit_plain(Vs);
    }
    if (row0 + C < row_end) {
      qst.fetch(Qu, row0 + C, row_end, stream_q != 0);
      kst.fetch(Ku, row0 + C, row_end);
      vst.fetch(Vu, row0 + C, row_end);
    }
    if (row0 > row_begin)
      store_row_pieces<DV, NOT>(finished, Ou, row0 - C + 16 * rg, row_end, l, col0);
    __syncthreads();

    // ---- inter-chunk part: O^T += S^T Q^T (contraction over d_key = rows of Sl)
    frag8 qf[Cfg::KSK];  // q rows of this wave: column-side operand of every product
#pragma unroll
    for (int ks = 0; ks < Cfg::KSK; ++ks)
      qf[ks] = lds_row_frag(Qs + (16 * rg + r) * TPK + 32 * ks + 8 * q4);
    // oacc[nt][v] = O[query 16 rg + r][value col0 + 16 nt + 4 q4 + v] before the row factor
    f32x4 oacc[NOT];
#pragma unroll
    for (int nt = 0; nt < NOT; ++nt) oacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < Cfg::KSK; ++ks) {
      frag8 sf[NOT];
#pragma unroll
      for (int nt = 0; nt < NOT; ++nt)
        sf[nt] = lds_col_frag(Sl, SP, 32 * ks + 8 * q4, 32 * ks + 8 * q4 + 4, col0 + 16 * nt, r);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int nt = 0; nt < NOT; ++nt) oacc[nt] = mma16(sf[nt], qf[ks], oacc[nt]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- intra-chunk part and state update, two key tiles (32 tokens) at a time
#pragma unroll
    for (int p = 0; p < Cfg::NP; ++p) {
      const bool diag_or_below = 2 * p <= rg;  // wave-uniform: else every key is masked
      // k slot (q4, e) of the P fragment is token 32p + 16*(e/4) + 4*q4 + e%4; V and K are
      // read down their rows in the same order
      const int t0 = 32 * p + 4 * q4, t1 = 32 * p + 16 + 4 * q4;
      frag8 vc[NOT], kcol[ST::NCT], vrow[ST::NRT], kr[2][Cfg::KSK];
#pragma unroll
      for (int nt = 0; nt < NOT; ++nt) vc[nt] = lds_col_frag(Vs, TPV, t0, t1, col0 + 16 * nt, r);
#pragma unroll
      for (int x = 0; x < ST::NCT; ++x)
        kcol[x] = lds_col_frag(Ks, TPK, t0, t1, 16 * ST::col_tile(rg, cp, x), r);
      if (!ST::ROW_OPERAND_IS_OUTPUT_V) {
#pragma unroll
        for (int y = 0; y < ST::NRT; ++y)
          vrow[y] = lds_col_frag(Vs, TPV, t0, t1, 16 * ST::row_tile(rg, cp, y), r);
      }
      if (diag_or_below) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
          for (int ks = 0; ks < Cfg::KSK; ++ks)
            kr[half][ks] = lds_row_frag(Ks + (16 * (2 * p + half) + r) * TPK + 32 * ks + 8 * q4);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (diag_or_below) {
        u32x4 pw;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int jt = 2 * p + half;
          f32x4 pacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < Cfg::KSK; ++ks) pacc = mma16(kr[half][ks], qf[ks], pacc);
          // pacc[v] = q_(16 rg + r) . k_(16jt + 4*q4 + v); keep key <= query
          float kept[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const bool keep = (jt < rg) || (jt == rg && 4 * q4 + v <= r);
            kept[v] = keep ? pacc[v] : 0.f;
          }
          pw[2 * half + 0] = pack2(kept[0], kept[1]);
          pw[2 * half + 1] = pack2(kept[2], kept[3]);
        }
        const frag8 pf = __builtin_bit_cast(frag8, pw);
#pragma unroll
        for (int nt = 0; nt < NOT; ++nt) oacc[nt] = mma16(vc[nt], pf, oacc[nt]);
      }
      // state update S^T += v^T kh over these 32 tokens
      if (ST::active(rg, cp)) {
#pragma unroll
        for (int y = 0; y < ST::NRT; ++y)
#pragma unroll
          for (int x = 0; x < ST::NCT; ++x)
            sacc[x][y] = mma16(ST::ROW_OPERAND_IS_OUTPUT_V ? vc[y] : vrow[y], kcol[x], sacc[x][y]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- O rows: factor s_h r_i, staged through the wave's own (now dead) rows of Qs, or
    // through its part of the staging tile
    const float row_factor = scale * rq[16 * rg + r];
    wave_lds_sync();
    gather_rows_transposed<DV, NOT>(oacc, row_factor, stage, l, finished, col0);
    __syncthreads();  // all reads of Ks, Vs, Sl done before the next chunk overwrites them
  }
  if (row_begin < row_end) {
    const int last = row_begin + (row_end - row_begin - 1) / C * C;
    store_row_pieces<DV, NOT>(finished, Ou, last + 16 * rg, row_end, l, col0);
  }

  if (seq_len != nullptr) zero_rows_e16<DV>(Ou, row_end, seg_end);  // rows that do not exist

  if (state_out != nullptr && g == G - 1 && ST::active(rg, cp)) {
    float* out = state_out + size_t(unit) * DK * DV;
#pragma unroll
    for (int x = 0; x < ST::NCT; ++x)
#pragma unroll
      for (int y = 0; y < ST::NRT; ++y)
        *reinterpret_cast<f32x4*>(out + (16 * ST::col_tile(rg, cp, x) + r) * DV +
                                  16 * ST::row_tile(rg, cp, y) + 4 * q4) = sacc[x][y];
  }
}

template <int DK, int DV, int C>
hipError_t run_fwd_causal(const CausalArgs& a) {
  using Cfg = FwdCfg<DK, DV, C>;
  const int units = a.B * a.H;
  const e16_t* Q = static_cast<const e16_t*>(a.Q);
  const e16_t* K = static_cast<const e16_t*>(a.K);
  const e16_t* V = static_cast<const e16_t*>(a.V);
  float* ws = static_cast<float*>(a.workspace);  // [units][G] states of DK x DV (tiled) when G > 1
  const float inv_eps = 1.0f / a.eps;
  hipError_t err = hipSuccess;
  // few segments: no carry launch, each scan workgroup adds up the totals before its segment
  const bool sum_in_scan = a.G <= kMaxSegmentsSummedInScan;
  if (a.G > 1) {
    err = COTTN_SYM(launch_fwd_segment_totals)(a, ws);
    if (err != hipSuccess) return err;
    if (!sum_in_scan) {
      err = launch_fwd_state_carry(ws, units, a.G, DK * DV, a.stream);
      if (err != hipSuccess) return err;
    }
  }
  constexpr int CS = FwdSplit<DK, DV, C>::CS;
  // Q rows are read once here.  When the call's four tensors exceed the 256 MB last-level cache
  // nothing of them survives until a backward call either, and loading them non-temporally
  // keeps the K, V rows the totals kernel left in the L2 in place (long context: scan 98 ->
  // 87 us); below that size a backward that follows finds the rows cached, and plain loads win.
  const bool stream_q = 2.0 * units * double(a.N) * (DK + DV) * sizeof(e16_t) > 256.0 * 1024 * 1024;
  return launch_kernel(COTTN_SYM_STR(fwd_causal_scan), COTTN_SYM(fwd_causal_scan)<DK, DV, C, CS>, dim3(units * a.G),
                       dim3(Cfg::NT * CS), 0, a.stream, Q, K, V, a.s, static_cast<e16_t*>(a.O), a.state,
                       a.G > 1 ? ws : nullptr, a.state_in, a.H, a.N, a.G, a.seg_rows, inv_eps,
                       sum_in_scan ? 1 : 0, a.seq_len, a.s_per_unit, stream_q ? 1 : 0);
}

}  // namespace

template <int DK, int DV, bool TILED>
static hipError_t run_segment_totals(const SegmentTotalsArgs& t) {
  const e16_t* X = static_cast<const e16_t*>(t.X);
  const e16_t* Y = static_cast<const e16_t*>(t.Y);
  const float inv_eps = 1.0f / t.eps;
  // The totals kernel takes 128-row tiles when the segment is that long: a 512-thread
  // workgroup has all of its loads in flight at once instead of paying one memory latency per
  // 64-row chunk, and several workgroups still fit a compute unit (two 256-row tiles of the
  // operand-tile pitch would leave room for one: measured 0.6 us slower on the GPT shape).
  const dim3 grid(t.units * t.G);
  if (t.seg_rows >= 128)
    return launch_kernel(COTTN_SYM_STR(fwd_segment_state), COTTN_SYM(fwd_segment_state)<DK, DV, 128, TILED>, grid, dim3(512),
                         0, t.stream, X, Y, t.dst, t.N, t.G, t.n_compute, t.seg_rows, inv_eps,
                         t.seq_len, t.H);
  return launch_kernel(COTTN_SYM_STR(fwd_segment_state), COTTN_SYM(fwd_segment_state)<DK, DV, 64, TILED>, grid, dim3(256), 0,
                       t.stream, X, Y, t.dst, t.N, t.G, t.n_compute, t.seg_rows, inv_eps, t.seq_len, t.H);
}

hipError_t COTTN_SYM(launch_segment_totals)(const SegmentTotalsArgs& t) {
  switch (t.dk * 1000 + t.dv) {
    case 32032: return t.tiled ? run_segment_totals<32, 32, true>(t) : run_segment_totals<32, 32, false>(t);
    case 32064: return t.tiled ? run_segment_totals<32, 64, true>(t) : run_segment_totals<32, 64, false>(t);
    case 32128: return t.tiled ? run_segment_totals<32, 128, true>(t) : run_segment_totals<32, 128, false>(t);
    case 64032: return t.tiled ? run_segment_totals<64, 32, true>(t) : run_segment_totals<64, 32, false>(t);
    case 64064: return t.tiled ? run_segment_totals<64, 64, true>(t) : run_segment_totals<64, 64, false>(t);
    case 64128: return t.tiled ? run_segment_totals<64, 128, true>(t) : run_segment_totals<64, 128, false>(t);
    case 128032: return t.tiled ? run_segment_totals<128, 32, true>(t) : run_segment_totals<128, 32, false>(t);
    case 128064: return t.tiled ? run_segment_totals<128, 64, true>(t) : run_segment_totals<128, 64, false>(t);
    case 128128: return t.tiled ? run_segment_totals<128, 128, true>(t) : run_segment_totals<128, 128, false>(t);
    default: return hipErrorInvalidValue;
  }
}

hipError_t COTTN_SYM(launch_fwd_segment_totals)(const CausalArgs& a, float* dst) {
  SegmentTotalsArgs t{};
  t.X = a.K; t.Y = a.V; t.dst = dst;
  t.units = a.B * a.H; t.N = a.N; t.dk = a.dk; t.dv = a.dv; t.G = a.G; t.n_compute = a.G - 1;
  t.seg_rows = a.seg_rows; t.eps = a.eps; t.stream = a.stream;
  t.seq_len = a.seq_len; t.H = a.H;
  t.tiled = true;  // read by the scan kernels only
  return COTTN_SYM(launch_segment_totals)(t);
}

#ifndef COTTN_ELEM_F16  // not specific to the element type: defined once, by the bf16 build
hipError_t launch_fwd_state_carry(float* seg_state, int units, int G, int elems, hipStream_t st) {
  const long total = long(units) * elems;
  return launch_kernel("fwd_state_carry", fwd_state_carry, dim3(unsigned((total / 4 + 255) / 256)),
                       dim3(256), 0, st, seg_state, G, elems, total);
}
#endif

hipError_t COTTN_SYM(fwd_causal)(const CausalArgs& a) {
  // d_key != d_value: chunks of 64 rows
  switch ((a.dk * 1000 + a.dv) * 1000 + a.C) {
    case 32032064: return run_fwd_causal<32, 32, 64>(a);
    case 32032128: return run_fwd_causal<32, 32, 128>(a);
    case 32032256: return run_fwd_causal<32, 32, 256>(a);
    case 64064064: return run_fwd_causal<64, 64, 64>(a);
    case 64064128: return run_fwd_causal<64, 64, 128>(a);
    case 64064256: return run_fwd_causal<64, 64, 256>(a);
    case 128128064: return run_fwd_causal<128, 128, 64>(a);
    case 32064064: return run_fwd_causal<32, 64, 64>(a);
    case 32128064: return run_fwd_causal<32, 128, 64>(a);
    case 64032064: return run_fwd_causal<64, 32, 64>(a);
    case 64128064: return run_fwd_causal<64, 128, 64>(a);
    case 128032064: return run_fwd_causal<128, 32, 64>(a);
    case 128064064: return run_fwd_causal<128, 64, 64>(a);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cottn
