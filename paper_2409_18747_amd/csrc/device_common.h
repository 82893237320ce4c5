// Device-side primitives shared by the gfx950 kernels: vector types, the bf16 MFMA
// wrapper, LDS fragment reads (plain and transposing), bf16 packing, lane reductions.
// Nothing in here knows about attention.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cottn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef uint16_t bf16_t;  // storage type of bf16 data in global memory and LDS

#define COTTN_LDS __attribute__((address_space(3)))

// Optional in-kernel timeline for tuning builds: a translation unit that defines
// COTTN_TRACE_POINT(i) before including the kernel sources gets a hook at the phase
// boundaries of the scan kernels; the library build leaves it empty.
#ifndef COTTN_TRACE_POINT
#define COTTN_TRACE_POINT(i)
#endif

// Row pitch (in elements) of a bf16 LDS tile with `cols` columns: 8 extra elements (16 B)
// shift consecutive rows by 4 banks, which makes both the 16-byte row reads of 16 rows and
// the 8-byte transposing reads conflict-free.
__host__ __device__ constexpr int lds_pitch(int cols) { return cols + 8; }

// D(16x16) += A(16x32) * B(32x16), bf16 in, fp32 accumulate.
// Lane l = 16*g + r holds  A[row r][k = 8g..8g+7],  B[k = 8g..8g+7][col r],
// and D[row 4g+v][col r] in acc[v].  The order of the k slots is free as long as A and B
// use the same one, which several kernels exploit to feed an accumulator tile straight
// back in as an operand.
__device__ __forceinline__ f32x4 mma16(bf16x8 a, bf16x8 b, f32x4 acc) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 zero_frag() {
  s16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
  return __builtin_bit_cast(bf16x8, z);
}

// Operand fragment whose k index runs along an LDS row: 8 consecutive elements.
__device__ __forceinline__ bf16x8 lds_row_frag(const bf16_t* p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p));
}

// Transposing 8-byte LDS read (gfx950): inside each group of 16 lanes, lane i passes the
// address of 4 consecutive elements, taken as row i/4, columns 4*(i%4).. of a 4x16 block;
// it receives column i of the block's 4 rows.
__device__ __forceinline__ s16x4 lds_read_tr(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((COTTN_LDS s16x4*)(p));
}

// Operand fragment whose k index runs DOWN the rows of a row-major LDS tile (pitch in
// elements): the lane with r = lane%16 receives tile[k0 + 0..3][col0 + r] and
// tile[k1 + 0..3][col0 + r].  k0/k1 are the first rows of the two 4-row groups that
// fill this lane's 8 k slots.
__device__ __forceinline__ bf16x8 lds_col_frag(const bf16_t* tile, int pitch, int k0, int k1,
                                               int col0, int r) {
  const int sub_row = r >> 2, sub_col = (r & 3) * 4;
  s16x4 lo = lds_read_tr(tile + (k0 + sub_row) * pitch + col0 + sub_col);
  s16x4 hi = lds_read_tr(tile + (k1 + sub_row) * pitch + col0 + sub_col);
  s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __builtin_bit_cast(float, uint32_t(b) << 16);
}
// round to nearest even
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(bf16_t, static_cast<__bf16>(f));
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return uint32_t(f32_to_bf16(lo)) | (uint32_t(f32_to_bf16(hi)) << 16);
}
__device__ __forceinline__ void unpack8(uint4 raw, float* f) {
  f[0] = __builtin_bit_cast(float, raw.x << 16);
  f[1] = __builtin_bit_cast(float, raw.x & 0xFFFF0000u);
  f[2] = __builtin_bit_cast(float, raw.y << 16);
  f[3] = __builtin_bit_cast(float, raw.y & 0xFFFF0000u);
  f[4] = __builtin_bit_cast(float, raw.z << 16);
  f[5] = __builtin_bit_cast(float, raw.z & 0xFFFF0000u);
  f[6] = __builtin_bit_cast(float, raw.w << 16);
  f[7] = __builtin_bit_cast(float, raw.w & 0xFFFF0000u);
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 r;
  r.x = pack_bf16(f[0], f[1]);
  r.y = pack_bf16(f[2], f[3]);
  r.z = pack_bf16(f[4], f[5]);
  r.w = pack_bf16(f[6], f[7]);
  return r;
}

// x of another lane of the same row of 16 lanes, chosen by a DPP control word: no LDS
// traffic and no extra latency, unlike a general cross-lane permute.
template <int DPP_CTRL>
__device__ __forceinline__ float dpp_read(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), DPP_CTRL, 0xF, 0xF, true));
}

// Sum over the `width` consecutive lanes (a power of two <= 64) that contain this lane; every
// lane of the group ends with the total.  Up to 16 lanes this is DPP only: swap within
// pairs, swap pairs within quads, then mirror the 8-lane half-row and the 16-lane row (after
// the earlier steps every lane of a quad holds the same value, so a mirror pairs each quad
// with a quad of the other half).
template <int width>
__device__ __forceinline__ float group_sum(float x) {
  static_assert(width == 1 || width == 2 || width == 4 || width == 8 || width == 16 ||
                width == 32 || width == 64, "width must be a power of two");
  if (width >= 2) x += dpp_read<0xB1>(x);    // quad_perm [1,0,3,2]
  if (width >= 4) x += dpp_read<0x4E>(x);    // quad_perm [2,3,0,1]
  if (width >= 8) x += dpp_read<0x141>(x);   // row_half_mirror
  if (width >= 16) x += dpp_read<0x140>(x);  // row_mirror
  if (width >= 32) x += __shfl_xor(x, 16, 64);
  if (width >= 64) x += __shfl_xor(x, 32, 64);
  return x;
}

// Orders this wave's earlier LDS writes before its later LDS reads (lanes exchange data
// through LDS without a workgroup barrier).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Padded batches (sequences of different lengths in one [B][H][N][d] tensor): rows at or
// beyond seq_len[batch] do not exist.  They are never read, contribute to no sum, and the
// rows of every output tensor there are written as zeros.  Without lengths all N rows exist.
__device__ __forceinline__ int valid_rows(const int* __restrict__ seq_len, int unit, int H, int N) {
  return seq_len != nullptr ? min(N, max(0, seq_len[unit / H])) : N;
}
// The scale is one value per head, or, for padded batches whose stabiliser depends on each
// sequence's own length (Sec. 3.3), one per (batch, head).
__device__ __forceinline__ float unit_scale(const float* __restrict__ s, int unit, int H,
                                            int per_unit) {
  return s[per_unit ? unit : unit % H];
}
// Zeros rows row_lo..row_hi-1 of a [.][D] tensor of 2-byte elements (whole workgroup).
template <int D>
__device__ __forceinline__ void zero_rows_bf16(bf16_t* __restrict__ dst, int row_lo, int row_hi) {
  const long pieces = long(max(0, row_hi - row_lo)) * (D / 8);
  uint4* p = reinterpret_cast<uint4*>(dst + size_t(row_lo) * D);
  for (long i = threadIdx.x; i < pieces; i += blockDim.x) p[i] = uint4{0u, 0u, 0u, 0u};
}

// 16-byte store of a result that this library does not read again soon: marked non-temporal,
// so that the line does not displace input rows another kernel of the same step re-reads
// from this XCD's L2.
__device__ __forceinline__ void store_streaming(void* dst, uint4 v) {
#ifdef COTTN_PLAIN_OUTPUT_STORES
  *reinterpret_cast<uint4*>(dst) = v;
#else
  __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4*>(dst));
#endif
}

// Stores of segment states to the workspace: read next by workgroups on other XCDs, which this
// XCD's L2 cannot serve, so they are marked non-temporal as well.
__device__ __forceinline__ void store_state_word(float* dst, float v) {
#ifdef COTTN_PLAIN_STATE_STORES
  *dst = v;
#else
  __builtin_nontemporal_store(v, dst);
#endif
}
__device__ __forceinline__ void store_state_words(float* dst, f32x4 v) {
#ifdef COTTN_PLAIN_STATE_STORES
  *reinterpret_cast<f32x4*>(dst) = v;
#else
  __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst));
#endif
}

// 1 / max(sqrt(sum_sq), eps)
__device__ __forceinline__ float inv_norm(float sum_sq, float eps) {
  return 1.0f / fmaxf(sqrtf(sum_sq), eps);
}

}  // namespace cottn
