// Device-side primitives shared by the gfx950 kernels: vector types, the 16-bit MFMA
// wrapper, LDS fragment reads (plain and transposing), packing, lane reductions.
// Nothing in here knows about attention.
//
// The MFMA kernels are written once for a 16-bit floating-point element and compiled twice:
// bfloat16 by default, IEEE half when the translation unit defines COTTN_ELEM_F16 before
// including anything (the *_f16.hip files do exactly that and then include the kernel
// source).  COTTN_SYM(name) appends the element's suffix to kernel and launcher names.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cottn {

#ifdef COTTN_ELEM_F16
typedef _Float16 elem_native;  // the compiler's type for one element
#define COTTN_SYM(name) name##_f16
#define COTTN_SYM_STR(name) #name "_f16"
#else
typedef __bf16 elem_native;
#define COTTN_SYM(name) name##_bf16
#define COTTN_SYM_STR(name) #name "_bf16"
#endif
typedef __attribute__((ext_vector_type(8))) elem_native frag8;  // one MFMA operand fragment
typedef __attribute__((ext_vector_type(2))) elem_native elem2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef uint16_t e16_t;  // storage type of a 16-bit element in global memory and LDS

#define COTTN_LDS __attribute__((address_space(3)))

// Row pitches (in elements) of 16-bit LDS arrays.  The LDS moves 64 lanes x 16 bytes in 4
// cycles and 64 x 8 bytes in 2.4 at best (4 for a transposing read of rows that are 8 apart);
// how the 64 addresses of an instruction fall into banks decides whether it gets there.
// Measured on gfx950 with every access pattern of these kernels (cycles per wave instruction,
// 16 waves issuing; the same at d = 32, 64, 128):
//                                         pitch = cols + 8        pitch = cols + 16
//   16-byte row fragments (16 rows)            8.0                     4.1
//   transposing reads over the tokens          4.1                     2.4
//   8-byte writes / reads of 4 cols of a row   8.0 / 2.4              16.0 / 4.1
//   16-byte pieces read back row by row        8.0                    12.0
//   (16-byte writes cost 13 and transposing reads of a state 4.1 with either.)
// So the [rows][cols] operand tiles (read as row fragments and token-column fragments) use
// cols + 16 (unless four such tiles and a state copy would not fit the 160 KB of a compute
// unit: 256-row chunks at d = 64), the state copies and the staging of finished rows
// (8-byte writes) cols + 8.
__host__ __device__ constexpr int lds_pitch(int cols) { return cols + 8; }
__host__ __device__ constexpr int tile_pitch(int cols, int rows) {
  return 2 * (4 * rows * (cols + 16) + cols * lds_pitch(cols)) + 1024 <= 160 * 1024 ? cols + 16
                                                                                  : cols + 8;
}

// D(16x16) += A(16x32) * B(32x16), 16-bit elements in, fp32 accumulate.
// Lane l = 16*g + r holds  A[row r][k = 8g..8g+7],  B[k = 8g..8g+7][col r],
// and D[row 4g+v][col r] in acc[v].  The order of the k slots is free as long as A and B
// use the same one, which several kernels exploit to feed an accumulator tile straight
// back in as an operand.
__device__ __forceinline__ f32x4 mma16(frag8 a, frag8 b, f32x4 acc) {
#ifdef COTTN_ELEM_F16
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc, 0, 0, 0);
#else
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
#endif
}

__device__ __forceinline__ frag8 zero_frag() {
  s16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
  return __builtin_bit_cast(frag8, z);
}

// Operand fragment whose k index runs along an LDS row: 8 consecutive elements.
__device__ __forceinline__ frag8 lds_row_frag(const e16_t* p) {
  return __builtin_bit_cast(frag8, *reinterpret_cast<const uint4*>(p));
}

// Transposing 8-byte LDS read (gfx950): inside each group of 16 lanes, lane i passes the
// address of 4 consecutive elements, taken as row i/4, columns 4*(i%4).. of a 4x16 block;
// it receives column i of the block's 4 rows.
__device__ __forceinline__ s16x4 lds_read_tr(const e16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((COTTN_LDS s16x4*)(p));
}

// Operand fragment whose k index runs DOWN the rows of a row-major LDS tile (pitch in
// elements): the lane with r = lane%16 receives tile[k0 + 0..3][col0 + r] and
// tile[k1 + 0..3][col0 + r].  k0/k1 are the first rows of the two 4-row groups that
// fill this lane's 8 k slots.
__device__ __forceinline__ frag8 lds_col_frag(const e16_t* tile, int pitch, int k0, int k1,
                                               int col0, int r) {
  const int sub_row = r >> 2, sub_col = (r & 3) * 4;
  s16x4 lo = lds_read_tr(tile + (k0 + sub_row) * pitch + col0 + sub_col);
  s16x4 hi = lds_read_tr(tile + (k1 + sub_row) * pitch + col0 + sub_col);
  s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(frag8, v);
}

// element <-> fp32; to_e16 rounds to nearest even
__device__ __forceinline__ float from_e16(e16_t b) {
#ifdef COTTN_ELEM_F16
  return float(__builtin_bit_cast(_Float16, b));
#else
  return __builtin_bit_cast(float, uint32_t(b) << 16);
#endif
}
__device__ __forceinline__ e16_t to_e16(float f) {
  return __builtin_bit_cast(e16_t, static_cast<elem_native>(f));
}
// two values rounded and packed into one word (low half first): written as one vector
// conversion so that it becomes the packed convert instruction, not two converts and a merge
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, elem2));
}
// the two elements of a 32-bit word (low half first)
__device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
#ifdef COTTN_ELEM_F16
  const elem2 p = __builtin_bit_cast(elem2, w);
  lo = float(p[0]);
  hi = float(p[1]);
#else
  lo = __builtin_bit_cast(float, w << 16);
  hi = __builtin_bit_cast(float, w & 0xFFFF0000u);
#endif
}
// fp32 sum of squares of the two elements of a word, added to acc
__device__ __forceinline__ float dot2_self(uint32_t w, float acc) {
  const elem2 p = __builtin_bit_cast(elem2, w);
#ifdef COTTN_ELEM_F16
  return __builtin_amdgcn_fdot2(p, p, acc, false);
#else
  return __builtin_amdgcn_fdot2_f32_bf16(p, p, acc, false);
#endif
}
__device__ __forceinline__ void unpack8(uint4 raw, float* f) {
  unpack2(raw.x, f[0], f[1]);
  unpack2(raw.y, f[2], f[3]);
  unpack2(raw.z, f[4], f[5]);
  unpack2(raw.w, f[6], f[7]);
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 r;
  r.x = pack2(f[0], f[1]);
  r.y = pack2(f[2], f[3]);
  r.z = pack2(f[4], f[5]);
  r.w = pack2(f[6], f[7]);
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
__device__ __forceinline__ void zero_rows_e16(e16_t* __restrict__ dst, int row_lo, int row_hi) {
  const long pieces = long(max(0, row_hi - row_lo)) * (D / 8);
  uint4* p = reinterpret_cast<uint4*>(dst + size_t(row_lo) * D);
  for (long i = threadIdx.x; i < pieces; i += blockDim.x) p[i] = uint4{0u, 0u, 0u, 0u};
}

// 16-byte store of a result that this library does not read again soon: marked non-temporal,
// so that the line does not displace input rows another kernel of the same step re-reads
// from this XCD's L2.
__device__ __forceinline__ void store_streaming(void* dst, uint4 v) {
  __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4*>(dst));
}

// Stores of segment states to the workspace.  A state is read by the next kernel, by
// workgroups of the same (batch, head) unit, which unit_and_segment() puts on this XCD: plain
// stores leave the lines in this XCD's L2 for them (0.5 us of the 52 us step on B8 H12 N1024 d64
// against non-temporal stores).
__device__ __forceinline__ void store_state_word(float* dst, float v) { *dst = v; }
__device__ __forceinline__ void store_state_words(float* dst, f32x4 v) {
  *reinterpret_cast<f32x4*>(dst) = v;
}

// States that only two kernels of this library hand to each other (workspace arrays that no
// caller reads) need not be row-major.  Stored tile by tile in the order the accumulator
// registers hold them - the 16x16 tile (a, b) as 256 consecutive floats, the four values of
// lane l at 4 l - a wave writes or reads a tile with one instruction that covers 1 KB of
// consecutive addresses.  Row-major, the same four-value pieces lie a matrix row apart and one
// instruction touches 16 to 64 cache lines, which the vector L1 looks up one per cycle: with
// up to three stored states per workgroup that was most of the 2 us by which a scan
// workgroup's first chunk started later than its rows arrived.
__device__ __forceinline__ int tiled_state_offset(int tile_a, int tile_b, int tiles_b, int lane) {
  return (tile_a * tiles_b + tile_b) * 256 + 4 * lane;
}

// Makes the compiler fetch a kernel argument where this stands.  Left alone it fetches each
// argument where it is first used, one scalar load and one wait after the other down the
// kernel's prologue (six or more round trips to the scalar cache before the first row is
// requested); pinned at the top, all of them come with one or two wide loads and one wait.
template <class T>
__device__ __forceinline__ void fetch_argument_now(const T& x) {
  asm volatile("" ::"s"(x));
}
template <class T, class... Rest>
__device__ __forceinline__ void fetch_argument_now(const T& x, const Rest&... rest) {
  fetch_argument_now(x);
  fetch_argument_now(rest...);
}

// Which (batch-head unit, segment) a workgroup of a units * G grid works on.  Workgroups are
// dealt to the 8 XCDs round robin by their index, and each XCD has an L2 of its own.  The
// kernels of one call that share this numbering pass data to each other through that L2: the
// rows a totals workgroup read are there for the scan workgroup of the same (unit, segment),
// and the G segments of a unit all land on one XCD (workgroup indices 8 apart), so the segment
// states that the workgroups of a unit write for each other never cross to another L2.
// (Measured on B8 H12 N1024 d64: 1.6 us of a 56 us step against unit = index / G.)
// Units beyond the last whole group of 8 are numbered plainly.
__device__ __forceinline__ void unit_and_segment(int index, int G, int& unit, int& g) {
  const int n_units = gridDim.x / G;
  const int grouped = (n_units / 8) * 8 * G;
  if (index < grouped) {
    const int in_group = index % (8 * G);
    unit = (index / (8 * G)) * 8 + in_group % 8;
    g = in_group / 8;
  } else {
    unit = (n_units / 8) * 8 + (index - grouped) / G;
    g = (index - grouped) % G;
  }
}

// In place, for 4 neighbouring elements of a stack of n matrices `stride` floats apart:
// matrix k (in walking order: first to last, or last to first with `reverse`) <- sum of the
// matrices walked before it.  The last matrix walked never held a value and is not read.  The
// matrices are taken eight at a time with all loads of a batch issued before the first store:
// the sum itself is serial, but a thread then pays one memory latency per eight matrices.
__device__ __forceinline__ void exclusive_running_sum(float* __restrict__ p, int n, size_t stride,
                                                      bool reverse) {
  constexpr int BATCH = 8;
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < n; k0 += BATCH) {
    f32x4 t[BATCH];
#pragma unroll
    for (int i = 0; i < BATCH; ++i) {
      const int k = k0 + i;
      t[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (k + 1 < n) t[i] = *reinterpret_cast<const f32x4*>(p + size_t(reverse ? n - 1 - k : k) * stride);
    }
#pragma unroll
    for (int i = 0; i < BATCH; ++i) {
      const int k = k0 + i;
      if (k < n) {
        *reinterpret_cast<f32x4*>(p + size_t(reverse ? n - 1 - k : k) * stride) = run;
        run += t[i];
      }
    }
  }
}

// 1 / max(sqrt(sum_sq), eps)
__device__ __forceinline__ float inv_norm(float sum_sq, float eps) {
  return 1.0f / fmaxf(sqrtf(sum_sq), eps);
}

}  // namespace cottn
