// One recurrent decode step (Sec. 5, eq. hidden_state_obs) for B*H independent fp32 states of
// d_key x d_value (DK x DV; q and k are DK wide, v and o DV wide):
// S <- S + kh^T v (in place), then o = s_h * qh S with the updated state.
//
// The kernel is a pure stream of the state through the chip (read + write of every state
// byte per step); all arithmetic is fp32 FMAs on the vector ALU.  One workgroup owns one
// state: a row of the state is covered by d/4 lanes holding a float4 each, so every wave
// reads and writes whole contiguous rows; all row loads of a thread are issued before any
// is consumed to keep many requests in flight.  The column sums of qh[row] * S[row][:] are
// kept per thread and combined across the row groups through LDS at the end.
#include "device_common.h"
#include "launch.h"

namespace cottn {
namespace {

// q, k, v, o elements: float, or one of the two 16-bit types (converted with the compiler's
// round-to-nearest-even casts)
template <typename T> struct Elem {
  typedef __attribute__((ext_vector_type(4))) T vec4;
  static __device__ __forceinline__ float load(const T* p) { return float(*p); }
  static __device__ __forceinline__ void store(T* p, float x) { *p = static_cast<T>(x); }
  static __device__ __forceinline__ float4 load4(const T* p) {
    const vec4 raw = *reinterpret_cast<const vec4*>(p);
    return float4{float(raw[0]), float(raw[1]), float(raw[2]), float(raw[3])};
  }
};

// Cache policy of the state stream.  The updated state is always written with non-temporal
// stores: nothing reads a written line again before the whole set of states has passed through
// the caches.  The loads are non-temporal too (`stream`, uniform over the launch) when the
// states of the call exceed what the L2s hold (32 MB): a decoder has a set of states per layer,
// so by the time a step comes back to this set it has left the caches, every step reads it from
// HBM, and lines left behind only get in the way (4096 states of 128 x 128, rotating over three
// such sets: 89.6 us per step against 107.8 us with plain loads).  A small set of states is
// re-read from the L2 by the next step, and there plain loads win.
__device__ __forceinline__ float4 load_state_row(const float* p, bool stream) {
  if (stream) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return float4{v[0], v[1], v[2], v[3]};
  }
  return *reinterpret_cast<const float4*>(p);
}
__device__ __forceinline__ void store_state_row(float* p, float4 x) {
  __builtin_nontemporal_store(f32x4{x.x, x.y, x.z, x.w}, reinterpret_cast<f32x4*>(p));
}

template <typename T, int DK, int DV>
__global__ __launch_bounds__(256) void decode_step_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
    const float* __restrict__ s, float* __restrict__ state, T* __restrict__ o, int H, float eps,
    int stream_state) {
  constexpr int TPR = DV / 4;         // threads per state row
  constexpr int RPP = 256 / TPR;      // rows per pass
  constexpr int PASSES = (DK + RPP - 1) / RPP;
  constexpr int D = DK;               // width of q and k
  __shared__ float qh[DK], kh[DK];
  __shared__ float partial[RPP][DV];

  const int unit = blockIdx.x;
  const int tid = threadIdx.x;
  const size_t vbase = size_t(unit) * DK;   // of q, k
  const size_t obase = size_t(unit) * DV;   // of v, o

  // every wave normalises q and k for itself (d <= 128: at most two elements per lane);
  // wave 0 publishes them
  {
    const int l = tid % 64;
    float q0 = Elem<T>::load(q + vbase + (l % D));
    float k0 = Elem<T>::load(k + vbase + (l % D));
    float q1 = 0.f, k1 = 0.f;
    if (D > 64) {
      q1 = Elem<T>::load(q + vbase + ((l + 64) % D));
      k1 = Elem<T>::load(k + vbase + ((l + 64) % D));
    }
    const bool own = l < D;  // for d = 32 lanes 32..63 duplicate lanes 0..31
    float qs = own ? q0 * q0 + q1 * q1 : 0.f;
    float ks = own ? k0 * k0 + k1 * k1 : 0.f;
    qs = group_sum<64>(qs);
    ks = group_sum<64>(ks);
    const float rq = inv_norm(qs, eps), rk = inv_norm(ks, eps);
    if (tid < 64 && own) {
      qh[l] = q0 * rq;
      kh[l] = k0 * rk;
      if (D > 64) {
        qh[l + 64] = q1 * rq;
        kh[l + 64] = k1 * rk;
      }
    }
  }
  const int col = (tid % TPR) * 4;
  const int row_in_pass = tid / TPR;
  const float4 v4 = Elem<T>::load4(v + obase + col);
  float* Su = state + size_t(unit) * DK * DV;

  // (a pass may reach beyond the last key row when DK < 256 / (DV/4): those threads idle)
  float4 rows[PASSES];
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    const int row = p * RPP + row_in_pass;
    rows[p] = float4{0.f, 0.f, 0.f, 0.f};
    if (DK % RPP == 0 || row < DK) rows[p] = load_state_row(Su + size_t(row) * DV + col, stream_state != 0);
  }
  __syncthreads();

  float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    const int row = p * RPP + row_in_pass;
    if (DK % RPP == 0 || row < DK) {
      const float kr = kh[row], qr = qh[row];
      float4 x = rows[p];
      x.x += kr * v4.x;
      x.y += kr * v4.y;
      x.z += kr * v4.z;
      x.w += kr * v4.w;
      store_state_row(Su + size_t(row) * DV + col, x);
      acc.x += qr * x.x;
      acc.y += qr * x.y;
      acc.z += qr * x.z;
      acc.w += qr * x.w;
    }
  }
  *reinterpret_cast<float4*>(&partial[row_in_pass][col]) = acc;
  __syncthreads();
  if (tid < DV) {
    float sum = 0.f;
#pragma unroll
    for (int rpp = 0; rpp < RPP; ++rpp) sum += partial[rpp][tid];
    Elem<T>::store(o + obase + tid, s[unit % H] * sum);
  }
}

template <typename T>
hipError_t run_step(const StepArgs& a) {
  const int units = a.B * a.H;
  const T* q = static_cast<const T*>(a.q);
  const T* k = static_cast<const T*>(a.k);
  const T* v = static_cast<const T*>(a.v);
  T* o = static_cast<T*>(a.o);
  const dim3 grid(units), block(256);
  const int stream_state = double(units) * a.dk * a.dv * sizeof(float) > 32.0 * 1024 * 1024 ? 1 : 0;
#define COTTN_STEP_CASE(DK, DV)                                                                   \
  case DK * 1000 + DV:                                                                            \
    return launch_kernel("decode_step_kernel", decode_step_kernel<T, DK, DV>, grid, block, 0,     \
                         a.stream, q, k, v, a.s, a.state, o, a.H, a.eps, stream_state);
  switch (a.dk * 1000 + a.dv) {
    COTTN_STEP_CASE(32, 32) COTTN_STEP_CASE(32, 64) COTTN_STEP_CASE(32, 128)
    COTTN_STEP_CASE(64, 32) COTTN_STEP_CASE(64, 64) COTTN_STEP_CASE(64, 128)
    COTTN_STEP_CASE(128, 32) COTTN_STEP_CASE(128, 64) COTTN_STEP_CASE(128, 128)
    default:
      return hipErrorInvalidValue;
  }
#undef COTTN_STEP_CASE
}

}  // namespace

hipError_t step_any(const StepArgs& a, int dtype) {
  return dtype == 0 ? run_step<float>(a) : dtype == 1 ? run_step<__bf16>(a) : run_step<_Float16>(a);
}

}  // namespace cottn
