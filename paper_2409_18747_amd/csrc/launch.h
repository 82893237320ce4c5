// Host-side glue between the C-ABI entry points and the kernel files: argument bundles,
// the per-dtype launch functions each kernel file defines, and the launch wrapper that
// optionally attaches timing events to a kernel.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace cottn {

// Sequence split chosen on the host: G segments of seg_rows rows (a multiple of C) per
// (batch, head); the last segment may be shorter.
struct CausalArgs {
  const void* Q; const void* K; const void* V; const float* s;
  const void* dO;                 // backward only
  void* O; float* state;          // forward only (state may be null)
  // a sequence processed in pieces (causal only): null, or the forward-time state Kh^T V of
  // the rows before this piece (forward and backward), the reverse-time state Qh^T dO of the
  // rows after it (backward, in), and that state with this piece added (backward, out)
  const float* state_in;
  const float* rev_state_in;
  float* rev_state_out;
  // padded batches: null, or int[B] row counts (then s and ds are [B][H], see s_per_unit)
  const int* seq_len;
  int s_per_unit;                 // s (and ds) indexed by (batch, head) instead of head
  void* dQ; void* dK; void* dV; float* ds;  // backward only
  // backward only: null, or the segment states the forward call with the same split left in
  // its workspace (then the backward does not recompute them)
  const float* saved_fwd_states;
  void* workspace;
  // dk, dv: head dimensions of queries / keys and of values / outputs (Sec. 2.1: d_H_key,
  // d_H_value); Q, K, dQ, dK are [B][H][N][dk], V, O, dO, dV [B][H][N][dv], states [dk][dv]
  int B, H, N, dk, dv, C, G, seg_rows;
  float eps;
  hipStream_t stream;
};

// Up to this many segments per (batch, head) the scan kernels add up the segment totals they
// need themselves and no carry kernel is launched; above it the state arrays hold prefixes
// (suffixes for the reverse-time states).  The forward and the backward must agree on it for
// the backward to take over the forward's saved states.
constexpr int kMaxSegmentsSummedInScan = 4;

struct StepArgs {
  const void* q; const void* k; const void* v; const float* s; float* state; void* o;
  int B, H, dk, dv;  // q, k are [B][H][dk]; v, o [B][H][dv]; state [B][H][dk][dv]
  float eps;
  hipStream_t stream;
};

// defined in the kernel files; every function only enqueues work on args.stream
hipError_t fwd_causal_bf16(const CausalArgs& a);
hipError_t bwd_causal_bf16(const CausalArgs& a);
hipError_t fwd_bidir_bf16(const CausalArgs& a);
hipError_t bwd_bidir_bf16(const CausalArgs& a);
hipError_t fwd_causal_f16(const CausalArgs& a);
hipError_t bwd_causal_f16(const CausalArgs& a);
hipError_t fwd_bidir_f16(const CausalArgs& a);
hipError_t bwd_bidir_f16(const CausalArgs& a);
hipError_t fwd_causal_f32(const CausalArgs& a);
hipError_t bwd_causal_f32(const CausalArgs& a);
hipError_t fwd_bidir_f32(const CausalArgs& a);
hipError_t bwd_bidir_f32(const CausalArgs& a);
hipError_t step_any(const StepArgs& a, int dtype);

// small fp32 state kernels shared by the 16-bit and fp32 paths (defined next to their kernels)
hipError_t launch_fwd_state_carry(float* seg_state, int units, int G, int elems, hipStream_t st);
// either array may be null: then only the other one is carried
hipError_t launch_bwd_state_carry(float* fwd_tot, float* rev_tot, int units, int G, int elems,
                                  hipStream_t st);
// 16-bit paths: segment totals of Kh^T V for all segments but the last, [units][G][d][d] fp32 in `dst`
// (the first kernel of the causal forward, also used by a backward without saved states)
hipError_t launch_fwd_segment_totals_bf16(const CausalArgs& a, float* dst);
hipError_t launch_fwd_segment_totals_f16(const CausalArgs& a, float* dst);

// The same kernel in general: dst[unit][g] = sum over the rows of segment g of N(X)^T Y
// (dk x dv) for g < n_compute (G slots per unit).
struct SegmentTotalsArgs {
  const void* X; const void* Y; float* dst;
  int units, N, dk, dv, G, n_compute, seg_rows;  // X rows are dk wide, Y rows dv wide
  float eps;
  const int* seq_len; int H;  // padded batches: rows at or beyond seq_len[unit / H] do not exist
  // dst row-major [dk][dv] per slot (false), or in the tile order the causal scan kernels read
  // their stored states in (device_common.h: tiled_state_offset, tile (key tile, value tile))
  bool tiled;
  hipStream_t stream;
};
hipError_t launch_segment_totals_bf16(const SegmentTotalsArgs& t);
hipError_t launch_segment_totals_f16(const SegmentTotalsArgs& t);
// ds[h] = sum over batches b and j < n of partial[(b H + h) n + j]; per_unit: ds[b][h] instead
hipError_t launch_reduce_ds(const float* partial, float* ds, int B, int H, int n, int per_unit,
                            hipStream_t st);
hipError_t launch_bidir_combine(float* totals, size_t pair_stride, int n_pairs, int units, int G,
                                int elems, float* state, float* ds_partial, hipStream_t st);

// the stabiliser map of Sec. 3.3 and its gradient (scale.hip)
hipError_t launch_scale_from_m(const float* m, float* s, int H, float n, hipStream_t st);
hipError_t launch_scale_backward(const float* m, const float* ds, float* dm, int H, float n,
                                 hipStream_t st);

hipError_t launch_scale_from_m_varlen(const float* m, const int* seq_len, float* s, int B, int H,
                                      hipStream_t st);
hipError_t launch_scale_backward_varlen(const float* m, const int* seq_len, const float* ds,
                                        float* dm, int B, int H, hipStream_t st);

// profiling hooks (api.hip): when profiling is on, hands out a fresh pair of events that the
// launch attaches to the kernel itself, so they time the kernel's own begin and end.
bool profile_on();
void profile_events(const char* kernel_name, hipEvent_t* begin, hipEvent_t* end);

// Enqueues one kernel on `stream` and returns the launch status.
template <class... Params, class... Args>
inline hipError_t launch_kernel(const char* kernel_name, void (*kernel)(Params...), dim3 grid,
                                dim3 block, size_t dynamic_lds, hipStream_t stream, Args... args) {
  hipEvent_t begin = nullptr, end = nullptr;
  if (profile_on()) profile_events(kernel_name, &begin, &end);
  hipExtLaunchKernelGGL(kernel, grid, block, dynamic_lds, stream, begin, end, 0,
                        static_cast<Params>(args)...);
  return hipGetLastError();
}

}  // namespace cottn
