// Host-side glue between the C-ABI entry points and the kernel files: argument bundles,
// the per-dtype launch functions each kernel file defines, and the launch wrapper that
// optionally brackets a kernel with timing events.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace cottn {

// Sequence split chosen on the host: G segments of seg_rows rows (a multiple of C) per
// (batch, head); the last segment may be shorter.
struct CausalArgs {
  const void* Q; const void* K; const void* V; const float* s;
  const void* dO;                 // backward only
  void* O; float* state;          // forward only (state may be null)
  void* dQ; void* dK; void* dV; float* ds;  // backward only
  void* workspace;
  int B, H, N, d, C, G, seg_rows;
  float eps;
  hipStream_t stream;
};

struct StepArgs {
  const void* q; const void* k; const void* v; const float* s; float* state; void* o;
  int B, H, d;
  float eps;
  hipStream_t stream;
};

// defined in the kernel files; every function only enqueues work on args.stream
hipError_t fwd_causal_bf16(const CausalArgs& a);
hipError_t bwd_causal_bf16(const CausalArgs& a);
hipError_t fwd_bidir_bf16(const CausalArgs& a);
hipError_t bwd_bidir_bf16(const CausalArgs& a);
hipError_t fwd_causal_f32(const CausalArgs& a);
hipError_t bwd_causal_f32(const CausalArgs& a);
hipError_t fwd_bidir_f32(const CausalArgs& a);
hipError_t bwd_bidir_f32(const CausalArgs& a);
hipError_t step_any(const StepArgs& a, int dtype);

// small fp32 state kernels shared by the bf16 and fp32 paths (defined next to their kernels)
hipError_t launch_fwd_state_carry(float* seg_state, int units, int G, int elems, hipStream_t st);
hipError_t launch_bwd_state_carry(float* fwd_tot, float* rev_tot, int units, int G, int elems,
                                  hipStream_t st);
hipError_t launch_reduce_ds(const float* partial, float* ds, int B, int H, int G, hipStream_t st);
hipError_t launch_bidir_combine(float* totals, size_t pair_stride, int n_pairs, int units, int G,
                                int elems, float* state, float* ds_partial, hipStream_t st);

// profiling hooks (api.hip)
bool profile_on();
void profile_begin(const char* kernel_name, hipStream_t stream);
void profile_end(hipStream_t stream);

// Runs `enqueue` (one kernel launch) and returns the launch status.
template <class F>
inline hipError_t launch(const char* kernel_name, hipStream_t stream, F&& enqueue) {
  const bool prof = profile_on();
  if (prof) profile_begin(kernel_name, stream);
  enqueue();
  hipError_t err = hipGetLastError();
  if (prof) profile_end(stream);
  return err;
}

}  // namespace cottn
