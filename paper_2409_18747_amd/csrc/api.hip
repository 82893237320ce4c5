// C-ABI entry points of libcottn: argument validation (before anything is enqueued, so it
// works on a host without a GPU), the host-side choice of the sequence split, dispatch to
// the per-dtype kernel launchers, and the optional per-kernel event timing.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/cottn.h"
#include "launch.h"
#include "workspace.h"

namespace cottn {
namespace {

// <= 0: heuristic.  Per thread: a thread that tunes does not change what other threads get.
thread_local int g_tuned_segments = 0;

// ---- profiling state -------------------------------------------------------------------
struct PendingSpan { const char* name; hipEvent_t begin, end; };
struct KernelTotal { const char* name; long launches; double ms; };
bool g_profile_on = false;
std::vector<PendingSpan> g_pending;
std::vector<KernelTotal> g_totals;

bool is_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

bool dim_ok(int d) { return d == 32 || d == 64 || d == 128; }

bool dims_ok(int B, int H, int N, int dk, int dv) {
  if (B < 1 || H < 1 || N < 0) return false;
  if (!dim_ok(dk) || !dim_ok(dv)) return false;
  // element counts must fit comfortably in 64-bit offsets and the grid in 31 bits
  if (double(B) * H > 16777216.0) return false;
  if (double(B) * H * double(N) * (dk > dv ? dk : dv) > 9.0e15) return false;
  return true;
}

}  // namespace

// Split of one (batch, head) sequence into segments; see workspace.h.
bool make_plan(int op, int B, int H, int N, int dk, int dv, int chunk, int dtype, SeqPlan* plan) {
  if (dtype != COTTN_F32 && dtype != COTTN_BF16 && dtype != COTTN_F16) return false;
  if (!dims_ok(B, H, N, dk, dv)) return false;
  int C;
  if (dtype != COTTN_F32) {
    C = chunk == 0 ? 64 : chunk;
    if (C != 64 && C != 128 && C != 256) return false;
    // the larger chunks are built for d_key = d_value in {32, 64}
    if ((dk == 128 || dv == 128 || dk != dv) && C != 64) return false;
  } else {
    C = chunk == 0 ? 32 : chunk;
    if (C != 32) return false;
  }
  const long units = long(B) * H;
  const long n_chunks = (long(N) + C - 1) / C;
  long want;
  if (g_tuned_segments > 0) {
    want = g_tuned_segments;
  } else {
    if (dtype != COTTN_F32 && dk == 128 && dv == 128) {
      // one workgroup fills the LDS of a compute unit at d = 128: a second round of
      // workgroups costs more than shorter segments gain, so never more than one per unit
      // (measured on B8 H12 N1024: 2 segments 143 us, 4 segments 178 us per step)
      want = 256 / units;
    } else {
      // about one and a half workgroups per compute unit: measured best for the scan kernels
      // (more segments shorten the serial chain but add totals to reduce and to add up)
      const long target = 384;
      want = (target + units - 1) / units;
      // the bidirectional kernels have no chain to shorten and little to set up: three
      // workgroups per compute unit measured best there (B32 H12 N512: 59.2 us per forward +
      // backward with 2 segments, 60.7 with 1), as long as the kernels still add up the
      // segment totals themselves
      if (op == COTTN_OP_FWD_BIDIR || op == COTTN_OP_BWD_BIDIR) {
        want = (768 + units - 1) / units;
        if (want > kMaxSegmentsSummedInScan) want = kMaxSegmentsSummedInScan;
      }
      // long serial chains (16 chunks or more per segment) are bound by the memory path, not
      // by the prologue: there two workgroups on every compute unit measured best
      if (n_chunks >= 16 * want) want = (512 + units - 1) / units;
    }
  }
  if (want > n_chunks) want = n_chunks;
  if (want < 1) want = 1;
  const long chunks_per_seg = n_chunks > 0 ? (n_chunks + want - 1) / want : 1;
  const long G = n_chunks > 0 ? (n_chunks + chunks_per_seg - 1) / chunks_per_seg : 1;
  if (units * G > 2147483647L / 4) return false;
  plan->C = C;
  plan->G = int(G);
  plan->seg_rows = int(chunks_per_seg * C);
  return true;
}

bool profile_on() { return g_profile_on; }

void profile_events(const char* kernel_name, hipEvent_t* begin, hipEvent_t* end) {
  PendingSpan sp{kernel_name, nullptr, nullptr};
  if (hipEventCreate(&sp.begin) != hipSuccess) return;
  if (hipEventCreate(&sp.end) != hipSuccess) {
    (void)hipEventDestroy(sp.begin);
    return;
  }
  g_pending.push_back(sp);
  *begin = sp.begin;
  *end = sp.end;
}

namespace {

__global__ void fill_zero_f32(float* p, long n) {
  const long i = long(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

hipError_t zero_f32(float* p, long n, hipStream_t st) {
  if (p == nullptr || n <= 0) return hipSuccess;
  return launch_kernel("fill_zero_f32", fill_zero_f32, dim3(unsigned((n + 255) / 256)), dim3(256),
                       0, st, p, n);
}

int check_common(const void* const* ptrs, int n_ptrs, int B, int H, int N, int dk, int dv,
                 int dtype, float eps) {
  for (int i = 0; i < n_ptrs; ++i)
    if (ptrs[i] == nullptr) return COTTN_E_NULL;
  if (dtype != COTTN_F32 && dtype != COTTN_BF16 && dtype != COTTN_F16) return COTTN_E_DTYPE;
  if (!dims_ok(B, H, N, dk, dv)) return COTTN_E_SHAPE;
  if (!(eps > 0.f)) return COTTN_E_ARG;
  for (int i = 0; i < n_ptrs; ++i)
    if (!is_aligned(ptrs[i], 16)) return COTTN_E_ALIGN;
  return COTTN_OK;
}

int check_workspace(const void* ws, size_t have, size_t need) {
  if (need == 0) return COTTN_OK;
  if (ws == nullptr || have < need) return COTTN_E_WORKSPACE;
  if (!is_aligned(ws, 256)) return COTTN_E_ALIGN;
  return COTTN_OK;
}

int map_hip(hipError_t e) { return e == hipSuccess ? COTTN_OK : COTTN_E_HIP; }

}  // namespace
}  // namespace cottn

using namespace cottn;

extern "C" {

size_t cottn_workspace_bytes_dkdv(int op, int B, int H, int N, int dk, int dv, int chunk,
                                  int dtype) {
  if (op == COTTN_OP_STEP) {
    return (dtype == COTTN_F32 || dtype == COTTN_BF16 || dtype == COTTN_F16) &&
                   dims_ok(B, H, 1, dk, dv)
               ? 0
               : size_t(-1);
  }
  if (op < COTTN_OP_FWD_CAUSAL || op > COTTN_OP_STEP) return size_t(-1);
  SeqPlan plan;
  if (!make_plan(op, B, H, N, dk, dv, chunk, dtype, &plan)) return size_t(-1);
  return workspace_bytes_for(op, B, H, dk, dv, plan);
}

size_t cottn_workspace_bytes(int op, int B, int H, int N, int d, int chunk, int dtype) {
  return cottn_workspace_bytes_dkdv(op, B, H, N, d, d, chunk, dtype);
}

int cottn_segments_dkdv(int op, int B, int H, int N, int dk, int dv, int chunk, int dtype) {
  if (op < COTTN_OP_FWD_CAUSAL || op > COTTN_OP_BWD_BIDIR) return 0;
  SeqPlan plan;
  if (!make_plan(op, B, H, N, dk, dv, chunk, dtype, &plan)) return 0;
  return plan.G;
}

int cottn_segments(int op, int B, int H, int N, int d, int chunk, int dtype) {
  return cottn_segments_dkdv(op, B, H, N, d, d, chunk, dtype);
}

void cottn_tune_segments(int segments) { g_tuned_segments = segments; }

const char* cottn_status_string(int status) {
  switch (status) {
    case COTTN_OK: return "ok";
    case COTTN_E_NULL: return "a required pointer is NULL";
    case COTTN_E_SHAPE: return "unsupported shape: need B,H >= 1, N >= 0, d (d_key, d_value) in "
                               "{32,64,128}, chunk in {0,64,128,256} (16-bit; 64 only when a "
                               "dimension is 128 or d_key != d_value) or {0,32} (fp32)";
    case COTTN_E_DTYPE: return "dtype must be COTTN_F32 (0), COTTN_BF16 (1) or COTTN_F16 (2)";
    case COTTN_E_ALIGN: return "tensor pointers must be 16-byte aligned, the workspace 256-byte aligned";
    case COTTN_E_WORKSPACE: return "workspace is NULL or smaller than cottn_workspace_bytes()";
    case COTTN_E_HIP: return "a HIP call failed";
    case COTTN_E_ARG: return "invalid argument";
    default: return "unknown status";
  }
}

namespace {

__global__ void copy_f32(const float* __restrict__ src, float* __restrict__ dst, long n) {
  const long i = long(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

hipError_t copy_state(float* dst, const float* src, long n, hipStream_t st) {
  return launch_kernel("copy_f32", copy_f32, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, src,
                       dst, n);
}

// seq_len != null in the *_any functions: a padded batch, with s and ds per (batch, head)
int check_lengths(const int* seq_len) {
  return seq_len == nullptr || is_aligned(seq_len, 4) ? COTTN_OK : COTTN_E_ALIGN;
}

int fwd_causal_any(const void* Q, const void* K, const void* V, const float* s, const int* seq_len,
                   const float* state_in, void* O, float* state, void* workspace,
                   size_t workspace_bytes, int B, int H, int N, int dk, int dv, int chunk, int dtype,
                   float eps, void* hip_stream) {
  const void* req[] = {Q, K, V, s, O};
  int st = check_common(req, 5, B, H, N, dk, dv, dtype, eps);
  if (st != COTTN_OK) return st;
  if (state != nullptr && !is_aligned(state, 16)) return COTTN_E_ALIGN;
  if (state_in != nullptr && !is_aligned(state_in, 16)) return COTTN_E_ALIGN;
  if (state_in != nullptr && state_in == state) return COTTN_E_ARG;
  if ((st = check_lengths(seq_len)) != COTTN_OK) return st;
  SeqPlan plan;
  if (!make_plan(COTTN_OP_FWD_CAUSAL, B, H, N, dk, dv, chunk, dtype, &plan)) return COTTN_E_SHAPE;
  st = check_workspace(workspace, workspace_bytes,
                       workspace_bytes_for(COTTN_OP_FWD_CAUSAL, B, H, dk, dv, plan));
  if (st != COTTN_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (N == 0) {
    const long n = long(B) * H * dk * dv;
    if (state == nullptr) return COTTN_OK;
    if (state_in == nullptr) return map_hip(zero_f32(state, n, stream));
    return map_hip(copy_state(state, state_in, n, stream));
  }
  CausalArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.s = s; a.O = O; a.state = state; a.state_in = state_in;
  a.workspace = workspace; a.seq_len = seq_len; a.s_per_unit = seq_len != nullptr;
  a.B = B; a.H = H; a.N = N; a.dk = dk; a.dv = dv; a.C = plan.C; a.G = plan.G; a.seg_rows = plan.seg_rows;
  a.eps = eps; a.stream = stream;
  return map_hip(dtype == COTTN_BF16 ? fwd_causal_bf16(a) : dtype == COTTN_F16 ? fwd_causal_f16(a) : fwd_causal_f32(a));
}

}  // namespace

int cottn_fwd_causal(const void* Q, const void* K, const void* V, const float* s, void* O,
                     float* state, void* workspace, size_t workspace_bytes, int B, int H, int N,
                     int d, int chunk, int dtype, float eps, void* hip_stream) {
  return fwd_causal_any(Q, K, V, s, nullptr, nullptr, O, state, workspace, workspace_bytes, B, H, N,
                        d, d, chunk, dtype, eps, hip_stream);
}

// ---- the causal forward for callers that cannot allocate ------------------------------------
// Its workspace (the fp32 segment states) is this array, part of the library's code object: every
// GPU the library runs on holds its own copy, at its own address, until the process ends.  In
// host code the name below only stands for the symbol; the address kernels can use comes from
// hipGetSymbolAddress, asked once per device with that device current.
namespace {

static __device__ __align__(256) unsigned char scratch[COTTN_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_workspace(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return COTTN_E_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr)
      return COTTN_E_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return COTTN_OK;
}

}  // namespace

int cottn_fwd_causal_static(const void* Q, const void* K, const void* V, const float* s, void* O,
                            float* state, int B, int H, int N, int d, int chunk, int dtype,
                            float eps, void* hip_stream) {
  const void* req[] = {Q, K, V, s, O};
  int st = check_common(req, 5, B, H, N, d, d, dtype, eps);
  if (st != COTTN_OK) return st;
  SeqPlan plan;
  if (!make_plan(COTTN_OP_FWD_CAUSAL, B, H, N, d, d, chunk, dtype, &plan)) return COTTN_E_SHAPE;
  const size_t need = workspace_bytes_for(COTTN_OP_FWD_CAUSAL, B, H, d, d, plan);
  if (need > size_t(COTTN_STATIC_WORKSPACE_BYTES)) return COTTN_E_WORKSPACE;
  void* ws = nullptr;
  if (need > 0 && (st = static_workspace(&ws)) != COTTN_OK) return st;
  // every slot of the segment-state array that a kernel reads is written earlier in the same
  // call, so what the previous call left in the array needs no clearing
  return fwd_causal_any(Q, K, V, s, nullptr, nullptr, O, state, ws, need, B, H, N,
                        d, d, chunk, dtype, eps, hip_stream);
}

int cottn_fwd_causal_from_state(const void* Q, const void* K, const void* V, const float* s,
                                const float* state_in, void* O, float* state, void* workspace,
                                size_t workspace_bytes, int B, int H, int N, int d, int chunk,
                                int dtype, float eps, void* hip_stream) {
  if (state_in == nullptr) return COTTN_E_NULL;
  return fwd_causal_any(Q, K, V, s, nullptr, state_in, O, state, workspace, workspace_bytes, B, H, N,
                        d, d, chunk, dtype, eps, hip_stream);
}

namespace {

int bwd_causal_any(const void* Q, const void* K, const void* V, const float* s, const int* seq_len,
                   const void* dO, const float* state_in, const float* rev_state_in, void* dQ,
                   void* dK, void* dV, float* ds, float* rev_state_out,
                   const void* fwd_workspace, size_t fwd_workspace_bytes, void* workspace,
                   size_t workspace_bytes, int B, int H, int N, int dk, int dv, int chunk, int dtype,
                   float eps, void* hip_stream) {
  const void* req[] = {Q, K, V, s, dO, dQ, dK, dV, ds};
  int st = check_common(req, 9, B, H, N, dk, dv, dtype, eps);
  if (st != COTTN_OK) return st;
  if ((st = check_lengths(seq_len)) != COTTN_OK) return st;
  if (!is_aligned(state_in, 16) || !is_aligned(rev_state_in, 16) || !is_aligned(rev_state_out, 16))
    return COTTN_E_ALIGN;
  // workgroups read the one while others write the other
  if (rev_state_out != nullptr && rev_state_out == rev_state_in) return COTTN_E_ARG;
  SeqPlan plan;
  if (!make_plan(COTTN_OP_BWD_CAUSAL, B, H, N, dk, dv, chunk, dtype, &plan)) return COTTN_E_SHAPE;
  st = check_workspace(workspace, workspace_bytes,
                       workspace_bytes_for(COTTN_OP_BWD_CAUSAL, B, H, dk, dv, plan));
  if (st != COTTN_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (N == 0) {
    const long n = long(B) * H * dk * dv;
    hipError_t e = zero_f32(ds, seq_len != nullptr ? long(B) * H : H, stream);
    if (e == hipSuccess && rev_state_out != nullptr)
      e = rev_state_in != nullptr ? copy_state(rev_state_out, rev_state_in, n, stream)
                                  : zero_f32(rev_state_out, n, stream);
    return map_hip(e);
  }
  CausalArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.s = s; a.dO = dO; a.dQ = dQ; a.dK = dK; a.dV = dV; a.ds = ds;
  a.state_in = state_in; a.rev_state_in = rev_state_in; a.rev_state_out = rev_state_out;
  a.workspace = workspace; a.seq_len = seq_len; a.s_per_unit = seq_len != nullptr;
  a.B = B; a.H = H; a.N = N; a.dk = dk; a.dv = dv; a.C = plan.C; a.G = plan.G; a.seg_rows = plan.seg_rows;
  a.eps = eps; a.stream = stream;
  // the forward's segment states are taken over only if the forward split the sequence as
  // the backward does
  if (fwd_workspace != nullptr && dtype != COTTN_F32 && plan.G > 1) {
    SeqPlan fwd_plan;
    if (make_plan(COTTN_OP_FWD_CAUSAL, B, H, N, dk, dv, chunk, dtype, &fwd_plan) &&
        fwd_plan.C == plan.C && fwd_plan.G == plan.G && fwd_plan.seg_rows == plan.seg_rows) {
      st = check_workspace(fwd_workspace, fwd_workspace_bytes,
                           workspace_bytes_for(COTTN_OP_FWD_CAUSAL, B, H, dk, dv, fwd_plan));
      if (st != COTTN_OK) return st;
      a.saved_fwd_states = static_cast<const float*>(fwd_workspace);
    }
  }
  return map_hip(dtype == COTTN_BF16 ? bwd_causal_bf16(a) : dtype == COTTN_F16 ? bwd_causal_f16(a) : bwd_causal_f32(a));
}

int fwd_bidir_any(const void* Q, const void* K, const void* V, const float* s, const int* seq_len,
                  void* O, float* state, void* workspace, size_t workspace_bytes, int B, int H,
                  int N, int dk, int dv, int dtype, float eps, void* hip_stream) {
  const void* req[] = {Q, K, V, s, O};
  int st = check_common(req, 5, B, H, N, dk, dv, dtype, eps);
  if (st != COTTN_OK) return st;
  if (state != nullptr && !is_aligned(state, 16)) return COTTN_E_ALIGN;
  if ((st = check_lengths(seq_len)) != COTTN_OK) return st;
  SeqPlan plan;
  if (!make_plan(COTTN_OP_FWD_BIDIR, B, H, N, dk, dv, 0, dtype, &plan)) return COTTN_E_SHAPE;
  st = check_workspace(workspace, workspace_bytes,
                       workspace_bytes_for(COTTN_OP_FWD_BIDIR, B, H, dk, dv, plan));
  if (st != COTTN_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (N == 0) return map_hip(zero_f32(state, long(B) * H * dk * dv, stream));
  CausalArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.s = s; a.O = O; a.state = state; a.workspace = workspace;
  a.seq_len = seq_len; a.s_per_unit = seq_len != nullptr;
  a.B = B; a.H = H; a.N = N; a.dk = dk; a.dv = dv; a.C = plan.C; a.G = plan.G; a.seg_rows = plan.seg_rows;
  a.eps = eps; a.stream = stream;
  return map_hip(dtype == COTTN_BF16 ? fwd_bidir_bf16(a) : dtype == COTTN_F16 ? fwd_bidir_f16(a) : fwd_bidir_f32(a));
}

int bwd_bidir_any(const void* Q, const void* K, const void* V, const float* s, const int* seq_len,
                  const void* dO, void* dQ, void* dK, void* dV, float* ds,
                  const void* fwd_workspace, size_t fwd_workspace_bytes, void* workspace,
                  size_t workspace_bytes, int B, int H, int N, int dk, int dv, int dtype, float eps,
                  void* hip_stream) {
  const void* req[] = {Q, K, V, s, dO, dQ, dK, dV, ds};
  int st = check_common(req, 9, B, H, N, dk, dv, dtype, eps);
  if (st != COTTN_OK) return st;
  if ((st = check_lengths(seq_len)) != COTTN_OK) return st;
  SeqPlan plan;
  if (!make_plan(COTTN_OP_BWD_BIDIR, B, H, N, dk, dv, 0, dtype, &plan)) return COTTN_E_SHAPE;
  st = check_workspace(workspace, workspace_bytes,
                       workspace_bytes_for(COTTN_OP_BWD_BIDIR, B, H, dk, dv, plan));
  if (st != COTTN_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (N == 0) return map_hip(zero_f32(ds, seq_len != nullptr ? long(B) * H : H, stream));
  CausalArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.s = s; a.dO = dO; a.dQ = dQ; a.dK = dK; a.dV = dV; a.ds = ds;
  a.workspace = workspace; a.seq_len = seq_len; a.s_per_unit = seq_len != nullptr;
  a.B = B; a.H = H; a.N = N; a.dk = dk; a.dv = dv; a.C = plan.C; a.G = plan.G; a.seg_rows = plan.seg_rows;
  a.eps = eps; a.stream = stream;
  if (fwd_workspace != nullptr && dtype != COTTN_F32 && plan.G <= kMaxSegmentsSummedInScan) {
    SeqPlan fwd_plan;
    if (make_plan(COTTN_OP_FWD_BIDIR, B, H, N, dk, dv, 0, dtype, &fwd_plan) && fwd_plan.C == plan.C &&
        fwd_plan.G == plan.G && fwd_plan.seg_rows == plan.seg_rows) {
      st = check_workspace(fwd_workspace, fwd_workspace_bytes,
                           workspace_bytes_for(COTTN_OP_FWD_BIDIR, B, H, dk, dv, fwd_plan));
      if (st != COTTN_OK) return st;
      a.saved_fwd_states = static_cast<const float*>(fwd_workspace);
    }
  }
  return map_hip(dtype == COTTN_BF16 ? bwd_bidir_bf16(a) : dtype == COTTN_F16 ? bwd_bidir_f16(a) : bwd_bidir_f32(a));
}

}  // namespace

int cottn_bwd_causal(const void* Q, const void* K, const void* V, const float* s, const void* dO,
                     void* dQ, void* dK, void* dV, float* ds, const void* fwd_workspace,
                     size_t fwd_workspace_bytes, void* workspace, size_t workspace_bytes, int B,
                     int H, int N, int d, int chunk, int dtype, float eps, void* hip_stream) {
  return bwd_causal_any(Q, K, V, s, nullptr, dO, nullptr, nullptr, dQ, dK, dV, ds, nullptr,
                        fwd_workspace, fwd_workspace_bytes,
                        workspace, workspace_bytes, B, H, N, d, d, chunk, dtype, eps, hip_stream);
}

int cottn_bwd_causal_from_state(const void* Q, const void* K, const void* V, const float* s,
                                const void* dO, const float* state_in, const float* rev_state_in,
                                void* dQ, void* dK, void* dV, float* ds, float* rev_state_out,
                                const void* fwd_workspace, size_t fwd_workspace_bytes,
                                void* workspace, size_t workspace_bytes, int B, int H, int N, int d,
                                int chunk, int dtype, float eps, void* hip_stream) {
  return bwd_causal_any(Q, K, V, s, nullptr, dO, state_in, rev_state_in, dQ, dK, dV, ds,
                        rev_state_out, fwd_workspace, fwd_workspace_bytes, workspace,
                        workspace_bytes, B, H, N, d, d, chunk, dtype, eps, hip_stream);
}

int cottn_fwd_bidir(const void* Q, const void* K, const void* V, const float* s, void* O,
                    float* state, void* workspace, size_t workspace_bytes, int B, int H, int N,
                    int d, int dtype, float eps, void* hip_stream) {
  return fwd_bidir_any(Q, K, V, s, nullptr, O, state, workspace, workspace_bytes, B, H, N, d, d, dtype,
                       eps, hip_stream);
}

int cottn_bwd_bidir(const void* Q, const void* K, const void* V, const float* s, const void* dO,
                    void* dQ, void* dK, void* dV, float* ds, const void* fwd_workspace,
                    size_t fwd_workspace_bytes, void* workspace, size_t workspace_bytes, int B,
                    int H, int N, int d, int dtype, float eps, void* hip_stream) {
  return bwd_bidir_any(Q, K, V, s, nullptr, dO, dQ, dK, dV, ds, fwd_workspace, fwd_workspace_bytes,
                       workspace, workspace_bytes, B, H, N, d, d, dtype, eps, hip_stream);
}

// ---- padded batches: seq_len[B] rows exist per sequence; s and ds are [B][H] -------------------
int cottn_fwd_causal_varlen(const void* Q, const void* K, const void* V, const float* s,
                            const int* seq_len, void* O, float* state, void* workspace,
                            size_t workspace_bytes, int B, int H, int N, int d, int chunk,
                            int dtype, float eps, void* hip_stream) {
  if (seq_len == nullptr) return COTTN_E_NULL;
  return fwd_causal_any(Q, K, V, s, seq_len, nullptr, O, state, workspace, workspace_bytes, B, H, N,
                        d, d, chunk, dtype, eps, hip_stream);
}

int cottn_bwd_causal_varlen(const void* Q, const void* K, const void* V, const float* s,
                            const int* seq_len, const void* dO, void* dQ, void* dK, void* dV,
                            float* ds, const void* fwd_workspace, size_t fwd_workspace_bytes,
                            void* workspace, size_t workspace_bytes, int B, int H, int N, int d,
                            int chunk, int dtype, float eps, void* hip_stream) {
  if (seq_len == nullptr) return COTTN_E_NULL;
  return bwd_causal_any(Q, K, V, s, seq_len, dO, nullptr, nullptr, dQ, dK, dV, ds, nullptr,
                        fwd_workspace, fwd_workspace_bytes,
                        workspace, workspace_bytes, B, H, N, d, d, chunk, dtype, eps, hip_stream);
}

int cottn_fwd_bidir_varlen(const void* Q, const void* K, const void* V, const float* s,
                           const int* seq_len, void* O, float* state, void* workspace,
                           size_t workspace_bytes, int B, int H, int N, int d, int dtype, float eps,
                           void* hip_stream) {
  if (seq_len == nullptr) return COTTN_E_NULL;
  return fwd_bidir_any(Q, K, V, s, seq_len, O, state, workspace, workspace_bytes, B, H, N, d, d, dtype,
                       eps, hip_stream);
}

int cottn_bwd_bidir_varlen(const void* Q, const void* K, const void* V, const float* s,
                           const int* seq_len, const void* dO, void* dQ, void* dK, void* dV,
                           float* ds, const void* fwd_workspace, size_t fwd_workspace_bytes,
                           void* workspace, size_t workspace_bytes, int B, int H, int N, int d,
                           int dtype, float eps, void* hip_stream) {
  if (seq_len == nullptr) return COTTN_E_NULL;
  return bwd_bidir_any(Q, K, V, s, seq_len, dO, dQ, dK, dV, ds, fwd_workspace, fwd_workspace_bytes,
                       workspace, workspace_bytes, B, H, N, d, d, dtype, eps, hip_stream);
}

int cottn_scale_from_m(const float* m, float* s, int H, float n, void* hip_stream) {
  if (m == nullptr || s == nullptr) return COTTN_E_NULL;
  if (H < 1) return COTTN_E_SHAPE;
  if (!(n >= 1.0f) || !(n <= 3.0e38f)) return COTTN_E_ARG;
  if (!is_aligned(m, 4) || !is_aligned(s, 4)) return COTTN_E_ALIGN;
  return map_hip(launch_scale_from_m(m, s, H, n, static_cast<hipStream_t>(hip_stream)));
}

int cottn_scale_backward(const float* m, const float* ds, float* dm, int H, float n,
                         void* hip_stream) {
  if (m == nullptr || ds == nullptr || dm == nullptr) return COTTN_E_NULL;
  if (H < 1) return COTTN_E_SHAPE;
  if (!(n >= 1.0f) || !(n <= 3.0e38f)) return COTTN_E_ARG;
  if (!is_aligned(m, 4) || !is_aligned(ds, 4) || !is_aligned(dm, 4)) return COTTN_E_ALIGN;
  return map_hip(launch_scale_backward(m, ds, dm, H, n, static_cast<hipStream_t>(hip_stream)));
}

int cottn_scale_from_m_varlen(const float* m, const int* seq_len, float* s, int B, int H,
                              void* hip_stream) {
  if (m == nullptr || seq_len == nullptr || s == nullptr) return COTTN_E_NULL;
  if (B < 1 || H < 1 || double(B) * H > 16777216.0) return COTTN_E_SHAPE;
  if (!is_aligned(m, 4) || !is_aligned(seq_len, 4) || !is_aligned(s, 4)) return COTTN_E_ALIGN;
  return map_hip(launch_scale_from_m_varlen(m, seq_len, s, B, H,
                                            static_cast<hipStream_t>(hip_stream)));
}

int cottn_scale_backward_varlen(const float* m, const int* seq_len, const float* ds, float* dm,
                                int B, int H, void* hip_stream) {
  if (m == nullptr || seq_len == nullptr || ds == nullptr || dm == nullptr) return COTTN_E_NULL;
  if (B < 1 || H < 1 || double(B) * H > 16777216.0) return COTTN_E_SHAPE;
  if (!is_aligned(m, 4) || !is_aligned(seq_len, 4) || !is_aligned(ds, 4) || !is_aligned(dm, 4))
    return COTTN_E_ALIGN;
  return map_hip(launch_scale_backward_varlen(m, seq_len, ds, dm, B, H,
                                              static_cast<hipStream_t>(hip_stream)));
}

int cottn_step_dkdv(const void* q, const void* k, const void* v, const float* s, float* state,
                    void* o, int B, int H, int dk, int dv, int dtype, float eps, void* hip_stream) {
  const void* req[] = {q, k, v, s, state, o};
  int st = check_common(req, 6, B, H, 1, dk, dv, dtype, eps);
  if (st != COTTN_OK) return st;
  StepArgs a{q, k, v, s, state, o, B, H, dk, dv, eps, static_cast<hipStream_t>(hip_stream)};
  return map_hip(step_any(a, dtype));
}

int cottn_step(const void* q, const void* k, const void* v, const float* s, float* state,
               void* o, int B, int H, int d, int dtype, float eps, void* hip_stream) {
  return cottn_step_dkdv(q, k, v, s, state, o, B, H, d, d, dtype, eps, hip_stream);
}

// ---- d_key != d_value (Sec. 2.1): Q, K, dQ, dK are [B][H][N][dk]; V, O, dO, dV [B][H][N][dv] ----
int cottn_fwd_causal_dkdv(const void* Q, const void* K, const void* V, const float* s, void* O,
                          float* state, void* workspace, size_t workspace_bytes, int B, int H,
                          int N, int dk, int dv, int chunk, int dtype, float eps, void* hip_stream) {
  return fwd_causal_any(Q, K, V, s, nullptr, nullptr, O, state, workspace, workspace_bytes, B, H, N,
                        dk, dv, chunk, dtype, eps, hip_stream);
}

int cottn_bwd_causal_dkdv(const void* Q, const void* K, const void* V, const float* s,
                          const void* dO, void* dQ, void* dK, void* dV, float* ds,
                          const void* fwd_workspace, size_t fwd_workspace_bytes, void* workspace,
                          size_t workspace_bytes, int B, int H, int N, int dk, int dv, int chunk,
                          int dtype, float eps, void* hip_stream) {
  return bwd_causal_any(Q, K, V, s, nullptr, dO, nullptr, nullptr, dQ, dK, dV, ds, nullptr,
                        fwd_workspace, fwd_workspace_bytes, workspace, workspace_bytes, B, H, N, dk,
                        dv, chunk, dtype, eps, hip_stream);
}

int cottn_fwd_bidir_dkdv(const void* Q, const void* K, const void* V, const float* s, void* O,
                         float* state, void* workspace, size_t workspace_bytes, int B, int H, int N,
                         int dk, int dv, int dtype, float eps, void* hip_stream) {
  return fwd_bidir_any(Q, K, V, s, nullptr, O, state, workspace, workspace_bytes, B, H, N, dk, dv,
                       dtype, eps, hip_stream);
}

int cottn_bwd_bidir_dkdv(const void* Q, const void* K, const void* V, const float* s,
                         const void* dO, void* dQ, void* dK, void* dV, float* ds,
                         const void* fwd_workspace, size_t fwd_workspace_bytes, void* workspace,
                         size_t workspace_bytes, int B, int H, int N, int dk, int dv, int dtype,
                         float eps, void* hip_stream) {
  return bwd_bidir_any(Q, K, V, s, nullptr, dO, dQ, dK, dV, ds, fwd_workspace, fwd_workspace_bytes,
                       workspace, workspace_bytes, B, H, N, dk, dv, dtype, eps, hip_stream);
}

int cottn_profile_start(void) {
  g_pending.clear();
  g_totals.clear();
  g_profile_on = true;
  return COTTN_OK;
}

int cottn_profile_stop(void) {
  g_profile_on = false;
  int status = COTTN_OK;
  for (const PendingSpan& sp : g_pending) {
    float ms = 0.f;
    if (sp.end == nullptr || hipEventSynchronize(sp.end) != hipSuccess ||
        hipEventElapsedTime(&ms, sp.begin, sp.end) != hipSuccess) {
      status = COTTN_E_HIP;
    } else {
      KernelTotal* slot = nullptr;
      for (KernelTotal& t : g_totals)
        if (std::strcmp(t.name, sp.name) == 0) slot = &t;
      if (slot == nullptr) {
        g_totals.push_back(KernelTotal{sp.name, 0, 0.0});
        slot = &g_totals.back();
      }
      slot->launches += 1;
      slot->ms += ms;
    }
    if (sp.begin) (void)hipEventDestroy(sp.begin);
    if (sp.end) (void)hipEventDestroy(sp.end);
  }
  g_pending.clear();
  return status;
}

int cottn_profile_count(void) { return int(g_totals.size()); }
const char* cottn_profile_name(int i) {
  return (i >= 0 && i < int(g_totals.size())) ? g_totals[i].name : "";
}
long cottn_profile_launches(int i) {
  return (i >= 0 && i < int(g_totals.size())) ? g_totals[i].launches : 0;
}
double cottn_profile_ms(int i) {
  return (i >= 0 && i < int(g_totals.size())) ? g_totals[i].ms : 0.0;
}

}  // extern "C"
