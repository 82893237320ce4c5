// The learned stabiliser of Sec. 3.3: the similarity scores are divided by n^sigma(m_h), with
// n the sequence length and m_h one learned scalar per head, so that the row sums (at most n)
// stay bounded while the model can choose anything between no scaling and division by n.
// The attention entry points take the resulting factor s_h = n^(-sigma(m_h)) as a number;
// these two kernels map m to s before the forward and ds back to dm after the backward:
//     s_h = exp(-sigma(m_h) ln n),     dm_h = ds_h * (-ln n) sigma(m_h) (1 - sigma(m_h)) s_h.
// H values each: one thread per head, fp32.
#include "device_common.h"
#include "launch.h"

namespace cottn {
namespace {

__device__ __forceinline__ float sigmoid(float x) { return 1.0f / (1.0f + __expf(-x)); }

__global__ __launch_bounds__(256) void scale_from_m_kernel(const float* __restrict__ m,
                                                           float* __restrict__ s, int H,
                                                           float ln_n) {
  const int h = blockIdx.x * 256 + threadIdx.x;
  if (h < H) s[h] = expf(-sigmoid(m[h]) * ln_n);
}

__global__ __launch_bounds__(256) void scale_backward_kernel(const float* __restrict__ m,
                                                             const float* __restrict__ ds,
                                                             float* __restrict__ dm, int H,
                                                             float ln_n) {
  const int h = blockIdx.x * 256 + threadIdx.x;
  if (h < H) {
    const float sg = sigmoid(m[h]);
    dm[h] = ds[h] * (-ln_n) * sg * (1.0f - sg) * expf(-sg * ln_n);
  }
}

// Padded batches: n is each sequence's own length, so s is [B][H] (a length below 1 counts as 1:
// an empty sequence has no rows the factor could apply to) and dm sums over the batch.
__global__ __launch_bounds__(256) void scale_from_m_varlen_kernel(const float* __restrict__ m,
                                                                  const int* __restrict__ seq_len,
                                                                  float* __restrict__ s, int B,
                                                                  int H) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < B * H) s[i] = expf(-sigmoid(m[i % H]) * logf(float(max(1, seq_len[i / H]))));
}

__global__ __launch_bounds__(256) void scale_backward_varlen_kernel(const float* __restrict__ m,
                                                                    const int* __restrict__ seq_len,
                                                                    const float* __restrict__ ds,
                                                                    float* __restrict__ dm, int B,
                                                                    int H) {
  const int h = blockIdx.x * 256 + threadIdx.x;
  if (h >= H) return;
  const float sg = sigmoid(m[h]);
  float acc = 0.f;
  for (int b = 0; b < B; ++b) {
    const float ln_n = logf(float(max(1, seq_len[b])));
    acc += ds[size_t(b) * H + h] * (-ln_n) * expf(-sg * ln_n);
  }
  dm[h] = acc * sg * (1.0f - sg);
}

}  // namespace

hipError_t launch_scale_from_m_varlen(const float* m, const int* seq_len, float* s, int B, int H,
                                      hipStream_t st) {
  return launch_kernel("scale_from_m_varlen_kernel", scale_from_m_varlen_kernel,
                       dim3((B * H + 255) / 256), dim3(256), 0, st, m, seq_len, s, B, H);
}

hipError_t launch_scale_backward_varlen(const float* m, const int* seq_len, const float* ds,
                                        float* dm, int B, int H, hipStream_t st) {
  return launch_kernel("scale_backward_varlen_kernel", scale_backward_varlen_kernel,
                       dim3((H + 255) / 256), dim3(256), 0, st, m, seq_len, ds, dm, B, H);
}

hipError_t launch_scale_from_m(const float* m, float* s, int H, float n, hipStream_t st) {
  return launch_kernel("scale_from_m_kernel", scale_from_m_kernel, dim3((H + 255) / 256), dim3(256),
                       0, st, m, s, H, logf(n));
}

hipError_t launch_scale_backward(const float* m, const float* ds, float* dm, int H, float n,
                                 hipStream_t st) {
  return launch_kernel("scale_backward_kernel", scale_backward_kernel, dim3((H + 255) / 256),
                       dim3(256), 0, st, m, ds, dm, H, logf(n));
}

}  // namespace cottn
