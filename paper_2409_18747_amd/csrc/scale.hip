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

}  // namespace

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
