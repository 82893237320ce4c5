// Probe, not part of the library: the HBM bandwidth a streaming kernel reaches on this machine
// (read-only, write-only, copy; plain and non-temporal accesses; by workgroup count; each
// workgroup walks a contiguous slice of 1 GiB buffers).  The copy rate it prints is the
// practical ceiling the scan kernels are compared with.
//   hipcc --offload-arch=gfx950 -O3 -o hbm_streaming hbm_streaming.hip && ./hbm_streaming
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

template <int MODE, bool NT>
__global__ __launch_bounds__(256) void k(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                         size_t n_vec, unsigned* sink) {
  const size_t per_wg = n_vec / gridDim.x;
  const size_t base = per_wg * blockIdx.x;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = threadIdx.x; i + 3 * 256 < per_wg; i += 4 * 256) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (MODE != 1) v[u] = NT ? __builtin_nontemporal_load(src + base + i + u * 256) : src[base + i + u * 256];
      else v[u] = u32x4{unsigned(i), 1u, 2u, 3u};
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (MODE == 0) acc ^= v[u];
      else if (NT) __builtin_nontemporal_store(v[u], dst + base + i + u * 256);
      else dst[base + i + u * 256] = v[u];
    }
  }
  if (MODE == 0 && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = 1;
}

template <int MODE, bool NT>
double run(const u32x4* src, u32x4* dst, size_t bytes, int wgs, unsigned* sink) {
  hipEvent_t e0, e1;
  hipEventCreate(&e0); hipEventCreate(&e1);
  const size_t n_vec = bytes / 16;
  for (int i = 0; i < 2; ++i) hipLaunchKernelGGL((k<MODE, NT>), dim3(wgs), dim3(256), 0, 0, src, dst, n_vec, sink);
  hipEventRecord(e0);
  const int reps = 10;
  for (int i = 0; i < reps; ++i) hipLaunchKernelGGL((k<MODE, NT>), dim3(wgs), dim3(256), 0, 0, src, dst, n_vec, sink);
  hipEventRecord(e1);
  hipEventSynchronize(e1);
  float ms = 0;
  hipEventElapsedTime(&ms, e0, e1);
  hipEventDestroy(e0); hipEventDestroy(e1);
  const double moved = double(bytes) * (MODE == 2 ? 2 : 1);
  return moved * reps / (ms * 1e-3) / 1e12;
}

int main() {
  const size_t bytes = size_t(1) << 30;  // 1 GiB per buffer: beyond the 256 MB last-level cache
  u32x4 *src, *dst; unsigned* sink;
  if (hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&dst, bytes) != hipSuccess) return 1;
  hipMalloc(&sink, 4);
  hipMemset(src, 1, bytes); hipMemset(dst, 2, bytes);
  printf("TB/s by workgroups of 256 threads (1 GiB buffers; copy counts read + write)\n");
  printf("%-22s", "workgroups");
  const int wgs[] = {256, 512, 1024, 2048, 4096, 16384};
  for (int w : wgs) printf("%8d", w);
  printf("\n");
  printf("%-22s", "read plain"); for (int w : wgs) printf("%8.2f", run<0, false>(src, dst, bytes, w, sink)); printf("\n");
  printf("%-22s", "read non-temporal"); for (int w : wgs) printf("%8.2f", run<0, true>(src, dst, bytes, w, sink)); printf("\n");
  printf("%-22s", "write plain"); for (int w : wgs) printf("%8.2f", run<1, false>(src, dst, bytes, w, sink)); printf("\n");
  printf("%-22s", "write non-temporal"); for (int w : wgs) printf("%8.2f", run<1, true>(src, dst, bytes, w, sink)); printf("\n");
  printf("%-22s", "copy plain"); for (int w : wgs) printf("%8.2f", run<2, false>(src, dst, bytes, w, sink)); printf("\n");
  printf("%-22s", "copy non-temporal"); for (int w : wgs) printf("%8.2f", run<2, true>(src, dst, bytes, w, sink)); printf("\n");
  fflush(stdout);
  return hipDeviceSynchronize() == hipSuccess ? 0 : 1;
}
