// Probe, not part of the library: what each LDS access pattern of the kernels costs on gfx950
// as a function of the row pitch.  16 waves of one workgroup issue the same LDS instruction
// (the exact instruction is forced with inline asm) with the address pattern under test; the
// program prints cycles per wave instruction.  Its table is where the two row pitches in
// device_common.h come from.
//   hipcc --offload-arch=gfx950 -O3 -o lds_access_patterns lds_access_patterns.hip && ./lds_access_patterns
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
#define LDS __attribute__((address_space(3)))

enum { RD128, RD64, RD64TR, RD32, WR128, WR64 };

template <int OP>
__device__ __forceinline__ unsigned op8(unsigned a, unsigned seed) {
  unsigned acc = 0;
  if (OP == RD128) {
    u32x4 v0, v1, v2, v3, v4, v5, v6, v7;
    asm volatile(
        "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:4096\n ds_read_b128 %2, %8 offset:8192\n"
        "ds_read_b128 %3, %8 offset:12288\n ds_read_b128 %4, %8 offset:16384\n"
        "ds_read_b128 %5, %8 offset:20480\n ds_read_b128 %6, %8 offset:24576\n"
        "ds_read_b128 %7, %8 offset:28672\n s_waitcnt lgkmcnt(0)"
        : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
        : "v"(a));
    acc = v0.x ^ v1.x ^ v2.x ^ v3.x ^ v4.x ^ v5.x ^ v6.x ^ v7.x;
  } else if (OP == RD64 || OP == RD64TR) {
    u32x2 v0, v1, v2, v3, v4, v5, v6, v7;
    if (OP == RD64)
      asm volatile(
          "ds_read_b64 %0, %8\n ds_read_b64 %1, %8 offset:4096\n ds_read_b64 %2, %8 offset:8192\n"
          "ds_read_b64 %3, %8 offset:12288\n ds_read_b64 %4, %8 offset:16384\n"
          "ds_read_b64 %5, %8 offset:20480\n ds_read_b64 %6, %8 offset:24576\n"
          "ds_read_b64 %7, %8 offset:28672\n s_waitcnt lgkmcnt(0)"
          : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
          : "v"(a));
    else
      asm volatile(
          "ds_read_b64_tr_b16 %0, %8\n ds_read_b64_tr_b16 %1, %8 offset:4096\n"
          "ds_read_b64_tr_b16 %2, %8 offset:8192\n ds_read_b64_tr_b16 %3, %8 offset:12288\n"
          "ds_read_b64_tr_b16 %4, %8 offset:16384\n ds_read_b64_tr_b16 %5, %8 offset:20480\n"
          "ds_read_b64_tr_b16 %6, %8 offset:24576\n ds_read_b64_tr_b16 %7, %8 offset:28672\n"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
          : "v"(a));
    acc = v0.x ^ v1.x ^ v2.x ^ v3.x ^ v4.x ^ v5.x ^ v6.x ^ v7.x;
  } else if (OP == RD32) {
    unsigned v0, v1, v2, v3, v4, v5, v6, v7;
    asm volatile(
        "ds_read_b32 %0, %8\n ds_read_b32 %1, %8 offset:4096\n ds_read_b32 %2, %8 offset:8192\n"
        "ds_read_b32 %3, %8 offset:12288\n ds_read_b32 %4, %8 offset:16384\n"
        "ds_read_b32 %5, %8 offset:20480\n ds_read_b32 %6, %8 offset:24576\n"
        "ds_read_b32 %7, %8 offset:28672\n s_waitcnt lgkmcnt(0)"
        : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
        : "v"(a));
    acc = v0 ^ v1 ^ v2 ^ v3 ^ v4 ^ v5 ^ v6 ^ v7;
  } else if (OP == WR128) {
    u32x4 d = {seed, seed + 1, seed + 2, seed + 3};
    asm volatile(
        "ds_write_b128 %0, %1\n ds_write_b128 %0, %1 offset:4096\n ds_write_b128 %0, %1 offset:8192\n"
        "ds_write_b128 %0, %1 offset:12288\n ds_write_b128 %0, %1 offset:16384\n"
        "ds_write_b128 %0, %1 offset:20480\n ds_write_b128 %0, %1 offset:24576\n"
        "ds_write_b128 %0, %1 offset:28672\n s_waitcnt lgkmcnt(0)" ::"v"(a), "v"(d)
        : "memory");
  } else {
    u32x2 d = {seed, seed + 1};
    asm volatile(
        "ds_write_b64 %0, %1\n ds_write_b64 %0, %1 offset:4096\n ds_write_b64 %0, %1 offset:8192\n"
        "ds_write_b64 %0, %1 offset:12288\n ds_write_b64 %0, %1 offset:16384\n"
        "ds_write_b64 %0, %1 offset:20480\n ds_write_b64 %0, %1 offset:24576\n"
        "ds_write_b64 %0, %1 offset:28672\n s_waitcnt lgkmcnt(0)" ::"v"(a), "v"(d)
        : "memory");
  }
  return acc;
}

// byte address of this lane for pattern PAT with row pitch `pe` (elements of 2 bytes)
__device__ __forceinline__ unsigned lane_addr(int pat, int pe, int l) {
  const int r = l % 16, q4 = l / 16;
  int e;
  switch (pat) {
    case 0: e = r * pe + 8 * q4; break;                      // row fragment (b128): rows r, 8 q4
    case 1: e = (8 * q4 + r / 4) * pe + 4 * (r % 4); break;  // col fragment of a state (b64_tr)
    case 2: e = (4 * q4 + r / 4) * pe + 4 * (r % 4); break;  // col fragment over tokens (b64_tr)
    case 3: e = r * pe + 4 * q4; break;                      // 4 columns of row r (b64): publish, staging, chain rule
    case 4: e = (l / 8) * pe + (l % 8) * 8; break;           // 16-byte pieces of rows, 8 per row (b128): commit, gather
    case 5: e = (l / 4) * pe + (l % 4) * 8; break;           // the same with 4 pieces per row (d = 32)
    case 6: e = (l / 16) * pe + (l % 16) * 8; break;         // 16 pieces per row (d = 128)
    default: e = 0;
  }
  return unsigned(e) * 2u;
}

template <int OP>
__global__ __launch_bounds__(1024) void k(int pat, int pe, int iters, int consecutive, long* cycles,
                                          unsigned* sink) {
  __shared__ __attribute__((aligned(16))) uint16_t buf[32768];
  for (int i = threadIdx.x; i < 32768; i += 1024) buf[i] = uint16_t(i * 7);
  __syncthreads();
  const int l = threadIdx.x % 64;
  const unsigned base = unsigned(uintptr_t((LDS uint16_t*)buf));
  const unsigned width = OP == RD128 || OP == WR128 ? 16 : OP == RD32 ? 4 : 8;
  const unsigned a = base + (consecutive ? l * width : lane_addr(pat, pe, l));
  unsigned acc = 0;
  __syncthreads();
  const long t0 = clock64();
  for (int it = 0; it < iters; ++it) acc ^= op8<OP>(a, acc + it);
  __syncthreads();
  const long t1 = clock64();
  if (threadIdx.x == 0) cycles[0] = t1 - t0;
  sink[threadIdx.x] = acc ^ buf[threadIdx.x * 3];
}

template <int OP>
double run(int pat, int pe, int consecutive, long* d_cycles, unsigned* d_sink) {
  const int iters = 1000;
  for (int rep = 0; rep < 2; ++rep)
    hipLaunchKernelGGL(k<OP>, dim3(1), dim3(1024), 0, 0, pat, pe, iters, consecutive, d_cycles, d_sink);
  long c = 0;
  if (hipMemcpy(&c, d_cycles, sizeof(long), hipMemcpyDeviceToHost) != hipSuccess) return -1;
  return double(c) / (double(iters) * 8 * 16);
}

int main() {
  long* d_cycles; unsigned* d_sink;
  if (hipMalloc(&d_cycles, sizeof(long)) != hipSuccess) return 1;
  if (hipMalloc(&d_sink, 1024 * sizeof(unsigned)) != hipSuccess) return 1;
  printf("cycles per wave instruction, 16 waves of one CU issuing together\n");
  printf("consecutive lanes: rd32 %.2f rd64 %.2f rd64tr %.2f rd128 %.2f wr64 %.2f wr128 %.2f\n",
         run<RD32>(0, 0, 1, d_cycles, d_sink), run<RD64>(0, 0, 1, d_cycles, d_sink),
         run<RD64TR>(0, 0, 1, d_cycles, d_sink), run<RD128>(0, 0, 1, d_cycles, d_sink),
         run<WR64>(0, 0, 1, d_cycles, d_sink), run<WR128>(0, 0, 1, d_cycles, d_sink));
  const int pitches[] = {40, 48, 72, 80, 88, 96, 104, 136, 144, 152};
  printf("%-34s", "pitch (elements)");
  for (int p : pitches) printf("%7d", p);
  printf("\n");
  struct Row { const char* name; int op; int pat; };
  const Row rows[] = {
      {"rd128 row fragment", RD128, 0}, {"rd64tr state col fragment", RD64TR, 1},
      {"rd64tr token col fragment", RD64TR, 2}, {"wr64 4 cols of row r", WR64, 3},
      {"rd64 4 cols of row r", RD64, 3}, {"wr128 row pieces (8/row)", WR128, 4},
      {"rd128 row pieces (8/row)", RD128, 4}, {"wr128 row pieces (4/row)", WR128, 5},
      {"wr128 row pieces (16/row)", WR128, 6}};
  for (const Row& row : rows) {
    printf("%-34s", row.name);
    for (int p : pitches) {
      double c = 0;
      switch (row.op) {
        case RD128: c = run<RD128>(row.pat, p, 0, d_cycles, d_sink); break;
        case RD64: c = run<RD64>(row.pat, p, 0, d_cycles, d_sink); break;
        case RD64TR: c = run<RD64TR>(row.pat, p, 0, d_cycles, d_sink); break;
        case WR128: c = run<WR128>(row.pat, p, 0, d_cycles, d_sink); break;
        case WR64: c = run<WR64>(row.pat, p, 0, d_cycles, d_sink); break;
      }
      printf("%7.2f", c);
    }
    printf("\n");
    fflush(stdout);
  }
  return hipDeviceSynchronize() == hipSuccess ? 0 : 1;
}
