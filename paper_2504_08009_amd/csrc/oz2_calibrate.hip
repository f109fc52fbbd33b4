// MFMA-only calibration kernel: what the matrix cores of this card sustain for v_mfma_i32_32x32x32_i8
// with no memory traffic, with constant or with random INT8 operands (the card lowers its clock under a
// power cap, and operand bit toggling sets the power).  Measurement support for the benchmark; not part
// of the GEMM path.
#include "oz2_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(256) mfma_only_kernel(int iters, int random_operands, int* sink, long long* clocks) {
  unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  v4i a[2], b[2];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      h = h * 1664525u + 1013904223u;
      a[s][e] = random_operands ? (int)h : 0x01010101;
      h = h * 1664525u + 1013904223u;
      b[s][e] = random_operands ? (int)h : 0x01010101;
    }
  v16i acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0;
  long long c0 = clock64();
  long long w0 = wall_clock64();
  if (random_operands == 2) {
    // eight different fragments per operand, every MFMA with another pair: as in a product, where no operand
    // register is reused by the next instruction (the two-fragment loop below toggles fewer operand bits)
    v4i a8[8], b8[8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        h = h * 1664525u + 1013904223u;
        a8[s][e] = (int)h;
        h = h * 1664525u + 1013904223u;
        b8[s][e] = (int)h;
      }
    c0 = clock64();
    w0 = wall_clock64();
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i)
          acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a8[(i + u) & 7], b8[(i + 3 * u) & 7], acc[i], 0, 0, 0);
    }
  } else {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i & 1], b[(i >> 1) & 1], acc[i], 0, 0, 0);
    }
  }
  const long long c1 = clock64();
  const long long w1 = wall_clock64();
  int s = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    clocks[0] = c1 - c0;  // shader clock cycles
    clocks[1] = w1 - w0;  // constant 100 MHz counter
  }
}

}  // namespace

hipError_t oz2_launch_mfma_calibration(int workgroups, int iters, int random_operands, int* sink, long long* clocks,
                                       hipStream_t st) {
  hipLaunchKernelGGL(mfma_only_kernel, dim3((unsigned)workgroups), dim3(256), 0, st, iters, random_operands, sink,
                     clocks);
  return hipGetLastError();
}
