// Exceptional inputs (Section 3.1, closing remark): infinities and NaNs in A or B are detected in stage 1 (the row /
// column maxima are taken on bit patterns, where every non-finite value compares above every finite one) and the
// whole update C := alpha * op(A) * op(B) + beta * C is then formed in ordinary FP64 arithmetic (the tile routine
// of oz2_fallback_tile.h).  The kernel below is launched after stage 3 of a checked call and returns at once when
// the flag is clear, so the decision needs no device-to-host synchronisation; small problems carry its blocks in
// the launch of stage 3 instead.
#include "oz2_fallback_tile.h"
#include "oz2_internal.h"

namespace {

constexpr int kThreads = kFallbackThreads;

__global__ void __launch_bounds__(kThreads) copy_if_kernel(const unsigned long long* __restrict__ flag, int64_t m,
                                                           const double* __restrict__ src, double* __restrict__ dst,
                                                           int64_t ld) {
  if (*flag == 0ull) return;
  const int64_t i = (int64_t)blockIdx.y * kThreads + threadIdx.x, j = blockIdx.x;
  if (i < m) dst[i + j * ld] = src[i + j * m];
}

__global__ void __launch_bounds__(kThreads) fp64_fallback_kernel(const unsigned long long* __restrict__ flag,
                                                                 const Oz2FallbackArgs f) {
  if (*flag == 0ull) return;
  oz2_fallback_tile(f, (int64_t)blockIdx.x);
}

}  // namespace

hipError_t oz2_launch_fallback(const unsigned long long* flag, int transa, int transb, int64_t m, int64_t n, int64_t k,
                               double alpha, const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
                               double* C, int64_t ldc, int triangle, int tri_a, int tri_b, hipStream_t st) {
  const int64_t tiles_m = (m + kFallbackTile - 1) / kFallbackTile, tiles_n = (n + kFallbackTile - 1) / kFallbackTile;
  if (tiles_m * tiles_n >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
  const Oz2FallbackArgs f = {transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, tiles_m, triangle, tri_a, tri_b};
  hipLaunchKernelGGL(fp64_fallback_kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), 0, st, flag, f);
  return hipGetLastError();
}

hipError_t oz2_launch_copy_if(const unsigned long long* flag, int64_t m, int64_t n, const double* src, double* dst,
                              int64_t ld, hipStream_t st) {
  dim3 grid((unsigned)n, (unsigned)((m + kThreads - 1) / kThreads));
  hipLaunchKernelGGL(copy_if_kernel, grid, dim3(kThreads), 0, st, flag, m, src, dst, ld);
  return hipGetLastError();
}
