// Exceptional inputs (Section 3.1, closing remark): the emulation reproduces FP64 products of finite matrices
// only, so infinities and NaNs in A or B are detected in stage 1 (the row / column maxima are taken on bit
// patterns, where every non-finite value compares above every finite one) and the whole update
//   C := alpha * op(A) * op(B) + beta * C
// is then formed in ordinary FP64 arithmetic by the kernel below, which propagates them by the IEEE rules.
// The kernel is launched after stage 3 of every checked call and returns at once when the flag is clear, so
// the decision needs no device-to-host synchronisation.  It is a plain LDS-tiled FP64 kernel (128 x 128 tile,
// 8 x 8 outputs per thread), not tuned: it only runs for inputs the method does not cover.
#include "oz2_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int FT = 128;  // tile of C
constexpr int FK = 8;    // inner-dimension step

// element of a triangular operand: (r, c) = row and column in the stored array; tri & 3: 0 full, 1 lower,
// 2 upper; tri & 4: unit diagonal; what is not stored counts as zero and is never propagated
__device__ __forceinline__ double tri_value(double v, int64_t r, int64_t c, int tri) {
  if (tri == 0) return v;
  if (r == c) return (tri & 4) ? 1.0 : v;
  const bool stored = (tri & 3) == 1 ? r > c : r < c;
  return stored ? v : 0.0;
}

__global__ void __launch_bounds__(kThreads) copy_if_kernel(const unsigned long long* __restrict__ flag, int64_t m,
                                                           const double* __restrict__ src, double* __restrict__ dst,
                                                           int64_t ld) {
  if (*flag == 0ull) return;
  const int64_t i = (int64_t)blockIdx.y * kThreads + threadIdx.x, j = blockIdx.x;
  if (i < m) dst[i + j * ld] = src[i + j * m];
}

__global__ void __launch_bounds__(kThreads) fp64_fallback_kernel(const unsigned long long* __restrict__ flag, int transa,
                                                                 int transb, int64_t m, int64_t n, int64_t k, double alpha,
                                                                 const double* __restrict__ A, int64_t lda,
                                                                 const double* __restrict__ B, int64_t ldb, double beta,
                                                                 double* __restrict__ C, int64_t ldc, int64_t tiles_m,
                                                                 int triangle, int tri_a, int tri_b) {
  if (*flag == 0ull) return;
  // symmetric update: tiles wholly outside the lower (1) / upper (2) triangle have nothing to write
  if ((triangle == 1 && (int64_t)(blockIdx.x % tiles_m) < (int64_t)(blockIdx.x / tiles_m)) ||
      (triangle == 2 && (int64_t)(blockIdx.x % tiles_m) > (int64_t)(blockIdx.x / tiles_m)))
    return;
  __shared__ double As[FK][FT];
  __shared__ double Bs[FK][FT];
  const int64_t i0 = (int64_t)(blockIdx.x % tiles_m) * FT, j0 = (int64_t)(blockIdx.x / tiles_m) * FT;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  double acc[8][8];
#pragma unroll
  for (int r = 0; r < 8; ++r)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[r][c] = 0.0;
  for (int64_t l0 = 0; l0 < k; l0 += FK) {
    // 128 x 8 elements of op(A) and of op(B): four each per thread; out-of-range elements are zero
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int e = threadIdx.x + q * kThreads;
      int ii, ll;
      if (transa) { ll = e % FK; ii = e / FK; } else { ii = e % FT; ll = e / FT; }
      const int64_t i = i0 + ii, l = l0 + ll;
      As[ll][ii] = (i < m && l < k) ? (transa ? tri_value(A[l + i * lda], l, i, tri_a) : tri_value(A[i + l * lda], i, l, tri_a))
                                    : 0.0;
      int jj, lb;
      if (transb) { jj = e % FT; lb = e / FT; } else { lb = e % FK; jj = e / FK; }
      const int64_t j = j0 + jj, lq = l0 + lb;
      Bs[lb][jj] = (j < n && lq < k)
                       ? (transb ? tri_value(B[j + lq * ldb], j, lq, tri_b) : tri_value(B[lq + j * ldb], lq, j, tri_b))
                       : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int l = 0; l < FK; ++l) {
      double a[8], b[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) a[r] = As[l][tx + 16 * r];
#pragma unroll
      for (int c = 0; c < 8; ++c) b[c] = Bs[l][ty + 16 * c];
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[r][c] = fma(a[r], b[c], acc[r][c]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const int64_t j = j0 + ty + 16 * c;
    if (j >= n) continue;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int64_t i = i0 + tx + 16 * r;
      if (i >= m || (triangle == 1 && i < j) || (triangle == 2 && i > j)) continue;
      double* dst = C + i + j * ldc;
      const double t = beta == 0.0 ? 0.0 : beta * *dst;  // C is not read when beta is zero
      *dst = fma(alpha, acc[r][c], t);
    }
  }
}

}  // namespace

hipError_t oz2_launch_fallback(const unsigned long long* flag, int transa, int transb, int64_t m, int64_t n, int64_t k,
                               double alpha, const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
                               double* C, int64_t ldc, int triangle, int tri_a, int tri_b, hipStream_t st) {
  const int64_t tiles_m = (m + FT - 1) / FT, tiles_n = (n + FT - 1) / FT;
  if (tiles_m * tiles_n >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fp64_fallback_kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), 0, st, flag, transa, transb, m,
                     n, k, alpha, A, lda, B, ldb, beta, C, ldc, tiles_m, triangle, tri_a, tri_b);
  return hipGetLastError();
}

hipError_t oz2_launch_copy_if(const unsigned long long* flag, int64_t m, int64_t n, const double* src, double* dst,
                              int64_t ld, hipStream_t st) {
  dim3 grid((unsigned)n, (unsigned)((m + kThreads - 1) / kThreads));
  hipLaunchKernelGGL(copy_if_kernel, grid, dim3(kThreads), 0, st, flag, m, src, dst, ld);
  return hipGetLastError();
}
