// One 128 x 128 tile of C := alpha * op(A) * op(B) + beta * C in plain FP64 arithmetic, as device code shared by the
// fallback kernel and by the small-problem kernel of stage 3 that carries the fallback's blocks in its own launch.
// Exceptional inputs (Section 3.1, closing remark): the emulation reproduces FP64 products of finite matrices only,
// so infinities and NaNs in A or B are detected in stage 1 and the whole update is then formed here, which
// propagates them by the IEEE rules.  A plain LDS-tiled loop (8 x 8 outputs per thread, the inner dimension in
// ascending order with one fused multiply-add per term), not tuned: it only runs for inputs the method does not
// cover.
#ifndef OZ2_FALLBACK_TILE_H_
#define OZ2_FALLBACK_TILE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

constexpr int kFallbackThreads = 256;
constexpr int kFallbackTile = 128;  // tile of C
constexpr int kFallbackStep = 8;    // inner-dimension step

struct Oz2FallbackArgs {
  int transa, transb;
  int64_t m, n, k;
  double alpha;
  const double* A;
  int64_t lda;
  const double* B;
  int64_t ldb;
  double beta;
  double* C;
  int64_t ldc;
  int64_t tiles_m;         // tiles along the rows of C; tile index = tile row + tiles_m * tile column
  int triangle;            // of C: 0 full, 1 lower, 2 upper
  int tri_a, tri_b;        // triangular structure of the stored A / B (0 = full)
};

// element of a triangular operand: (r, c) = row and column in the stored array; tri & 3: 0 full, 1 lower,
// 2 upper; tri & 4: unit diagonal; what is not stored counts as zero and is never propagated
__device__ __forceinline__ double oz2_tri_value(double v, int64_t r, int64_t c, int tri) {
  if (tri == 0) return v;
  if (r == c) return (tri & 4) ? 1.0 : v;
  const bool stored = (tri & 3) == 1 ? r > c : r < c;
  return stored ? v : 0.0;
}

// all kFallbackThreads threads of the block call this with the same tile
__device__ __forceinline__ void oz2_fallback_tile(const Oz2FallbackArgs& f, int64_t tile) {
  constexpr int FT = kFallbackTile, FK = kFallbackStep;
  const int64_t ti = tile % f.tiles_m, tj = tile / f.tiles_m;
  // symmetric update: tiles wholly outside the lower (1) / upper (2) triangle have nothing to write
  if ((f.triangle == 1 && ti < tj) || (f.triangle == 2 && ti > tj)) return;
  __shared__ double As[FK][FT];
  __shared__ double Bs[FK][FT];
  const int64_t i0 = ti * FT, j0 = tj * FT;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  double acc[8][8];
#pragma unroll
  for (int r = 0; r < 8; ++r)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[r][c] = 0.0;
  for (int64_t l0 = 0; l0 < f.k; l0 += FK) {
    // 128 x 8 elements of op(A) and of op(B): four each per thread; out-of-range elements are zero
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int e = threadIdx.x + q * kFallbackThreads;
      int ii, ll;
      if (f.transa) { ll = e % FK; ii = e / FK; } else { ii = e % FT; ll = e / FT; }
      const int64_t i = i0 + ii, l = l0 + ll;
      As[ll][ii] = (i < f.m && l < f.k) ? (f.transa ? oz2_tri_value(f.A[l + i * f.lda], l, i, f.tri_a)
                                                    : oz2_tri_value(f.A[i + l * f.lda], i, l, f.tri_a))
                                        : 0.0;
      int jj, lb;
      if (f.transb) { jj = e % FT; lb = e / FT; } else { lb = e % FK; jj = e / FK; }
      const int64_t j = j0 + jj, lq = l0 + lb;
      Bs[lb][jj] = (j < f.n && lq < f.k) ? (f.transb ? oz2_tri_value(f.B[j + lq * f.ldb], j, lq, f.tri_b)
                                                     : oz2_tri_value(f.B[lq + j * f.ldb], lq, j, f.tri_b))
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
    if (j >= f.n) continue;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int64_t i = i0 + tx + 16 * r;
      if (i >= f.m || (f.triangle == 1 && i < j) || (f.triangle == 2 && i > j)) continue;
      double* dst = f.C + i + j * f.ldc;
      const double t = f.beta == 0.0 ? 0.0 : f.beta * *dst;  // C is not read when beta is zero
      *dst = fma(f.alpha, acc[r][c], t);
    }
  }
}

#endif
