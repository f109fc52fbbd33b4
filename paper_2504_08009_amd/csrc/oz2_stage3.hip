// Stages 3 and 4 of Ozaki scheme II on gfx950: Algorithm 1 lines 7-11 fused in one pass.
//   per output element: c''_t = c'_t mod p_t (line 7), Y = sum_t c''_t W_t on 40-bit FP64 limbs (line 9),
//   X = Y mod M in the symmetric range (line 10), one rounding to FP64 and the exact power-of-two
//   scaling by 2^-(sa_i + sb_j) (line 11).
// 4N (INT32 planes) or N (UINT8 residue planes, line 7 already taken by the GEMM epilogue) bytes read and 8
// written per element: bound by HBM traffic with INT32 planes, by FP64 instruction issue with UINT8 planes.
#include "oz2_fallback_tile.h"
#include "oz2_math.h"

namespace {

constexpr int kThreads = 256;
static_assert(kThreads == kFallbackThreads, "the small-problem kernel runs both bodies with one block size");

// One plane's values for R consecutive rows: INT32 products (16-byte loads, R = 4) or UINT8 residues that
// the GEMM epilogue already reduced (8-byte loads, R = 8).
template <bool U8>
struct PlaneLoad;
template <>
struct PlaneLoad<false> {
  static constexpr int R = 4;
  typedef int Raw __attribute__((ext_vector_type(4)));
  static __device__ __forceinline__ void residues(const Raw& c, double p, double ip, double hip_, double* res) {
    res[0] = oz2_floor_mod(c.x, p, ip, hip_);
    res[1] = oz2_floor_mod(c.y, p, ip, hip_);
    res[2] = oz2_floor_mod(c.z, p, ip, hip_);
    res[3] = oz2_floor_mod(c.w, p, ip, hip_);
  }
};
template <>
struct PlaneLoad<true> {
  static constexpr int R = 8;
  typedef unsigned Raw __attribute__((ext_vector_type(2)));
  static __device__ __forceinline__ void residues(const Raw& c, double, double, double, double* res) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      res[r] = (double)((c.x >> (8 * r)) & 0xffu);
      res[4 + r] = (double)((c.y >> (8 * r)) & 0xffu);
    }
  }
};

// One thread: R consecutive rows i of one column j (chunk: which kThreads * R rows of the column the block takes).
template <int L, bool U8>
__device__ __forceinline__ void crt_rows(const void* __restrict__ cplanes, int64_t m_pad, int64_t n_pad,
                                         const int* __restrict__ sa, const int* __restrict__ sb, double* __restrict__ C,
                                         int64_t ldc, int64_t m, int64_t n, const double alpha, const double beta,
                                         const int triangle, const Oz2CrtConsts& cc, const int64_t j, const int64_t chunk) {
  typedef PlaneLoad<U8> PL;
  typedef typename PL::Raw Raw;
  constexpr int R = PL::R;
  const int64_t i0 = (chunk * kThreads + threadIdx.x) * R;
  if (i0 >= m) return;
  // symmetric product: only the lower (1: i >= j) or upper (2: i <= j) triangle of C exists and is written
  if ((triangle == 1 && i0 + R - 1 < j) || (triangle == 2 && i0 > j)) return;
  // element (i, j) of plane t sits at index (t*n_pad + j)*m_pad + i, in units of int32 or of bytes
  const size_t elem = (size_t)j * m_pad + i0;
  const Raw* src = reinterpret_cast<const Raw*>(static_cast<const char*>(cplanes) + elem * (U8 ? 1 : 4));
  const size_t stride = (size_t)n_pad * m_pad * (U8 ? 1 : 4) / sizeof(Raw);

  double S[R][L];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int l = 0; l < L; ++l) S[r][l] = 0.0;

  // Planes are read once (non-temporal loads), a batch ahead of the arithmetic: kBatch loads per thread in flight keep enough bytes
  // moving per CU to cover the memory latency (one load ahead does not).
  constexpr int kBatch = 4;
  const int N = cc.N;
  Raw nxt[kBatch];
#pragma unroll
  for (int d = 0; d < kBatch; ++d) nxt[d] = __builtin_nontemporal_load(src + (size_t)(d < N ? d : N - 1) * stride);
  for (int t0 = 0; t0 < N; t0 += kBatch) {
    Raw cur[kBatch];
#pragma unroll
    for (int d = 0; d < kBatch; ++d) cur[d] = nxt[d];
    if (t0 + kBatch < N) {
#pragma unroll
      for (int d = 0; d < kBatch; ++d) {
        const int t = t0 + kBatch + d;
        nxt[d] = __builtin_nontemporal_load(src + (size_t)(t < N ? t : N - 1) * stride);  // past the end: a harmless repeat of the last plane
      }
    }
#pragma unroll
    for (int d = 0; d < kBatch; ++d) {
      const int t = t0 + d;
      if (t < N) {
        double res[R];
        PL::residues(cur[d], cc.p[t], cc.inv_p[t], cc.half_inv_p[t], res);
#pragma unroll
        for (int l = 0; l < L; ++l) {
          const double w = cc.w[t][l];
#pragma unroll
          for (int r = 0; r < R; ++r) S[r][l] = fma(res[r], w, S[r][l]);
        }
      }
    }
  }
  const int sbj = sb[j];
  double* dst = C + i0 + j * ldc;
  double out[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    int e2;
    const double x = oz2_crt_reduce<L>(S[r], cc, &e2);
    out[r] = ldexp(x, e2 - sa[i0 + r] - sbj);  // sa is padded to m_pad (a multiple of 256): readable
  }
  if (alpha != 1.0 || beta != 0.0) {
    // C := alpha * P + beta * C with one rounding of beta * C and one fused multiply-add; C is not read when
    // beta is zero (BLAS convention)
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const bool mine = i0 + r < m && !(triangle == 1 && i0 + r < j) && !(triangle == 2 && i0 + r > j);
      const double tt = (beta == 0.0 || !mine) ? 0.0 : beta * dst[r];
      out[r] = fma(alpha, out[r], tt);
    }
  }
  // all R results of the thread leave together: its 8 R contiguous bytes complete their cache lines at once
  const bool whole = triangle == 0 || (triangle == 1 && i0 >= j) || (triangle == 2 && i0 + R - 1 <= j);
  if (whole && i0 + R <= m && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
#pragma unroll
    for (int r = 0; r < R; r += 2) *reinterpret_cast<double2*>(dst + r) = make_double2(out[r], out[r + 1]);
  } else {
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (i0 + r < m && !(triangle == 1 && i0 + r < j) && !(triangle == 2 && i0 + r > j)) dst[r] = out[r];
  }
}

template <int L, bool U8>
__global__ void __launch_bounds__(kThreads) crt_kernel(const void* __restrict__ cplanes, int64_t m_pad, int64_t n_pad,
                                                       const int* __restrict__ sa, const int* __restrict__ sb,
                                                       double* __restrict__ C, int64_t ldc, int64_t m, int64_t n,
                                                       const double alpha, const double beta,
                                                       const unsigned long long* __restrict__ skip_flag,
                                                       const int triangle, const Oz2CrtConsts cc) {
  // a non-finite input was found in stage 1: C is left to the FP64 fallback (uniform over the grid)
  if (skip_flag != nullptr && *skip_flag != 0ull) return;
  crt_rows<L, U8>(cplanes, m_pad, n_pad, sa, sb, C, ldc, m, n, alpha, beta, triangle, cc, blockIdx.x, blockIdx.y);
}

// Small problems, where every launch counts: the blocks of the FP64 fallback ride in the same launch.  Rows of
// blocks below crt_chunks are the kernel above; the rows after them are the fallback's tiles, numbered along x
// first.  Which of the two sets works is decided by the flag of stage 1, the other returns at once.
template <int L>
__global__ void __launch_bounds__(kThreads, 2) crt_or_fallback_kernel(const void* __restrict__ cplanes, int64_t m_pad,
                                                                   int64_t n_pad, const int* __restrict__ sa,
                                                                   const int* __restrict__ sb,
                                                                   const unsigned long long* __restrict__ flag,
                                                                   const unsigned crt_chunks, const int64_t tiles,
                                                                   const Oz2FallbackArgs f, const Oz2CrtConsts cc) {
  const bool nonfinite = *flag != 0ull;
  if (blockIdx.y < crt_chunks) {
    if (nonfinite) return;
    crt_rows<L, true>(cplanes, m_pad, n_pad, sa, sb, f.C, f.ldc, f.m, f.n, f.alpha, f.beta, 0, cc, blockIdx.x, blockIdx.y);
  } else {
    const int64_t tile = (int64_t)(blockIdx.y - crt_chunks) * gridDim.x + blockIdx.x;
    if (!nonfinite || tile >= tiles) return;
    oz2_fallback_tile(f, tile);
  }
}

// ---------------------------------------------------------------------------------------------------
// Lines 8-11 on UINT8 residue planes with the accumulation of line 9 on the matrix cores (at most 16 moduli).
// Y = sum_t c''_t W_t is a product of the residues (elements x moduli, bytes) with the weights (moduli x digits,
// bytes once the weights are written in balanced base-256 digits): one v_mfma_i32_32x32x32_i8 forms all sixteen
// digit sums of 64 output elements.  Operand roles: the 32 "rows" of the first operand run over the result
// registers and hold the digits, rows 0-15 with their weights on inner positions 0-15 and rows 16-31 with the same
// weights on inner positions 16-31; a lane of the second operand supplies inner positions 16 (lane / 32) + 0..15 of
// column lane % 32, i.e. the sixteen residues of ITS OWN element.  Lanes 0-31 therefore multiply against rows 0-15,
// lanes 32-63 against rows 16-31, and every lane's element gets its sixteen digit sums, half of them in the lane
// itself and half in the lane 32 away (result register e of lane l is row 8 (e / 4) + 4 (l / 32) + e % 4); eight
// v_permlane32_swap bring them together.  The residues enter as c'' - 128 (signed bytes); 128 sum_t dig, in limb
// form, is added when the digits become the 40-bit limbs the exact tail works on.
// A thread owns four consecutive rows (one 32-bit load per plane, transposed to four 16-byte operands with byte
// permutes) of kCrtCols consecutive columns, so that the set-up of the constant operand is spread over 64 elements.
// Against the FP64 accumulation: 120 instead of 156 instructions per element.
// ---------------------------------------------------------------------------------------------------
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));
constexpr int kCrtCols = 16;

// digit held by row rb (0..15) of a 16-row block: rows 0-3 and 8-11 land in lanes 0-31 (digits 0-7), rows 4-7 and
// 12-15 in lanes 32-63 (digits 8-15)
__device__ __forceinline__ constexpr int digit_of_row(int rb) { return ((rb >> 2) & 1) * 8 + (rb >> 3) * 4 + (rb & 3); }

template <int L>
__global__ void __launch_bounds__(kThreads) crt_mfma_kernel(const uint8_t* __restrict__ planes, int64_t m_pad, int64_t n_pad,
                                                            const int* __restrict__ sa, const int* __restrict__ sb,
                                                            double* __restrict__ C, int64_t ldc, int64_t m, int64_t n,
                                                            const double alpha, const double beta,
                                                            const unsigned long long* __restrict__ skip_flag,
                                                            const int triangle, const Oz2CrtConsts cc, const Oz2CrtDigits dg) {
  if (skip_flag != nullptr && *skip_flag != 0ull) return;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, half = lane >> 5;
  const int64_t i0 = ((int64_t)blockIdx.y * (kThreads / 64) + wv) * 256 + 4 * lane;  // this thread's four rows
  if (i0 - 4 * lane >= m) return;  // the whole wave (planes are padded to multiples of 256 rows: what it reads exists)
  const int64_t j0 = (int64_t)blockIdx.x * kCrtCols;
  const int N = cc.N;

  // first operand: row lane % 32, inner positions 16 (lane / 32) .. + 15; nonzero where the row's block is the half
  const v16i_t zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  v4i_t wop = {0, 0, 0, 0};
  {
    const int row = lane & 31;
    const int mine = (row >> 4) == half ? digit_of_row(row & 15) : -1;
#pragma unroll
    for (int d = 0; d < 16; ++d) {
      const int* w = reinterpret_cast<const int*>(dg.dig[d]);
      if (mine == d) wop = v4i_t{w[0], w[1], w[2], w[3]};
    }
  }

  const size_t plane_words = (size_t)n_pad * m_pad / 4;
  const unsigned* src = reinterpret_cast<const unsigned*>(planes) + ((size_t)j0 * m_pad + i0) / 4;
  unsigned nx[16];
  auto fetch = [&](int jj) {
#pragma unroll
    for (int t = 0; t < 16; ++t)
      nx[t] = (t < N && j0 + jj < n) ? __builtin_nontemporal_load(src + (size_t)t * plane_words + (size_t)jj * (m_pad / 4)) : 0x80808080u;
  };
  fetch(0);
  for (int jj = 0; jj < kCrtCols; ++jj) {
    const int64_t j = j0 + jj;
    if (j >= n) break;  // uniform
    unsigned x[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) x[t] = nx[t] ^ 0x80808080u;  // c'' - 128 as signed bytes
    if (jj + 1 < kCrtCols) fetch(jj + 1);
    // 16 words [modulus](4 rows) -> 4 operands [row](16 moduli)
    v4i_t y[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const unsigned a = __builtin_amdgcn_perm(x[4 * g + 1], x[4 * g], 0x05010400u);  // x0.b0 x1.b0 x0.b1 x1.b1
      const unsigned b = __builtin_amdgcn_perm(x[4 * g + 1], x[4 * g], 0x07030602u);  // x0.b2 x1.b2 x0.b3 x1.b3
      const unsigned c = __builtin_amdgcn_perm(x[4 * g + 3], x[4 * g + 2], 0x05010400u);
      const unsigned d = __builtin_amdgcn_perm(x[4 * g + 3], x[4 * g + 2], 0x07030602u);
      y[0][g] = (int)__builtin_amdgcn_perm(c, a, 0x05040100u);  // a.lo16 c.lo16
      y[1][g] = (int)__builtin_amdgcn_perm(c, a, 0x07060302u);  // a.hi16 c.hi16
      y[2][g] = (int)__builtin_amdgcn_perm(d, b, 0x05040100u);
      y[3][g] = (int)__builtin_amdgcn_perm(d, b, 0x07060302u);
    }
    const int sbj = sb[j];
    double out[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const v16i_t acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wop, y[r], zero16, 0, 0, 0);
      int D[16];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // lanes 0-31 keep register e (digit e) and get the other half's register e (digit 8 + e) in the place of
        // register 8 + e; lanes 32-63 the other way round
        const auto sw = __builtin_amdgcn_permlane32_swap((unsigned)acc[e], (unsigned)acc[8 + e], false, false);
        D[e] = (int)sw[0];
        D[8 + e] = (int)sw[1];
      }
      double S[L];
      oz2_digits_to_limbs<L>(D, dg.sinit, S);
      int e2;
      const double xv = oz2_crt_reduce<L>(S, cc, &e2);
      out[r] = ldexp(xv, e2 - sa[i0 + r] - sbj);
    }
    double* dst = C + i0 + j * ldc;
    if (alpha != 1.0 || beta != 0.0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool mine = i0 + r < m && !(triangle == 1 && i0 + r < j) && !(triangle == 2 && i0 + r > j);
        const double tt = (beta == 0.0 || !mine) ? 0.0 : beta * dst[r];
        out[r] = fma(alpha, out[r], tt);
      }
    }
    const bool whole = triangle == 0 || (triangle == 1 && i0 >= j) || (triangle == 2 && i0 + 3 <= j);
    if (whole && i0 + 4 <= m && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
      *reinterpret_cast<double2*>(dst) = make_double2(out[0], out[1]);
      *reinterpret_cast<double2*>(dst + 2) = make_double2(out[2], out[3]);
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (i0 + r < m && !(triangle == 1 && i0 + r < j) && !(triangle == 2 && i0 + r > j)) dst[r] = out[r];
    }
  }
}

// C := beta * C (zero without reading C when beta is zero): the k == 0 and alpha == 0 cases
__global__ void __launch_bounds__(kThreads) scale_c_kernel(double* __restrict__ C, int64_t ldc, int64_t m, double beta,
                                                           int triangle) {
  int64_t i = (int64_t)blockIdx.y * kThreads + threadIdx.x;
  const int64_t j = blockIdx.x;
  if (i < m && !(triangle == 1 && i < j) && !(triangle == 2 && i > j)) {
    double* p = C + i + (int64_t)blockIdx.x * ldc;
    *p = beta == 0.0 ? 0.0 : beta * *p;
  }
}

template <int L>
double host_crt(const Oz2CrtConsts& cc, const int32_t* cprod) {
  double S[L];
  for (int l = 0; l < L; ++l) S[l] = 0.0;
  for (int t = 0; t < cc.N; ++t) {
    double r = oz2_floor_mod(cprod[t], cc.p[t], cc.inv_p[t], cc.half_inv_p[t]);
    for (int l = 0; l < L; ++l) S[l] = fma(r, cc.w[t][l], S[l]);
  }
  int e2;
  double x = oz2_crt_reduce<L>(S, cc, &e2);
  return ldexp(x, e2);
}

}  // namespace

hipError_t oz2_launch_stage3(int64_t m, int64_t n, double alpha, double beta, double* C, int64_t ldc,
                             const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int residue_u8, int check_flag,
                             int triangle, hipStream_t st) {
  const void* cplanes = ws + lay.off_c;
  const unsigned long long* skip = check_flag ? reinterpret_cast<const unsigned long long*>(ws + lay.off_flags) : nullptr;
  const int* sa = reinterpret_cast<const int*>(ws + lay.off_sa);
  const int* sb = triangle ? sa : reinterpret_cast<const int*>(ws + lay.off_sb);  // symmetric: columns are A's rows
  const int64_t per_block = (int64_t)kThreads * (residue_u8 ? PlaneLoad<true>::R : PlaneLoad<false>::R);
  dim3 grid((unsigned)n, (unsigned)((m + per_block - 1) / per_block));
  // (from 2^24 elements on: below, a thread's 64 elements leave too few threads for the chip and the other kernel wins)
  if (residue_u8 && plan.digits.valid && m * n >= ((int64_t)1 << 24)) {
    // at most 16 moduli: the accumulation of line 9 on the matrix cores
    const uint8_t* p8 = static_cast<const uint8_t*>(cplanes);
    dim3 g2((unsigned)((n + kCrtCols - 1) / kCrtCols), (unsigned)((m + 1023) / 1024));
    switch (plan.crt.L) {
#define OZ2_CASE(LL)                                                                                                  \
  case LL:                                                                                                            \
    hipLaunchKernelGGL((crt_mfma_kernel<LL>), g2, dim3(kThreads), 0, st, p8, lay.m_pad, lay.n_pad, sa, sb, C, ldc, m, \
                       n, alpha, beta, skip, triangle, plan.crt, plan.digits);                                         \
    break;
      OZ2_CASE(1)
      OZ2_CASE(2)
      OZ2_CASE(3)
      OZ2_CASE(4)
#undef OZ2_CASE
      default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  switch (plan.crt.L) {
#define OZ2_CASE(LL)                                                                                              \
  case LL:                                                                                                        \
    if (residue_u8)                                                                                               \
      hipLaunchKernelGGL((crt_kernel<LL, true>), grid, dim3(kThreads), 0, st, cplanes, lay.m_pad, lay.n_pad, sa,  \
                         sb, C, ldc, m, n, alpha, beta, skip, triangle, plan.crt);                                \
    else                                                                                                          \
      hipLaunchKernelGGL((crt_kernel<LL, false>), grid, dim3(kThreads), 0, st, cplanes, lay.m_pad, lay.n_pad, sa, \
                         sb, C, ldc, m, n, alpha, beta, skip, triangle, plan.crt);                                \
    break;
    OZ2_CASE(1)
    OZ2_CASE(2)
    OZ2_CASE(3)
    OZ2_CASE(4)
    OZ2_CASE(5)
#undef OZ2_CASE
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Stage 3 on UINT8 residue planes and the FP64 fallback in one launch (general product, full C).
hipError_t oz2_launch_stage3_or_fallback(int transa, int transb, int64_t m, int64_t n, int64_t k, double alpha,
                                         const double* A, int64_t lda, const double* B, int64_t ldb, double beta, double* C,
                                         int64_t ldc, const Oz2Plan& plan, const Oz2Layout& lay, char* ws, hipStream_t st) {
  const void* cplanes = ws + lay.off_c;
  const unsigned long long* flag = reinterpret_cast<const unsigned long long*>(ws + lay.off_flags);
  const int* sa = reinterpret_cast<const int*>(ws + lay.off_sa);
  const int* sb = reinterpret_cast<const int*>(ws + lay.off_sb);
  const int64_t per_block = (int64_t)kThreads * PlaneLoad<true>::R;
  const int64_t chunks = (m + per_block - 1) / per_block;
  const int64_t tiles_m = (m + kFallbackTile - 1) / kFallbackTile, tiles_n = (n + kFallbackTile - 1) / kFallbackTile;
  const int64_t tiles = tiles_m * tiles_n, tile_rows = (tiles + n - 1) / n;
  if (chunks + tile_rows > 65535) return hipErrorInvalidValue;
  const Oz2FallbackArgs f = {transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, tiles_m, 0, 0, 0};
  dim3 grid((unsigned)n, (unsigned)(chunks + tile_rows));
  switch (plan.crt.L) {
#define OZ2_CASE(LL)                                                                                                 \
  case LL:                                                                                                           \
    hipLaunchKernelGGL((crt_or_fallback_kernel<LL>), grid, dim3(kThreads), 0, st, cplanes, lay.m_pad, lay.n_pad, sa, \
                       sb, flag, (unsigned)chunks, tiles, f, plan.crt);                                              \
    break;
    OZ2_CASE(1)
    OZ2_CASE(2)
    OZ2_CASE(3)
    OZ2_CASE(4)
    OZ2_CASE(5)
#undef OZ2_CASE
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t oz2_launch_scale_c(int64_t m, int64_t n, double beta, double* C, int64_t ldc, int triangle, hipStream_t st) {
  dim3 grid((unsigned)n, (unsigned)((m + kThreads - 1) / kThreads));
  hipLaunchKernelGGL(scale_c_kernel, grid, dim3(kThreads), 0, st, C, ldc, m, beta, triangle);
  return hipGetLastError();
}

template <int L>
double host_crt_digits(const Oz2CrtConsts& cc, const Oz2CrtDigits& dg, const uint8_t* res) {
  int D[16];
  for (int i = 0; i < 16; ++i) {
    int acc = 0;  // what the matrix core computes: signed bytes c'' - 128 against the digits
    for (int t = 0; t < cc.N; ++t) acc += ((int)res[t] - 128) * (int)dg.dig[i][t];
    D[i] = acc;
  }
  double S[L];
  oz2_digits_to_limbs<L>(D, dg.sinit, S);
  int e2;
  double x = oz2_crt_reduce<L>(S, cc, &e2);
  return ldexp(x, e2);
}

double oz2_host_crt_digits_impl(const Oz2CrtConsts& cc, const Oz2CrtDigits& dg, const uint8_t* res) {
  switch (cc.L) {
    case 1: return host_crt_digits<1>(cc, dg, res);
    case 2: return host_crt_digits<2>(cc, dg, res);
    case 3: return host_crt_digits<3>(cc, dg, res);
    default: return host_crt_digits<4>(cc, dg, res);
  }
}

double oz2_host_crt_impl(const Oz2CrtConsts& cc, const int32_t* cprod) {
  switch (cc.L) {
    case 1: return host_crt<1>(cc, cprod);
    case 2: return host_crt<2>(cc, cprod);
    case 3: return host_crt<3>(cc, cprod);
    case 4: return host_crt<4>(cc, cprod);
    default: return host_crt<5>(cc, cprod);
  }
}
