// Stage 1 of Ozaki scheme II on gfx950: Algorithm 1 lines 1-5.
//   1a  per-row maximum of |A| and per-column maximum of |B| (bit patterns, 64-bit atomic max)
//   1a' shifts  sa_i = kappa - 1 - floor(log2 max_l |a_il|),  sb_j likewise  (Section 3, D and E); or, in the
//       modes of Section 4.1, from an integer bound of the 2-norms (one more pass over A and B) or from the
//       row / column maxima of an INT8 product of 6-bit upper bounds of |A| and |B| (bound planes, one GEMM
//       launch, one pass over the product)
//   1b  a' = trunc(a * 2^sa_i) and its symmetric residues modulo every p_t, written as INT8 planes in the
//       blocked layout the GEMM reads (256 rows x 64 inner-dimension bytes per contiguous block), zero
//       padded up to the GEMM tile sizes.
// All are bound by HBM traffic: 8 bytes read per element in 1a, 8 read + N written in 1b.  The operands are far
// larger than the caches and every plane byte is written once, so loads and stores are non-temporal (measured:
// 3-6 % on stage 1).
// Infinities and NaNs are noticed in 1a (their bit patterns are above every finite magnitude) and recorded in
// a flag word of the workspace.  Triangular operands (TRMM shape) are masked while they are read.
// The maxima of both operands share one launch and so do their conversions (small problems are bound by the
// number of launches); a block picks its operand and its kernel body by its index.
#include "oz2_math.h"

namespace {

constexpr int kThreads = 256;
typedef unsigned v4u __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(kThreads) fill_u64_kernel(unsigned long long* p, int64_t count) {
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < count) p[i] = 0ull;
}

// Bit pattern of +infinity: as unsigned integers the magnitudes of infinities and NaNs are the values at or
// above it, every finite magnitude is below.
constexpr unsigned long long kInfBits = 0x7ff0000000000000ull;

// Triangular operands (TRMM shape): the array holds only one triangle; the rest is not referenced and counts
// as zero, the diagonal as one when it is declared unit.  (r, c) = row and column of the element in the
// stored array.  tri & 3: 0 = full matrix, 1 = lower (r >= c stored), 2 = upper (r <= c); tri & 4: unit diagonal.
__device__ __forceinline__ double tri_value(double v, int64_t r, int64_t c, int tri) {
  if (tri == 0) return v;
  if (r == c) return (tri & 4) ? 1.0 : v;
  const bool stored = (tri & 3) == 1 ? r > c : r < c;
  return stored ? v : 0.0;
}

__device__ __forceinline__ unsigned long long abs_bits(double v) {
  return (unsigned long long)__double_as_longlong(v) & 0x7fffffffffffffffull;
}

// A is m x k column-major: lanes run along rows (coalesced), each block covers 256 rows x KC columns.
constexpr int kRowMaxKC = 128;
__device__ __forceinline__ void strided_max(const double* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                            unsigned long long* __restrict__ rowmax,
                                            unsigned long long* __restrict__ nonfinite, int tri, unsigned bx,
                                            unsigned by) {
  int64_t i = (int64_t)bx * kThreads + threadIdx.x;
  if (i >= m) return;
  int64_t l0 = (int64_t)by * kRowMaxKC;
  int64_t l1 = l0 + kRowMaxKC < k ? l0 + kRowMaxKC : k;
  const double* p = A + i + l0 * lda;
  unsigned long long mx = 0ull;
  int64_t l = l0;
  for (; l + 8 <= l1; l += 8) {
    unsigned long long v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = abs_bits(tri_value(__builtin_nontemporal_load(p + (int64_t)u * lda), i, l + u, tri));
#pragma unroll
    for (int u = 0; u < 8; ++u) mx = v[u] > mx ? v[u] : mx;
    p += 8 * lda;
  }
  for (; l < l1; ++l) {
    unsigned long long v = abs_bits(tri_value(*p, i, l, tri));
    mx = v > mx ? v : mx;
    p += lda;
  }
  if (mx) atomicMax(rowmax + i, mx);
  if (mx >= kInfBits) *nonfinite = 1ull;
}

// B is k x n column-major: one block per (column, chunk of KC rows); lanes run down the column.
constexpr int kColMaxKC = 4096;
__device__ __forceinline__ void contig_max(const double* __restrict__ B, int64_t ldb, int64_t k,
                                           unsigned long long* __restrict__ colmax,
                                           unsigned long long* __restrict__ nonfinite, int tri, unsigned bx, unsigned by) {
  int64_t j = bx;
  int64_t l0 = (int64_t)by * kColMaxKC;
  const double* p = B + j * ldb;
  unsigned long long mx = 0ull;
#pragma unroll 4
  for (int u = 0; u < kColMaxKC / kThreads; ++u) {
    int64_t l = l0 + (int64_t)u * kThreads + threadIdx.x;
    if (l < k) {
      unsigned long long v = abs_bits(tri_value(__builtin_nontemporal_load(p + l), l, j, tri));
      mx = v > mx ? v : mx;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    unsigned long long o = __shfl_xor(mx, off, 64);
    mx = o > mx ? o : mx;
  }
  __shared__ unsigned long long part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) mx = part[w] > mx ? part[w] : mx;
    if (mx) atomicMax(colmax + j, mx);
    if (mx >= kInfBits) *nonfinite = 1ull;
  }
}

// Both operands of a call in one launch: a block belongs to the first job or to the second by its index.
// strided: the vectors are rows of a column-major array (lanes along the vectors); otherwise they are its
// columns (lanes along the inner dimension).  gx: extent of the job's first (fast) block coordinate.
struct MaxJob {
  const double* X;
  int64_t ld, nvec, k;
  unsigned long long* vmax;
  int tri, strided;
  unsigned gx, nblk;
};
__global__ void __launch_bounds__(kThreads) operand_max_kernel(const MaxJob ja, const MaxJob jb,
                                                               unsigned long long* __restrict__ nonfinite) {
  const bool first = blockIdx.x < ja.nblk;
  const MaxJob& j = first ? ja : jb;
  const unsigned id = first ? blockIdx.x : blockIdx.x - ja.nblk;
  const unsigned bx = id % j.gx, by = id / j.gx;
  if (j.strided)
    strided_max(j.X, j.ld, j.nvec, j.k, j.vmax, nonfinite, j.tri, bx, by);
  else
    contig_max(j.X, j.ld, j.k, j.vmax, nonfinite, j.tri, bx, by);
}

// ---- Cauchy-Schwarz shift mode (Section 4.1): integer upper bound of the 2-norm.
// With e = floor(log2 max |x|):  q_l = ceil(|x_l| 2^(19-e)) <= 2^20,  S = sum_l q_l^2  (exact in 64 bits for
// fewer than 2^23 terms, and independent of the order of summation).
__device__ __forceinline__ int exponent_of_bits(unsigned long long b) {  // floor(log2) of a positive double's bits
  int be = (int)(b >> 52);
  return be ? be - 1023 : (63 - __clzll((long long)b)) - 1074;
}

__device__ __forceinline__ double scaled_ceil_sq(double v, int sc) {
  double q = ceil(ldexp(fabs(v), sc));  // exact: a power-of-two scaling, then an integer at most 2^20
  if (v != 0.0 && q == 0.0) q = 1.0;    // the scaling underflowed: the ceiling of a positive value is 1
  return q * q;                         // exact: at most 2^40
}

__global__ void __launch_bounds__(kThreads) rownorm_kernel(const double* __restrict__ A, int64_t lda, int64_t m,
                                                           int64_t k, const unsigned long long* __restrict__ rowmax,
                                                           unsigned long long* __restrict__ rownorm, int tri) {
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= m) return;
  const unsigned long long mb = rowmax[i];
  if (!mb) return;
  const int sc = 19 - exponent_of_bits(mb);
  int64_t l0 = (int64_t)blockIdx.y * kRowMaxKC;
  int64_t l1 = l0 + kRowMaxKC < k ? l0 + kRowMaxKC : k;
  const double* p = A + i + l0 * lda;
  double acc = 0.0;  // at most 128 terms of at most 2^40: exact
  int64_t l = l0;
  for (; l + 8 <= l1; l += 8) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = tri_value(p[(int64_t)u * lda], i, l + u, tri);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += scaled_ceil_sq(v[u], sc);
    p += 8 * lda;
  }
  for (; l < l1; ++l) {
    acc += scaled_ceil_sq(tri_value(*p, i, l, tri), sc);
    p += lda;
  }
  atomicAdd(rownorm + i, (unsigned long long)acc);
}

__global__ void __launch_bounds__(kThreads) colnorm_kernel(const double* __restrict__ B, int64_t ldb, int64_t k,
                                                           const unsigned long long* __restrict__ colmax,
                                                           unsigned long long* __restrict__ colnorm, int tri) {
  int64_t j = blockIdx.x;
  const unsigned long long mb = colmax[j];
  if (!mb) return;  // uniform over the block
  const int sc = 19 - exponent_of_bits(mb);
  int64_t l0 = (int64_t)blockIdx.y * kColMaxKC;
  const double* p = B + j * ldb;
  double acc = 0.0;  // 16 terms
#pragma unroll 4
  for (int u = 0; u < kColMaxKC / kThreads; ++u) {
    int64_t l = l0 + (int64_t)u * kThreads + threadIdx.x;
    if (l < k) acc += scaled_ceil_sq(tri_value(p[l], l, j, tri), sc);
  }
  unsigned long long s = (unsigned long long)acc;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
  __shared__ unsigned long long part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) s += part[w];
    atomicAdd(colnorm + j, s);
  }
}

// Shifts of both operands in one launch (Algorithm 1 line 1).  Per vector, from the bit pattern b of its largest
// magnitude (e = floor(log2) of it) and, in the modes of Section 4.1, a second quantity v:
//   mode 0 (Section 3):       kappa - 1 - e                         (param = kappa)
//   mode 1 (Cauchy-Schwarz):  beta - (e - 19 + h), h = min{h : 4^h >= v}, v = integer norm bound S >= 2^38  (param = beta)
//   mode 2 (INT8 product):    floor((b2 - t)/2) - (e - 5), t = min{t : 2^t >= v}, v = largest element of the bound
//                             product in the vector's row / column      (param = b2)
// An all-zero vector gets shift 0.
// With unequal bit budgets (Section 3: k_A != k_B when the operands differ in precision) each operand has its
// own param (modes 0, 1) or an offset added at the end (mode 2).
struct ShiftJob {
  const unsigned long long* mx;
  const unsigned long long* aux;
  int* s;
  int64_t count;
  int param;
  int offset;
};
__global__ void __launch_bounds__(kThreads) shifts_kernel(const ShiftJob ja, const ShiftJob jb, int mode) {
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const bool first = i < ja.count;
  const ShiftJob& j = first ? ja : jb;
  if (!first) i -= ja.count;
  if (i >= j.count) return;
  const unsigned long long b = j.mx[i];
  const int param = j.param;
  int out = 0;
  if (b) {
    const int e = exponent_of_bits(b);
    if (mode == 0) {
      out = param - 1 - e;
    } else if (mode == 1) {
      const unsigned long long S = j.aux[i];
      const int bits = 64 - __clzll((long long)(S - 1));  // ceil(log2 S)
      out = param - (e - 19 + ((bits + 1) >> 1));
    } else {
      const unsigned long long R = j.aux[i];
      if (R) {
        const int t = R <= 1 ? 0 : 64 - __clzll((long long)(R - 1));
        const int d = param - t;
        out = (d >= 0 ? d / 2 : -((1 - d) / 2)) + j.offset - (e - 5);
      }
    }
  }
  j.s[i] = out;
}

// ---- Small operands: maxima and shifts (Section 3, the simple bound) of both operands in ONE launch and without
// atomics, so that nothing has to be cleared first: a workgroup owns 16 whole vectors, forms their maxima, writes
// them and the shifts kappa - 1 - floor(log2 max), and reports in a slot of its own whether it saw an infinity or
// a NaN.  The conversion launch that follows folds the slots into the flag word.  Three launches fewer than
// fill + maxima + shifts; used while the operands are small enough that 16 vectors per workgroup still fill the chip.
constexpr int kScanVecs = 16;
struct ScanJob {
  const double* X;
  int64_t ld, nvec, nvec_pad, k;
  unsigned long long* vmax;
  int* shifts;
  int param;  // kappa of this operand
  int tri, strided;
  unsigned nblk;
};
__global__ void __launch_bounds__(kThreads) vector_scan_kernel(const ScanJob ja, const ScanJob jb,
                                                               unsigned long long* __restrict__ slots) {
  __shared__ unsigned long long part[kThreads];
  const bool first = blockIdx.x < ja.nblk;
  const ScanJob& j = first ? ja : jb;
  const unsigned id = first ? blockIdx.x : blockIdx.x - ja.nblk;
  const int64_t v0 = (int64_t)id * kScanVecs;
  unsigned long long mx = 0ull;
  int vv;  // which of the 16 vectors this thread's partial maximum belongs to
  if (j.strided) {
    // element (v, l) at X[v + l ld]: 16 lanes along the vectors (128 contiguous bytes), 16 column phases
    vv = threadIdx.x & (kScanVecs - 1);
    const int64_t v = v0 + vv;
    if (v < j.nvec) {
      const double* p = j.X + v;
      int64_t l = threadIdx.x / kScanVecs;
      for (; l + 7 * (kThreads / kScanVecs) < j.k; l += 8 * (kThreads / kScanVecs)) {
        unsigned long long b[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int64_t lu = l + u * (kThreads / kScanVecs);
          b[u] = abs_bits(tri_value(p[lu * j.ld], v, lu, j.tri));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) mx = b[u] > mx ? b[u] : mx;
      }
      for (; l < j.k; l += kThreads / kScanVecs) {
        const unsigned long long b = abs_bits(tri_value(p[l * j.ld], v, l, j.tri));
        mx = b > mx ? b : mx;
      }
    }
    part[threadIdx.x] = mx;
    __syncthreads();
    if (threadIdx.x < kScanVecs) {
#pragma unroll
      for (int ph = 1; ph < kThreads / kScanVecs; ++ph) {
        const unsigned long long o = part[threadIdx.x + ph * kScanVecs];
        mx = o > mx ? o : mx;
      }
    }
  } else {
    // element (v, l) at X[l + v ld]: a wave takes four vectors in turn, its lanes run down the vector
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
    unsigned long long mine = 0ull;
#pragma unroll 1
    for (int q = 0; q < kScanVecs / 4; ++q) {
      const int64_t v = v0 + wv * (kScanVecs / 4) + q;
      unsigned long long m = 0ull;
      if (v < j.nvec) {
        const double* p = j.X + v * j.ld;
        int64_t l = lane;
        for (; l + 7 * 64 < j.k; l += 8 * 64) {
          unsigned long long b[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) b[u] = abs_bits(tri_value(p[l + u * 64], l + u * 64, v, j.tri));
#pragma unroll
          for (int u = 0; u < 8; ++u) m = b[u] > m ? b[u] : m;
        }
        for (; l < j.k; l += 64) {
          const unsigned long long b = abs_bits(tri_value(p[l], l, v, j.tri));
          m = b > m ? b : m;
        }
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(m, off, 64);
        m = o > m ? o : m;
      }
      if (lane == q) mine = m;
    }
    if (lane < kScanVecs / 4) part[wv * (kScanVecs / 4) + lane] = mine;
    __syncthreads();
    if (threadIdx.x < kScanVecs) mx = part[threadIdx.x];
  }
  // threads 0 .. 15 hold the maxima of the 16 vectors
  bool bad = false;
  if (threadIdx.x < kScanVecs) {
    const int64_t v = v0 + threadIdx.x;
    if (v < j.nvec_pad) {
      j.vmax[v] = mx;
      j.shifts[v] = mx ? j.param - 1 - exponent_of_bits(mx) : 0;
    }
    bad = mx >= kInfBits;
  }
  const int any = __syncthreads_or(bad ? 1 : 0);
  if (threadIdx.x == 0) slots[blockIdx.x] = any ? 1ull : 0ull;
}

// What the first workgroup of the conversion launch does for the launch above: the flag word (1 when any slot
// is set) and, cleared, the counters of the GEMM's round synchronisation.
struct ScanFinish {
  const unsigned long long* slots;  // null: nothing to do (the maxima came from the atomic kernels)
  unsigned count;
  unsigned long long* flags;        // 32 words
};
__device__ __forceinline__ void finish_scan(const ScanFinish& f) {
  int bad = 0;
  for (unsigned i = threadIdx.x; i < f.count; i += kThreads) bad |= f.slots[i] != 0ull;
  bad = __syncthreads_or(bad);
  if (threadIdx.x < 32) f.flags[threadIdx.x] = (threadIdx.x == 0 && bad) ? 1ull : 0ull;
}

__device__ __forceinline__ unsigned pack4(int r0, int r1, int r2, int r3) {
  return (unsigned)(r0 & 0xff) | ((unsigned)(r1 & 0xff) << 8) | ((unsigned)(r2 & 0xff) << 16) | ((unsigned)r3 << 24);
}

// sixteen consecutive inner-dimension values of one vector -> sixteen bound bytes
__device__ __forceinline__ void store_bounds(const double* mine, int shift, int8_t* dst) {
  int r[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) r[u] = oz2_bound6(mine[u], shift);
  uint4 v;
  v.x = pack4(r[0], r[1], r[2], r[3]);
  v.y = pack4(r[4], r[5], r[6], r[7]);
  v.z = pack4(r[8], r[9], r[10], r[11]);
  v.w = pack4(r[12], r[13], r[14], r[15]);
  *reinterpret_cast<uint4*>(dst) = v;
}

// ---- INT8-product shift mode (Section 4.1): row and column maxima of P = A''B'' (INT32, element (i,j) at
// j*m_pad + i).  One block: 256 rows x 64 columns; lanes run along the rows.
constexpr int kProdCols = 64;
__global__ void __launch_bounds__(kThreads) prodmax_kernel(const int* __restrict__ P, int64_t m_pad, int64_t m, int64_t n,
                                                           int64_t row_blocks, unsigned long long* __restrict__ rowtop,
                                                           unsigned long long* __restrict__ coltop) {
  const int64_t rb = blockIdx.x % row_blocks, cb = blockIdx.x / row_blocks;
  const int64_t i = rb * kThreads + threadIdx.x;  // < m_pad
  const int64_t j0 = cb * kProdCols;
  const int* src = P + i + j0 * m_pad;
  int rmax = 0;
  for (int jj = 0; jj < kProdCols; jj += 8) {
    int v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (i < m && j0 + jj + u < n) ? src[(int64_t)(jj + u) * m_pad] : 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      rmax = v[u] > rmax ? v[u] : rmax;
      int c = v[u];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        int o = __shfl_xor(c, off, 64);
        c = o > c ? o : c;
      }
      if ((threadIdx.x & 63) == 0 && c > 0) atomicMax(coltop + j0 + jj + u, (unsigned long long)c);
    }
  }
  if (rmax > 0) atomicMax(rowtop + i, (unsigned long long)rmax);
}

// Plane layout (shared with the GEMM kernel): blocks of 256 rows x 64 bytes of the inner dimension, each
// block contiguous; element (row, l) of plane t at
//   ((t*rows_pad + 256*(row/256)) * k_pad) + (l/64)*16384 + (row%256)*64 + (l%64).
constexpr int kBlkRows = OZ2_TILE_M;   // 256
constexpr int kBlkK = OZ2_TILE_K;      // 64
static_assert(OZ2_TILE_M == 256 && OZ2_TILE_N == 256 && OZ2_TILE_K == 64, "plane layout is 256 x 64 blocks");

// A (m x k column-major) -> planes.  Block: 64 rows x 64 columns.  Every column segment (64 rows, 512
// bytes) is read coalesced with lanes along the rows, transposed through LDS so that a thread holds 16
// consecutive inner-dimension values of one row, and wave w writes, for every plane, the 1 KiB that its 16
// rows x 64 bytes occupy contiguously in the output block.
constexpr int kConvARows = 64;
constexpr int kConvAPitch = 65;  // doubles per row in LDS
// KIND 0 / 1: residues of trunc(a 2^shift) with the one- / two-level split; KIND 2: the single plane of 6-bit
// upper bounds ceil(|a| 2^shift) of Section 4.1 (written where plane 0 goes).
template <int KIND>
__device__ __forceinline__ void convert_strided(const double* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                                int64_t m_pad, int64_t k_pad, const int* __restrict__ sa,
                                                int8_t* __restrict__ planes, const int tri, const Oz2ConvConsts& cc,
                                                double* tile, unsigned bx, unsigned by) {
  const int64_t r0 = (int64_t)bx * kConvARows;  // < m_pad
  const int64_t kb = by;
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  {
    const int64_t i = r0 + lane;
    const double* src = A + i;
#pragma unroll 4
    for (int c = 0; c < kBlkK / 4; ++c) {
      const int lc = c * 4 + wv;
      const int64_t l = kb * kBlkK + lc;
      double v = (i < m && l < k) ? tri_value(__builtin_nontemporal_load(src + l * lda), i, l, tri) : 0.0;
      tile[lane * kConvAPitch + lc] = v;
    }
  }
  __syncthreads();
  const int row = wv * 16 + (lane >> 2);
  const int chunk = lane & 3;
  const int64_t i = r0 + row;
  const int shift = i < m ? sa[i] : 0;
  const double* mine = tile + row * kConvAPitch + chunk * 16;
  const size_t plane_stride = (size_t)m_pad * k_pad;
  int8_t* dst = planes + (size_t)(i / kBlkRows) * kBlkRows * k_pad + (size_t)kb * (kBlkRows * kBlkK) +
                (i % kBlkRows) * kBlkK + chunk * 16;
  if constexpr (KIND == 2) {
    store_bounds(mine, shift, dst);
    return;
  }
  constexpr bool TWO_LEVEL = KIND == 1;
  Oz2Split xs[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) xs[u] = oz2_scale_trunc_split<TWO_LEVEL>(mine[u], shift);
  for (int t = 0; t < cc.N; ++t) {
    const double p = cc.p[t], ip = cc.inv_p[t], c32 = cc.c32[t], c64 = cc.c64[t];
    int r[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) r[u] = oz2_sym_residue<TWO_LEVEL>(xs[u], p, ip, c32, c64);
    uint4 v;
    v.x = pack4(r[0], r[1], r[2], r[3]);
    v.y = pack4(r[4], r[5], r[6], r[7]);
    v.z = pack4(r[8], r[9], r[10], r[11]);
    v.w = pack4(r[12], r[13], r[14], r[15]);
    // written once, read by a later kernel: non-temporal store
    __builtin_nontemporal_store(v4u{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u*>(dst + (size_t)t * plane_stride));
  }
}

// B (k x n column-major) -> planes (row index of a plane = column j of B).  Block: 16 columns x 256 rows
// of B.  Each column segment is read coalesced (one double per lane), transposed through LDS so that a
// thread holds 16 consecutive inner-dimension values of one column, and wave w writes, for every plane,
// the 1 KiB that 16 columns x 64 bytes occupy contiguously in the output block of k-tile w.
constexpr int kConvBCols = 16;
constexpr int kConvBKC = 256;
constexpr int kConvBGroup = 18;     // doubles per 16-element group in LDS (144 bytes)
constexpr int kConvBColPitch = 296; // doubles per column in LDS: 16 groups + 8 (2368 bytes = 64 mod 256)
template <int KIND>
__device__ __forceinline__ void convert_contig(const double* __restrict__ B, int64_t ldb, int64_t k, int64_t n,
                                               int64_t n_pad, int64_t k_pad, const int* __restrict__ sb,
                                               int8_t* __restrict__ planes, const int tri, const Oz2ConvConsts& cc,
                                               double* tile, unsigned bx, unsigned by) {
  const int64_t j0 = (int64_t)bx * kConvBCols;  // < n_pad, multiple of 16
  const int64_t lbase = (int64_t)by * kConvBKC;
  {
    const int64_t l = lbase + threadIdx.x;
    const int slot = (threadIdx.x >> 4) * kConvBGroup + (threadIdx.x & 15);
#pragma unroll 4
    for (int c = 0; c < kConvBCols; ++c) {
      const int64_t j = j0 + c;
      double v = (j < n && l < k) ? tri_value(__builtin_nontemporal_load(B + l + j * ldb), l, j, tri) : 0.0;
      tile[c * kConvBColPitch + slot] = v;
    }
  }
  __syncthreads();
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t l0 = lbase + wv * kBlkK + (lane & 3) * 16;
  if (lbase + wv * kBlkK >= k_pad) return;
  const int c = lane >> 2;
  const int64_t j = j0 + c;
  const int shift = j < n ? sb[j] : 0;
  const double* mine = tile + c * kConvBColPitch + (wv * 4 + (lane & 3)) * kConvBGroup;
  const size_t plane_stride = (size_t)n_pad * k_pad;
  int8_t* dst = planes + (size_t)(j / kBlkRows) * kBlkRows * k_pad + (size_t)(l0 / kBlkK) * (kBlkRows * kBlkK) +
                (j % kBlkRows) * kBlkK + (l0 % kBlkK);
  if constexpr (KIND == 2) {
    store_bounds(mine, shift, dst);
    return;
  }
  constexpr bool TWO_LEVEL = KIND == 1;
  Oz2Split xs[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) xs[u] = oz2_scale_trunc_split<TWO_LEVEL>(mine[u], shift);
  for (int t = 0; t < cc.N; ++t) {
    const double p = cc.p[t], ip = cc.inv_p[t], c32 = cc.c32[t], c64 = cc.c64[t];
    int r[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) r[u] = oz2_sym_residue<TWO_LEVEL>(xs[u], p, ip, c32, c64);
    uint4 v;
    v.x = pack4(r[0], r[1], r[2], r[3]);
    v.y = pack4(r[4], r[5], r[6], r[7]);
    v.z = pack4(r[8], r[9], r[10], r[11]);
    v.w = pack4(r[12], r[13], r[14], r[15]);
    // written once, read by a later kernel: non-temporal store
    __builtin_nontemporal_store(v4u{v.x, v.y, v.z, v.w}, reinterpret_cast<v4u*>(dst + (size_t)t * plane_stride));
  }
}

// Both operands of a call in one launch (see operand_max_kernel).  KA / KB: what is written for the first /
// second job (0, 1: residue planes with the one- / two-level split; 2: the bound plane).
struct ConvJob {
  const double* X;
  int64_t ld, nvec, k, nvec_pad, k_pad;
  const int* shifts;
  int8_t* planes;
  int tri, strided;
  unsigned gx, nblk;
};
constexpr int kConvTileDoubles =
    kConvARows * kConvAPitch > kConvBCols * kConvBColPitch ? kConvARows * kConvAPitch : kConvBCols * kConvBColPitch;
template <int KA, int KB>
__global__ void __launch_bounds__(kThreads) operand_convert_kernel(const ConvJob ja, const ConvJob jb,
                                                                   const Oz2ConvConsts cc, const ScanFinish fin) {
  __shared__ __attribute__((aligned(16))) double tile[kConvTileDoubles];
  if (fin.slots != nullptr && blockIdx.x == 0) finish_scan(fin);  // uniform over the workgroup
  if (blockIdx.x < ja.nblk) {
    const unsigned bx = blockIdx.x % ja.gx, by = blockIdx.x / ja.gx;
    if (ja.strided)
      convert_strided<KA>(ja.X, ja.ld, ja.nvec, ja.k, ja.nvec_pad, ja.k_pad, ja.shifts, ja.planes, ja.tri, cc, tile, bx, by);
    else
      convert_contig<KA>(ja.X, ja.ld, ja.k, ja.nvec, ja.nvec_pad, ja.k_pad, ja.shifts, ja.planes, ja.tri, cc, tile, bx, by);
  } else {
    const unsigned id = blockIdx.x - ja.nblk;
    const unsigned bx = id % jb.gx, by = id / jb.gx;
    if (jb.strided)
      convert_strided<KB>(jb.X, jb.ld, jb.nvec, jb.k, jb.nvec_pad, jb.k_pad, jb.shifts, jb.planes, jb.tri, cc, tile, bx, by);
    else
      convert_contig<KB>(jb.X, jb.ld, jb.k, jb.nvec, jb.nvec_pad, jb.k_pad, jb.shifts, jb.planes, jb.tri, cc, tile, bx, by);
  }
}

}  // namespace

namespace {

unsigned blocks_of(int64_t v, int64_t per) { return (unsigned)((v + per - 1) / per); }

// One operand of stage 1: a set of `nvec` vectors of length k (rows of op(A) or columns of op(B)).
// strided: element (v, l) at X[v + l*ld] (vectors are rows of a column-major matrix); otherwise element
// (v, l) at X[l + v*ld] (vectors are its columns).
struct Operand {
  const double* X;
  int64_t ld;
  bool strided;
  int64_t nvec, nvec_pad, k, k_pad;
  unsigned long long* vmax;   // bit pattern of the largest magnitude per vector
  unsigned long long* vaux;   // per-vector integer norm bound, or largest element of the bound product
  unsigned long long* flag;   // set to 1 when the operand holds an infinity or a NaN
  int tri;                    // triangular structure of the stored array (see tri_value), 0 for a full matrix
  int* shifts;
  int8_t* planes;
};

// maxima of one or two operands in one launch
hipError_t launch_max(const Operand* ops, int nops, hipStream_t st) {
  MaxJob job[2] = {};
  int64_t total = 0;
  for (int x = 0; x < nops; ++x) {
    const Operand& o = ops[x];
    const int64_t gx = o.strided ? blocks_of(o.nvec, kThreads) : o.nvec;
    const int64_t gy = o.strided ? blocks_of(o.k, kRowMaxKC) : blocks_of(o.k, kColMaxKC);
    total += gx * gy;
    if (total >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    job[x] = {o.X, o.ld, o.nvec, o.k, o.vmax, o.tri, o.strided ? 1 : 0, (unsigned)gx, (unsigned)(gx * gy)};
  }
  if (nops == 1) job[1] = job[0], job[1].nblk = 0;
  hipLaunchKernelGGL(operand_max_kernel, dim3((unsigned)total), dim3(kThreads), 0, st, job[0], job[1], ops[0].flag);
  return hipSuccess;
}

void launch_norm(const Operand& o, hipStream_t st) {
  const dim3 thr(kThreads);
  if (o.strided)
    hipLaunchKernelGGL(rownorm_kernel, dim3(blocks_of(o.nvec, kThreads), blocks_of(o.k, kRowMaxKC)), thr, 0, st, o.X, o.ld,
                       o.nvec, o.k, o.vmax, o.vaux, o.tri);
  else
    hipLaunchKernelGGL(colnorm_kernel, dim3((unsigned)o.nvec, blocks_of(o.k, kColMaxKC)), thr, 0, st, o.X, o.ld, o.k, o.vmax,
                       o.vaux, o.tri);
}

// planes of one or two operands in one launch; kind 0 / 1: residue planes with the one- / two-level split,
// kind 2: the bound plane
hipError_t launch_convert(const Operand* ops, int nops, const int* kind, const Oz2ConvConsts& conv, const ScanFinish& fin,
                          hipStream_t st) {
  ConvJob job[2] = {};
  int64_t total = 0;
  for (int x = 0; x < nops; ++x) {
    const Operand& o = ops[x];
    const int64_t gx = o.strided ? o.nvec_pad / kConvARows : o.nvec_pad / kConvBCols;
    const int64_t gy = o.strided ? o.k_pad / kBlkK : blocks_of(o.k_pad, kConvBKC);
    total += gx * gy;
    if (total >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    job[x] = {o.X, o.ld, o.nvec, o.k, o.nvec_pad, o.k_pad, o.shifts, o.planes, o.tri, o.strided ? 1 : 0, (unsigned)gx,
              (unsigned)(gx * gy)};
  }
  const int ka = kind[0], kb = nops == 2 ? kind[1] : kind[0];
  if (nops == 1) job[1] = job[0], job[1].nblk = 0;
  const dim3 grid((unsigned)total), thr(kThreads);
#define OZ2_CONV(KA, KB) hipLaunchKernelGGL((operand_convert_kernel<KA, KB>), grid, thr, 0, st, job[0], job[1], conv, fin)
  if (ka == 2)
    OZ2_CONV(2, 2);
  else if (ka == 0 && kb == 0)
    OZ2_CONV(0, 0);
  else if (ka == 0)
    OZ2_CONV(0, 1);
  else if (kb == 0)
    OZ2_CONV(1, 0);
  else
    OZ2_CONV(1, 1);
#undef OZ2_CONV
  return hipSuccess;
}

}  // namespace

// transa / transb: 0 = the operand is stored as op(X) (column-major), 1 = it is stored transposed.
// B == nullptr: the symmetric product op(A) op(A)^T (n == m); only A's vectors, shifts and planes are produced.
// tri_a / tri_b: triangular structure of the stored arrays (0 = full; see tri_value).
// strassen: lay is the layout of the Strassen form; shifts (and the bound product of the INT8-product mode) are
// formed as usual on its padded extents, only the residue planes differ.
hipError_t oz2_launch_stage1(int transa, int transb, int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                             const double* B, int64_t ldb, int tri_a, int tri_b, const Oz2Plan& plan, int shift_mode,
                             int bit_split, int strassen, const Oz2Layout& lay, char* ws, hipStream_t st) {
  // rows of op(A): strided in a stored m x k matrix, contiguous in a stored k x m matrix;
  // columns of op(B): contiguous in a stored k x n matrix, strided in a stored n x k matrix
  // Row maxima, flag words and column maxima are adjacent, and so are the two auxiliary vectors: one fill
  // launch clears each group.
  if (lay.off_flags != lay.off_rowmax + (size_t)lay.m_pad * 8 || lay.off_colmax != lay.off_flags + 256 ||
      lay.off_colnorm != lay.off_rownorm + (size_t)lay.m_pad * 8)
    return hipErrorInvalidValue;
  unsigned long long* flag = reinterpret_cast<unsigned long long*>(ws + lay.off_flags);
  const Operand ops[2] = {
      {A, lda, transa == 0, m, lay.m_pad, k, lay.k_pad, reinterpret_cast<unsigned long long*>(ws + lay.off_rowmax),
       reinterpret_cast<unsigned long long*>(ws + lay.off_rownorm), flag, tri_a,
       reinterpret_cast<int*>(ws + lay.off_sa), reinterpret_cast<int8_t*>(ws + lay.off_a)},
      {B, ldb, transb != 0, n, lay.n_pad, k, lay.k_pad, reinterpret_cast<unsigned long long*>(ws + lay.off_colmax),
       reinterpret_cast<unsigned long long*>(ws + lay.off_colnorm), flag, tri_b,
       reinterpret_cast<int*>(ws + lay.off_sb), reinterpret_cast<int8_t*>(ws + lay.off_b)}};
  const dim3 thr(kThreads);
  const int nops = B ? 2 : 1;
  const int64_t n_max = nops == 2 ? lay.m_pad + 32 + lay.n_pad : lay.m_pad + 32;
  const int64_t n_aux = nops == 2 ? lay.m_pad + lay.n_pad : lay.m_pad;
  auto fill = [&](unsigned long long* p, int64_t count) {
    hipLaunchKernelGGL(fill_u64_kernel, dim3(blocks_of(count, kThreads)), thr, 0, st, p, count);
  };
  auto shifts = [&](int mode, int param_a, int param_b, int off_a, int off_b) {
    const ShiftJob ja = {ops[0].vmax, ops[0].vaux, ops[0].shifts, ops[0].nvec_pad, param_a, off_a};
    const ShiftJob jb = {ops[1].vmax, ops[1].vaux, ops[1].shifts, nops == 2 ? ops[1].nvec_pad : 0, param_b, off_b};
    hipLaunchKernelGGL(shifts_kernel, dim3(blocks_of(ja.count + jb.count, kThreads)), thr, 0, st, ja, jb, mode);
  };
  Oz2ConvConsts conv = plan.conv;
  // Budgets per operand: bit_split moves that many bits from the first operand to the second, which also gets
  // the odd bit of the sum (bit_split == 0: the equal split; the symmetric product always uses it).
  const int d = bit_split;
  int xbits[2];  // |x'| < 2^xbits decides how deep the conversion kernels split an element
  ScanFinish fin = {nullptr, 0u, nullptr};
  // Small operands under the simple bound: maxima and shifts in one launch without atomics (nothing to clear
  // first); its per-workgroup reports become the flag word in the conversion launch.  "Small": at most 2^25 elements
  // in both operands together (4096 x 4096 twice), where 16 vectors per workgroup are work enough for the chip
  // and the launches saved still count.
  const bool scan = shift_mode == OZ2_SHIFT_MAX && !strassen &&
                    (lay.m_pad + (nops == 2 ? lay.n_pad : 0)) * lay.k_pad <= ((int64_t)1 << 25);
  if (scan) {
    const int kappa_a = plan.kappa - d, kappa_b = d == 0 ? plan.kappa : plan.kappa_sum - kappa_a;
    ScanJob sj[2] = {};
    unsigned total = 0;
    for (int x = 0; x < nops; ++x) {
      const Operand& o = ops[x];
      sj[x] = {o.X, o.ld, o.nvec, o.nvec_pad, o.k, o.vmax, o.shifts, x == 0 ? kappa_a : kappa_b, o.tri, o.strided ? 1 : 0,
               (unsigned)(o.nvec_pad / kScanVecs)};
      total += sj[x].nblk;
    }
    if (nops == 1) sj[1] = sj[0], sj[1].nblk = 0;
    // the slots live in the auxiliary vectors, which this shift mode does not use (one word per 16 vectors)
    unsigned long long* slots = ops[0].vaux;
    hipLaunchKernelGGL(vector_scan_kernel, dim3(total), thr, 0, st, sj[0], sj[1], slots);
    fin = {slots, total, flag};
    xbits[0] = kappa_a;
    xbits[1] = kappa_b;
  } else {
  fill(ops[0].vmax, n_max);
  if (hipError_t e = launch_max(ops, nops, st); e != hipSuccess) return e;
  }
  if (scan) {
    // shifts are written
  } else if (shift_mode == OZ2_SHIFT_INT8_PRODUCT) {
    // bound planes (in the slots of residue plane 0), their INT8 product (in the slot of product plane 0),
    // its row and column maxima, then the shifts.  In the symmetric case the product is A''A''^T and its
    // row maxima are its column maxima (those land in the unused column array).
    shifts(0, 6, 6, 0, 0);  // exponents 5 - e of the bounds
    {
      const int bound[2] = {2, 2};
      if (hipError_t e = launch_convert(ops, nops, bound, conv, ScanFinish{nullptr, 0u, nullptr}, st); e != hipSuccess) return e;
    }
    fill(ops[0].vaux, n_aux);
    hipError_t e = oz2_launch_bound_gemm(lay, ws, B == nullptr, st);
    if (e != hipSuccess) return e;
    const int64_t row_blocks = lay.m_pad / kThreads;
    const int64_t nblk = row_blocks * (int64_t)blocks_of(n, kProdCols);
    if (nblk >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(prodmax_kernel, dim3((unsigned)nblk), thr, 0, st, reinterpret_cast<const int*>(ws + lay.off_c),
                       lay.m_pad, m, n, row_blocks, ops[0].vaux, ops[1].vaux);
    shifts(2, plan.budget2, plan.budget2, -d, d);
    xbits[0] = plan.budget2 / 2 + 7 - d;  // |x'| < 2^(e + 1 + sa) <= 2^(floor(b/2) + 6 -+ d)
    xbits[1] = plan.budget2 / 2 + 7 + d;
  } else if (shift_mode == OZ2_SHIFT_CAUCHY_SCHWARZ) {
    fill(ops[0].vaux, n_aux);
    for (int x = 0; x < nops; ++x) launch_norm(ops[x], st);
    const int beta_a = plan.beta - d, beta_b = d == 0 ? plan.beta : plan.budget2 - beta_a;
    shifts(1, beta_a, beta_b, 0, 0);
    xbits[0] = beta_a + 1;
    xbits[1] = beta_b + 1;
  } else {
    const int kappa_a = plan.kappa - d, kappa_b = d == 0 ? plan.kappa : plan.kappa_sum - kappa_a;
    shifts(0, kappa_a, kappa_b, 0, 0);
    xbits[0] = kappa_a;
    xbits[1] = kappa_b;
  }
  const int kinds[2] = {xbits[0] > 75 ? 1 : 0, xbits[1] > 75 ? 1 : 0};
  if (strassen) {
    // general products only: the planes are the seven block combinations per modulus of the Strassen form
    if (!B || tri_a || tri_b) return hipErrorInvalidValue;
    return oz2_launch_strassen_convert(transa, transb, m, n, k, A, lda, B, ldb, plan, kinds, lay, ws, st);
  }
  if (hipError_t e = launch_convert(ops, nops, kinds, conv, fin, st); e != hipSuccess) return e;
  return hipGetLastError();
}

void oz2_host_residues_impl(const Oz2ConvConsts& c, double a, int shift, int8_t* out) {
  if (c.two_level) {
    Oz2Split s = oz2_scale_trunc_split<true>(a, shift);
    for (int t = 0; t < c.N; ++t) out[t] = (int8_t)(oz2_sym_residue<true>(s, c.p[t], c.inv_p[t], c.c32[t], c.c64[t]) & 0xff);
  } else {
    Oz2Split s = oz2_scale_trunc_split<false>(a, shift);
    for (int t = 0; t < c.N; ++t) out[t] = (int8_t)(oz2_sym_residue<false>(s, c.p[t], c.inv_p[t], c.c32[t], c.c64[t]) & 0xff);
  }
}
