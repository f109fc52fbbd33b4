// One level of Strassen's recursion applied to Algorithm 1 line 6, inside every residue ring.
//
// Line 6 only needs C'_t = A'_t B'_t modulo p_t.  Split A' and B' into 2 x 2 blocks (row / inner-dimension
// halves of mh, nh, kh elements, each a whole number of GEMM tiles; the matrices are zero padded up to twice
// those).  Modulo p_t the seven products
//   M1 = (A11 + A22)(B11 + B22)   M2 = (A21 + A22) B11     M3 = A11 (B12 - B22)    M4 = A22 (B21 - B11)
//   M5 = (A11 + A12) B22          M6 = (A21 - A11)(B11 + B12)                       M7 = (A12 - A22)(B21 + B22)
// give C11 = M1 + M4 - M5 + M7, C12 = M3 + M5, C21 = M2 + M4, C22 = M1 - M2 + M3 + M6.  Sums and differences of
// residues are reduced modulo p_t again, so every operand still fits INT8 and every product is an ordinary
// INT8 GEMM of half the size in each dimension: 7/8 of the matrix-core work of the plain form, for 7/4 of
// its plane traffic in the conversion and in the CRT pass.  All of it is integer arithmetic modulo p_t, so
// the residues c''_t, and with them X and C, are the same numbers as in the plain form.
//
// This file holds the two memory-bound ends: the conversion that writes the seven operand planes per modulus
// and the CRT pass that recombines the seven product planes.  The products themselves are the GEMM kernel of
// stage 2 run over 7 N planes.
#include "oz2_math.h"

namespace {

constexpr int kThreads = 256;
constexpr int kBlkRows = OZ2_TILE_M;  // plane layout of the GEMM: blocks of 256 rows x 64 bytes
constexpr int kBlkK = OZ2_TILE_K;
static_assert(OZ2_TILE_M == 256 && OZ2_TILE_N == 256 && OZ2_TILE_K == 64, "plane layout is 256 x 64 blocks");

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// Arithmetic modulo p on pairs of 16-bit lanes holding values in [0, p), p <= 256.  A sum a + b lies in [0, 2p):
// subtracting p wraps around to a large 16-bit value exactly when the sum was already below p, so the smaller
// of the two is the reduced sum.  A difference a - b wraps when it is negative, and adding p undoes the wrap.
__device__ __forceinline__ u16x2 add_mod(u16x2 a, u16x2 b, u16x2 p) {
  const u16x2 s = a + b;
  return __builtin_elementwise_min(s, (u16x2)(s - p));
}
__device__ __forceinline__ u16x2 sub_mod(u16x2 a, u16x2 b, u16x2 p) {
  const u16x2 d = a - b;
  return __builtin_elementwise_min(d, (u16x2)(d + p));
}
// a + b + c - d modulo p: a + b + c + (p - d) lies in (0, 4p), two conditional subtractions bring it below p
__device__ __forceinline__ u16x2 sum4_mod(u16x2 a, u16x2 b, u16x2 c, u16x2 d, u16x2 p, u16x2 p2) {
  u16x2 s = (a + b) + (c + (p - d));
  s = __builtin_elementwise_min(s, (u16x2)(s - p2));
  return __builtin_elementwise_min(s, (u16x2)(s - p));
}
__device__ __forceinline__ u16x2 as_pair(unsigned w) { return __builtin_bit_cast(u16x2, w); }
__device__ __forceinline__ unsigned as_word(u16x2 v) { return __builtin_bit_cast(unsigned, v); }

// ---------------------------------------------------------------------------------------------------
// Conversion.  An operand is a set of vectors (rows of op(A), columns of op(B)) of length k; X[a][b] is its
// block of vector half a and inner-dimension half b.  A workgroup takes the same 16 vectors x 64 inner
// positions of all four blocks: wave q copies block q into LDS with coalesced reads (lanes along whichever of
// the two directions is contiguous in memory), then every thread holds four consecutive inner positions of
// one vector in each block, forms their residues, the seven combinations, and writes four bytes per plane;
// the 16 lanes of a vector write its 64 bytes of the GEMM's block layout, a wave 256 contiguous bytes.
// Any representative in [-128, 127] serves as an INT8 operand: a value v in [0, p) is stored as v when it is
// below 128 and as v - p otherwise, i.e. its low byte plus 256 - p.
// ---------------------------------------------------------------------------------------------------
constexpr int kVecs = 16;
constexpr int kPitch = 68;  // doubles per vector in LDS: 64 + 4 keeps a thread's four values 32-byte aligned
constexpr int kTileDoubles = 4 * kVecs * kPitch;

struct StrassenJob {
  const double* X;
  int64_t ld, nvec, k;   // extent of the operand: nvec vectors of length k
  int64_t vh, kh;        // halves (multiples of 256 and of 64)
  const int* shifts;     // per vector, 2 vh entries readable
  int8_t* planes;        // 7 N planes of vh x kh bytes, plane 7 t + s = combination s of modulus t
  int strided;           // 1: element (v, l) at X[v + l ld]; 0: at X[l + v ld]
  int side;              // 0: first operand (A), 1: second operand (B)
  unsigned gx, nblk;
};

template <int KIND>
__device__ __forceinline__ void strassen_convert(const StrassenJob& j, const Oz2ConvConsts& cc, double* tile,
                                                 unsigned bx, unsigned by) {
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t r0 = (int64_t)bx * kVecs;   // first vector of the group inside a half
  const int64_t l0 = (int64_t)by * kBlkK;   // first inner position inside a half
  {
    // wave q copies block q = 2a + b
    const int a = wv >> 1, b = wv & 1;
    double* dstq = tile + wv * (kVecs * kPitch);
    if (j.strided) {
      const int vv = lane & 15, c0 = lane >> 4;
      const int64_t v = r0 + vv + a * j.vh;
      const double* src = j.X + v;
#pragma unroll 8
      for (int it = 0; it < kBlkK / 4; ++it) {
        const int lc = 4 * it + c0;
        const int64_t l = l0 + lc + b * j.kh;
        dstq[vv * kPitch + lc] = (v < j.nvec && l < j.k) ? __builtin_nontemporal_load(src + l * j.ld) : 0.0;
      }
    } else {
      const int64_t l = l0 + lane + b * j.kh;
      const double* src = j.X + l;
#pragma unroll 8
      for (int vv = 0; vv < kVecs; ++vv) {
        const int64_t v = r0 + vv + a * j.vh;
        dstq[vv * kPitch + lane] = (v < j.nvec && l < j.k) ? __builtin_nontemporal_load(src + v * j.ld) : 0.0;
      }
    }
  }
  __syncthreads();

  constexpr bool TWO_LEVEL = KIND == 1;
  const int vv = threadIdx.x >> 4, g = threadIdx.x & 15;
  const int64_t rq = r0 + vv;
  Oz2Split xs[2][2][4];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int64_t v = rq + a * j.vh;
    const int shift = v < j.nvec ? j.shifts[v] : 0;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const double* mine = tile + ((2 * a + b) * kVecs + vv) * kPitch + 4 * g;
#pragma unroll
      for (int u = 0; u < 4; ++u) xs[a][b][u] = oz2_scale_trunc_split<TWO_LEVEL>(mine[u], shift);
    }
  }
  const size_t plane_stride = (size_t)j.vh * j.kh;
  // byte offset of this thread's four bytes inside a plane (below 2^32: checked by the launcher); the plane's
  // base address is the same for the whole workgroup
  const unsigned off = (unsigned)((size_t)(rq / kBlkRows) * kBlkRows * j.kh + (size_t)by * (kBlkRows * kBlkK) +
                                  (rq % kBlkRows) * kBlkK + 4 * g);
  int8_t* plane = j.planes;
  const int side = j.side;
  for (int t = 0; t < cc.N; ++t) {
    const double p = cc.p[t], ip = cc.inv_p[t], c32 = cc.c32[t], c64 = cc.c64[t];
    const unsigned short ps = (unsigned short)(int)p;
    const u16x2 P = {ps, ps};
    // residues in [0, p) as pairs: x[a][b][h] = inner positions 2h, 2h + 1 of block (a, b)
    u16x2 x[2][2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int re = oz2_sym_residue<TWO_LEVEL>(xs[a][b][2 * h], p, ip, c32, c64);
          const int ro = oz2_sym_residue<TWO_LEVEL>(xs[a][b][2 * h + 1], p, ip, c32, c64);
          const u16x2 s = as_pair(((unsigned)re & 0xffffu) | ((unsigned)ro << 16));  // symmetric, wrapped when negative
          x[a][b][h] = __builtin_elementwise_min(s, (u16x2)(s + P));
        }
    u16x2 c[7][2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const u16x2 x00 = x[0][0][h], x01 = x[0][1][h], x10 = x[1][0][h], x11 = x[1][1][h];
      if (side == 0) {
        // A_pq = X[p][q]:  A11 + A22, A21 + A22, A11, A22, A11 + A12, A21 - A11, A12 - A22
        c[0][h] = add_mod(x00, x11, P);
        c[1][h] = add_mod(x10, x11, P);
        c[2][h] = x00;
        c[3][h] = x11;
        c[4][h] = add_mod(x00, x01, P);
        c[5][h] = sub_mod(x10, x00, P);
        c[6][h] = sub_mod(x01, x11, P);
      } else {
        // B_pq = X[q][p] (vectors are columns):  B11 + B22, B11, B12 - B22, B21 - B11, B22, B11 + B12, B21 + B22
        c[0][h] = add_mod(x00, x11, P);
        c[1][h] = x00;
        c[2][h] = sub_mod(x10, x11, P);
        c[3][h] = sub_mod(x01, x00, P);
        c[4][h] = x11;
        c[5][h] = add_mod(x00, x10, P);
        c[6][h] = add_mod(x01, x11, P);
      }
    }
    const unsigned short adj = (unsigned short)(256 - (int)p);
    const u16x2 ADJ = {adj, adj};
#pragma unroll
    for (int s = 0; s < 7; ++s) {
      const u16x2 f0 = c[s][0] + (c[s][0] >> 7) * ADJ;   // low bytes: v, or v - p when v >= 128
      const u16x2 f1 = c[s][1] + (c[s][1] >> 7) * ADJ;
      const unsigned w = __builtin_amdgcn_perm(as_word(f1), as_word(f0), 0x06040200u);
      __builtin_nontemporal_store(w, reinterpret_cast<unsigned*>(plane + off));  // written once, read by a later kernel
      plane += plane_stride;
    }
  }
}

template <int KA, int KB>
__global__ void __launch_bounds__(kThreads) strassen_convert_kernel(const StrassenJob ja, const StrassenJob jb,
                                                                    const Oz2ConvConsts cc) {
  __shared__ __attribute__((aligned(32))) double tile[kTileDoubles];
  if (blockIdx.x < ja.nblk) {
    strassen_convert<KA>(ja, cc, tile, blockIdx.x % ja.gx, blockIdx.x / ja.gx);
  } else {
    const unsigned id = blockIdx.x - ja.nblk;
    strassen_convert<KB>(jb, cc, tile, id % jb.gx, id / jb.gx);
  }
}

// ---------------------------------------------------------------------------------------------------
// CRT pass.  Product plane 7 t + s holds M_{s+1} modulo p_t as bytes in [0, p_t), element (i, j) of the
// mh x nh grid at j mh + i.  A thread takes two consecutive rows i of one column j of that grid, i.e. the
// elements (i, j), (i, j + nh), (i + mh, j), (i + mh, j + nh) of C: per modulus it reads seven 16-bit words,
// recombines them modulo p_t into the residues c''_t of the four blocks, and accumulates those exactly as the
// plain CRT kernel does (Algorithm 1 lines 9-11).
// ---------------------------------------------------------------------------------------------------
constexpr int kCrtRows = 2;  // rows per thread: 8 elements of C, 32 accumulators of two registers at four limbs
static_assert(kCrtRows == 2, "the kernel below loads two bytes per plane and stores two doubles per block");
template <int L>
__global__ void __launch_bounds__(kThreads) strassen_crt_kernel(const uint8_t* __restrict__ planes, int64_t mh, int64_t nh,
                                                                const int* __restrict__ sa, const int* __restrict__ sb,
                                                                double* __restrict__ C, int64_t ldc, int64_t m, int64_t n,
                                                                const double alpha, const double beta,
                                                                const unsigned long long* __restrict__ skip_flag,
                                                                const unsigned row_chunks, const Oz2CrtConsts cc) {
  if (skip_flag != nullptr && *skip_flag != 0ull) return;
  constexpr int R = kCrtRows;
  // consecutive workgroups walk down a column of the half grid: their reads of a plane are adjacent
  const int64_t jq = blockIdx.x / row_chunks;
  const int64_t i0 = ((int64_t)(blockIdx.x % row_chunks) * kThreads + threadIdx.x) * R;
  if (i0 >= mh || i0 >= m) return;
  // two bytes = rows i0, i0 + 1 of one product plane (mh is a multiple of 256 and i0 is even: aligned)
  const unsigned short* src = reinterpret_cast<const unsigned short*>(planes + (size_t)jq * mh + i0);
  const size_t stride = (size_t)mh * nh / 2;  // 16-bit words per plane

  double S[4][R][L];  // block 2a + b (row half a, column half b)
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int l = 0; l < L; ++l) S[q][r][l] = 0.0;

  // the seven words of two moduli are in flight while one modulus is worked on; the planes are read once
  // (non-temporal loads: measured 2-3 % on this kernel and on the conversion's stores)
  constexpr int kAhead = 2;
  const int N = cc.N;
  unsigned nxt[kAhead][7];
#pragma unroll
  for (int d = 0; d < kAhead; ++d) {
    const int td = d < N ? d : N - 1;
#pragma unroll
    for (int s = 0; s < 7; ++s) nxt[d][s] = __builtin_nontemporal_load(src + (size_t)(7 * td + s) * stride);
  }
  for (int t0 = 0; t0 < N; t0 += kAhead) {
    unsigned cur[kAhead][7];
#pragma unroll
    for (int d = 0; d < kAhead; ++d)
#pragma unroll
      for (int s = 0; s < 7; ++s) cur[d][s] = nxt[d][s];
    if (t0 + kAhead < N) {
#pragma unroll
      for (int d = 0; d < kAhead; ++d) {
        const int tn = t0 + kAhead + d < N ? t0 + kAhead + d : N - 1;  // past the end: a harmless repeat
#pragma unroll
        for (int s = 0; s < 7; ++s) nxt[d][s] = __builtin_nontemporal_load(src + (size_t)(7 * tn + s) * stride);
      }
    }
#pragma unroll
    for (int d = 0; d < kAhead; ++d) {
      const int t = t0 + d;
      if (t < N) {
        const unsigned short ps = (unsigned short)(int)cc.p[t];
        const u16x2 P = {ps, ps};
        u16x2 M[7];
#pragma unroll
        for (int s = 0; s < 7; ++s) M[s] = as_pair(__builtin_amdgcn_perm(0u, cur[d][s], 0x0c010c00u));  // bytes -> 16-bit lanes
        const u16x2 P2 = P + P;
        u16x2 c[4];
        c[0] = sum4_mod(M[0], M[3], M[6], M[4], P, P2);  // C11 = M1 + M4 + M7 - M5
        c[1] = add_mod(M[2], M[4], P);                   // C12 = M3 + M5
        c[2] = add_mod(M[1], M[3], P);                   // C21 = M2 + M4
        c[3] = sum4_mod(M[0], M[2], M[5], M[1], P, P2);  // C22 = M1 + M3 + M6 - M2
        double res[4][R];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          res[q][0] = (double)(unsigned)c[q].x;
          res[q][1] = (double)(unsigned)c[q].y;
        }
#pragma unroll
        for (int l = 0; l < L; ++l) {
          const double w = cc.w[t][l];
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int r = 0; r < R; ++r) S[q][r][l] = fma(res[q][r], w, S[q][r][l]);
        }
      }
    }
  }

#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int64_t ib = i0 + (q >> 1) * mh, j = jq + (q & 1) * nh;
    if (ib >= m || j >= n) continue;
    const int sbj = sb[j];
    double* dst = C + ib + j * ldc;
    double out[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      int e2;
      const double x = oz2_crt_reduce<L>(S[q][r], cc, &e2);
      out[r] = ldexp(x, e2 - sa[ib + r] - sbj);  // sa holds 2 mh entries: readable
    }
    if (alpha != 1.0 || beta != 0.0) {
      // C := alpha * P + beta * C with one rounding of beta * C and one fused multiply-add; C is not read when
      // beta is zero (BLAS convention)
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const double tt = (beta == 0.0 || ib + r >= m) ? 0.0 : beta * dst[r];
        out[r] = fma(alpha, out[r], tt);
      }
    }
    if (ib + R <= m && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
      *reinterpret_cast<double2*>(dst) = make_double2(out[0], out[1]);
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (ib + r < m) dst[r] = out[r];
    }
  }
}

}  // namespace

// Planes of both operands in the Strassen form.  lay holds the padded extents (twice the halves) and the plane
// regions; kinds: 0 / 1 = one- / two-level split of an element per operand (see the plain conversion).
hipError_t oz2_launch_strassen_convert(int transa, int transb, int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                       const double* B, int64_t ldb, const Oz2Plan& plan, const int* kinds,
                                       const Oz2Layout& lay, char* ws, hipStream_t st) {
  const int64_t mh = lay.m_pad / 2, nh = lay.n_pad / 2, kh = lay.k_pad / 2;
  if (mh % kBlkRows || nh % kBlkRows || kh % kBlkK) return hipErrorInvalidValue;
  if (mh * kh >= ((int64_t)1 << 32) || nh * kh >= ((int64_t)1 << 32)) return hipErrorInvalidValue;  // 32-bit offsets in a plane
  StrassenJob job[2];
  job[0] = {A, lda, m, k, mh, kh, reinterpret_cast<const int*>(ws + lay.off_sa), reinterpret_cast<int8_t*>(ws + lay.off_a),
            transa == 0 ? 1 : 0, 0, 0u, 0u};
  job[1] = {B, ldb, n, k, nh, kh, reinterpret_cast<const int*>(ws + lay.off_sb), reinterpret_cast<int8_t*>(ws + lay.off_b),
            transb != 0 ? 1 : 0, 1, 0u, 0u};
  int64_t total = 0;
  for (int x = 0; x < 2; ++x) {
    const int64_t gx = job[x].vh / kVecs, gy = job[x].kh / kBlkK;
    total += gx * gy;
    if (total >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    job[x].gx = (unsigned)gx;
    job[x].nblk = (unsigned)(gx * gy);
  }
  const dim3 grid((unsigned)total), thr(kThreads);
#define OZ2_CONV(KA, KB) hipLaunchKernelGGL((strassen_convert_kernel<KA, KB>), grid, thr, 0, st, job[0], job[1], plan.conv)
  if (kinds[0] == 0 && kinds[1] == 0)
    OZ2_CONV(0, 0);
  else if (kinds[0] == 0)
    OZ2_CONV(0, 1);
  else if (kinds[1] == 0)
    OZ2_CONV(1, 0);
  else
    OZ2_CONV(1, 1);
#undef OZ2_CONV
  return hipGetLastError();
}

hipError_t oz2_launch_strassen_crt(int64_t m, int64_t n, double alpha, double beta, double* C, int64_t ldc,
                                   const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int check_flag, hipStream_t st) {
  const int64_t mh = lay.m_pad / 2, nh = lay.n_pad / 2;
  const unsigned long long* skip = check_flag ? reinterpret_cast<const unsigned long long*>(ws + lay.off_flags) : nullptr;
  const uint8_t* planes = reinterpret_cast<const uint8_t*>(ws + lay.off_c);
  const int* sa = reinterpret_cast<const int*>(ws + lay.off_sa);
  const int* sb = reinterpret_cast<const int*>(ws + lay.off_sb);
  const int64_t rows = mh < m ? mh : m;  // rows of the half grid that hold an element of C
  const int64_t cols = nh < n ? nh : n;
  const int64_t row_chunks = (rows + kThreads * kCrtRows - 1) / (kThreads * kCrtRows);
  if (row_chunks * cols >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
  dim3 grid((unsigned)(row_chunks * cols));
  switch (plan.crt.L) {
#define OZ2_CASE(LL)                                                                                                 \
  case LL:                                                                                                           \
    hipLaunchKernelGGL((strassen_crt_kernel<LL>), grid, dim3(kThreads), 0, st, planes, mh, nh, sa, sb, C, ldc, m, n, \
                       alpha, beta, skip, (unsigned)row_chunks, plan.crt);                                           \
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
