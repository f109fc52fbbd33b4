// Internal declarations shared by the translation units of liboz2 (host side + kernel launchers).
#ifndef OZ2_INTERNAL_H
#define OZ2_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/oz2.h"

#define OZ2_MIN_N 2
#define OZ2_MAX_N 26   // greedy table 256 ... 139; M < 2^200
#define OZ2_MAX_L 5    // 40-bit limbs of M
#define OZ2_MAX_PLANES (7 * OZ2_MAX_N)  // planes of one GEMM launch: seven per modulus in the Strassen form
#define OZ2_LIMB_BITS 40

// GEMM tiling (stage 2): workgroup tile TILE_M x TILE_N, k-tile TILE_K bytes.
#define OZ2_TILE_M 256
#define OZ2_TILE_N 256
#define OZ2_TILE_K 64

// Constants of the conversion kernels (Algorithm 1 lines 2-5), passed by value as a kernel argument.
struct Oz2ConvConsts {
  int N;
  int two_level;             // 1 when kappa is too large for the one-level 2^32 split
  double p[OZ2_MAX_N];       // moduli as doubles
  double inv_p[OZ2_MAX_N];   // RN(1/p)
  double c32[OZ2_MAX_N];     // 2^32 reduced to the symmetric range modulo p
  double c64[OZ2_MAX_N];     // 2^64 likewise
};

// Constants of the CRT kernel (Algorithm 1 lines 7-10).
struct Oz2CrtConsts {
  int N;
  int L;                               // number of 40-bit limbs: 40*L >= bit length of M
  double p[OZ2_MAX_N];
  double inv_p[OZ2_MAX_N];             // RN(1/p)
  double half_inv_p[OZ2_MAX_N];        // 0.5 * inv_p
  double w[OZ2_MAX_N][OZ2_MAX_L];      // limbs of W_t = (M/p_t) * ((M/p_t)^-1 mod p_t), each < 2^40
  double mlimb[OZ2_MAX_L];             // limbs of M
  double mhalf[OZ2_MAX_L];             // limbs of M/2
  double rinv[OZ2_MAX_L];              // RN(2^(40 l) / M)
};

// Constants of the matrix-core form of lines 8-9 (at most 16 moduli, M < 2^128): the weights in the symmetric range,
// Ws_t = W_t or W_t - M with |Ws_t| <= M/2, as sixteen balanced base-256 digits each,
//   Ws_t = sum_i dig[i][t] 256^i,  dig in [-128, 127],
// so that one INT8 MFMA forms sum_t (c''_t - 128) dig[i][t] for all sixteen digits of 64 output elements at once;
// init[i] = 128 sum_t dig[i][t] makes up for the 128: sum_t c''_t dig[i][t] = (MFMA result) + init[i].
struct Oz2CrtDigits {
  int valid;            // 1 when the plan has them (N <= 16)
  int init[16];
  int8_t dig[16][16];   // [digit][modulus], zero beyond N
  double sinit[4];      // sum_i init[i] 256^i as 40-bit limbs (digits 5 l .. 5 l + 4 in limb l, the rest in the top one
                        // of the L in use): added after the MFMA, whose accumulator then starts at the inline zero
};

struct Oz2Plan {
  int N;
  int kappa;
  int beta;     // largest beta with 4^beta <= M/2 - 1 (Cauchy-Schwarz shift mode)
  int budget2;  // largest b with 2^b <= M/2 - 1 (INT8-product shift mode)
  int kappa_sum;  // largest S with k * 2^S <= M/2 - 1 (Section 3, first budget equation); 2 kappa or 2 kappa + 1
  int moduli[OZ2_MAX_N];
  Oz2ConvConsts conv;
  Oz2CrtConsts crt;
  Oz2CrtDigits digits;
};

// Host constants (oz2_host.cpp).  Returns 0, or -1 for an unsupported N, or 2 when kappa < 1.
int oz2_build_plan(int N, int64_t k, Oz2Plan* plan);
int oz2_table_moduli(int N, int* out);
int oz2_table_kappa(int N, int64_t k);
int oz2_table_kappa_sum(int N, int64_t k);

struct Oz2Layout {
  int64_t m_pad, n_pad, k_pad;
  size_t off_rowmax, off_colmax, off_sa, off_sb, off_a, off_b, off_c, off_rownorm, off_colnorm, off_flags, total;
};
void oz2_make_layout(int64_t m, int64_t n, int64_t k, int N, int c_elem_bytes, Oz2Layout* lay);
// Layout of the Strassen form (UINT8 residue planes): the padded extents are twice the halves (multiples of 256,
// 256 and 64), and each plane region holds 7 N planes of a quarter of the padded area.
void oz2_make_layout_strassen(int64_t m, int64_t n, int64_t k, int N, Oz2Layout* lay);

// Kernel launchers.  Each returns hipSuccess or the launch error.
hipError_t oz2_launch_stage1(int transa, int transb, int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                             const double* B, int64_t ldb, int tri_a, int tri_b, const Oz2Plan& plan, int shift_mode,
                             int bit_split, int strassen, const Oz2Layout& lay, char* ws, hipStream_t st);
// Strassen form of line 6 (oz2_strassen.hip, oz2_stage2.hip): operand planes, the 7 N products, CRT pass
hipError_t oz2_launch_strassen_convert(int transa, int transb, int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                                       const double* B, int64_t ldb, const Oz2Plan& plan, const int* kinds,
                                       const Oz2Layout& lay, char* ws, hipStream_t st);
hipError_t oz2_launch_strassen_gemm(const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int64_t kblock, int check_flag,
                                    hipStream_t st);
hipError_t oz2_launch_strassen_crt(int64_t m, int64_t n, double alpha, double beta, double* C, int64_t ldc,
                                   const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int check_flag, hipStream_t st);
// One-time device set-up of the GEMM kernels (function attributes, compute-unit count); also done lazily by the
// first launch.
hipError_t oz2_gemm_setup();
// Bound of one wait of the GEMM's round synchronisation in polls (0 switches the synchronisation off), and the
// clearing of its counters for a GEMM that no stage 1 precedes.
void oz2_gemm_set_sync_spins(int spins);
hipError_t oz2_launch_clear_sync(const Oz2Layout& lay, char* ws, hipStream_t st);

// Inner-dimension range of a tile when one operand is triangular (TRMM shape), in units of diagonal blocks:
//   UPTO_ROW / FROM_ROW: the first operand is lower / upper triangular (only l <= i / l >= i contribute);
//   FROM_COL / UPTO_COL: the second operand is lower / upper triangular (only l >= j / l <= j contribute).
#define OZ2_KRANGE_ALL 0
#define OZ2_KRANGE_UPTO_ROW 1
#define OZ2_KRANGE_FROM_ROW 2
#define OZ2_KRANGE_FROM_COL 3
#define OZ2_KRANGE_UPTO_COL 4

// check_flag != 0: return at once on the device when stage 1 found a non-finite input.
// triangle: 0 = general product; 1 / 2 = symmetric product op(A) op(A)^T (B's planes are A's), only the tiles of
// the lower / upper triangle are computed
hipError_t oz2_launch_stage2(const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int64_t kblock, int residue_u8,
                             int triangle, int krange, int check_flag, hipStream_t st);
// P = A''B'' of the INT8-product shift mode: bound planes in the slots of residue plane 0 -> INT32 in the slot of
// product plane 0.  Exact for k_pad * 64 * 64 < 2^31.
hipError_t oz2_launch_bound_gemm(const Oz2Layout& lay, char* ws, bool symmetric, hipStream_t st);
// check_flag != 0: do nothing when stage 1 found a non-finite input (the fallback forms C instead)
hipError_t oz2_launch_stage3(int64_t m, int64_t n, double alpha, double beta, double* C, int64_t ldc,
                             const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int residue_u8, int check_flag,
                             int triangle, hipStream_t st);
// Stage 3 on UINT8 residue planes of a general product and, in the same launch, the blocks of the FP64 fallback
// below: stage 1's flag decides on the device which of the two sets of blocks forms C.  For small problems.
hipError_t oz2_launch_stage3_or_fallback(int transa, int transb, int64_t m, int64_t n, int64_t k, double alpha,
                                         const double* A, int64_t lda, const double* B, int64_t ldb, double beta, double* C,
                                         int64_t ldc, const Oz2Plan& plan, const Oz2Layout& lay, char* ws, hipStream_t st);
// C := alpha * op(A) * op(B) + beta * C in plain FP64, only if *flag != 0 (checked on the device)
// tri_a / tri_b: triangular structure of the stored A / B (0 = full).  C must not overlap A or B.
hipError_t oz2_launch_fallback(const unsigned long long* flag, int transa, int transb, int64_t m, int64_t n, int64_t k,
                               double alpha, const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
                               double* C, int64_t ldc, int triangle, int tri_a, int tri_b, hipStream_t st);
// dst(m x n, ld) := src(m x n, contiguous columns of length m), only if *flag != 0
hipError_t oz2_launch_copy_if(const unsigned long long* flag, int64_t m, int64_t n, const double* src, double* dst,
                              int64_t ld, hipStream_t st);
hipError_t oz2_launch_scale_c(int64_t m, int64_t n, double beta, double* C, int64_t ldc, int triangle, hipStream_t st);

hipError_t oz2_launch_mfma_calibration(int workgroups, int iters, int random_operands, int* sink, long long* clocks,
                                       hipStream_t st);

// The library's own static device buffer (oz2_static.hip): address on the current device and size.  The first call
// on a device looks the address up; nothing is ever allocated.
hipError_t oz2_static_scratch(char** ptr, size_t* bytes);

// Host instantiations of the device math (oz2_stage1.hip / oz2_stage3.hip), for unit tests.
void oz2_host_residues_impl(const Oz2ConvConsts& c, double a, int shift, int8_t* out);
double oz2_host_crt_impl(const Oz2CrtConsts& c, const int32_t* cprod);
// the same element by the digit route of the matrix-core CRT kernel (res: num_moduli residues in [0, p_t))
double oz2_host_crt_digits_impl(const Oz2CrtConsts& c, const Oz2CrtDigits& d, const uint8_t* res);

#endif
