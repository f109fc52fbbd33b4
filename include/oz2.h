/* oz2.h -- C ABI of the MI355X (gfx950) library for Ozaki scheme II: FP64 matrix multiplication
 * C = A*B emulated with INT8 matrix products and the Chinese Remainder Theorem
 * (arXiv 2504.08009, Algorithm 1 and Sections 2.3, 3, 3.1).
 *
 * Conventions for every call
 *   - Matrices are column-major with leading dimensions (BLAS convention).
 *   - A, B, C and the workspace are DEVICE pointers owned by the caller; the library never frees them.
 *     A and B are read-only, C is overwritten, A/B must not overlap C or the workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue work;
 *     they return without waiting for the GPU, allocate nothing and record no memset, so a call can be captured
 *     into a HIP graph (after oz2_init or one earlier call).
 *   - Return value: 0 success; -i = the i-th argument is invalid (1-based, LAPACK style);
 *     OZ2_ERR_WORKSPACE (1) workspace missing or too small; OZ2_ERR_BUDGET (2) the moduli product is
 *     too small for this inner dimension (kappa < 1), or the inner dimension too long for the shift mode; OZ2_ERR_HIP (3) a HIP call failed.
 *     Nothing is printed and nothing throws across this boundary.
 *   - The method covers finite inputs (Section 3.1, last paragraph).  Infinities and NaNs in A or B are detected
 *     and handled by an FP64 fallback (oz2_set_nonfinite_check, on by default).  Signed zeros need no handling:
 *     -0 in A or B counts as zero and an emulated zero is +0, which is what an FP64 sum that starts from +0 gives
 *     for products that are all zero, whatever their signs; a result that underflows keeps its sign.  Results
 *     beyond the FP64 range become infinities as in FP64.
 *   - One GPU: the library is used from one device per process (kernel attributes are set once).
 *   - The library keeps one workspace registration per process (oz2_set_workspace).  Calls that use it
 *     must not overlap in time on different streams.
 */
#ifndef OZ2_H
#define OZ2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OZ2_OK 0
#define OZ2_ERR_WORKSPACE 1
#define OZ2_ERR_BUDGET 2
#define OZ2_ERR_HIP 3
#define OZ2_ERR_STATIC_LIMIT 4 /* oz2_dgemm_static only: the problem needs more than OZ2_STATIC_SCRATCH_BYTES */

/* Size of the library's own static workspace (one per GPU, held until the process ends); see oz2_dgemm_static. */
#define OZ2_STATIC_SCRATCH_BYTES (64u << 20)

#define OZ2_PRODUCT_INT32 0      /* stage 2 writes the INT32 products C'_t (Algorithm 1 line 6) */
#define OZ2_PRODUCT_RESIDUE_U8 1 /* stage 2 writes C''_t = C'_t mod p_t as UINT8 (lines 6 and 7 together); default */

#define OZ2_GEMM_AUTO (-1)    /* Strassen form for large general products when the workspace allows it; default */
#define OZ2_GEMM_CLASSICAL 0  /* Algorithm 1 line 6 as printed: one INT8 product of the full size per modulus */
#define OZ2_GEMM_STRASSEN 1   /* one level of Strassen's recursion inside every residue ring: 7 products of half size */

#define OZ2_SHIFT_MAX 0            /* shifts from row/column maxima: the simple bound of Section 3 */
#define OZ2_SHIFT_CAUCHY_SCHWARZ 1 /* shifts from row/column 2-norms: Section 4.1, the "fast" variant */
#define OZ2_SHIFT_INT8_PRODUCT 2   /* shifts from an INT8 product of upper bounds: Section 4.1, the "accu" variant */

/* One-time set-up on the current device (kernel attributes, compute-unit count, address of the static workspace
 * of oz2_dgemm_static).  The first call that launches the GEMM does the same by itself; call this first when that
 * call would otherwise be made under stream capture, where attributes cannot be set.  Returns 0 or OZ2_ERR_HIP. */
int oz2_init(void);

/* Smallest and largest supported number of moduli (Section 3.1: the table starts at s = 2). */
int oz2_min_moduli(void);
int oz2_max_moduli(void);

/* Moduli table and bit budget (Section 3.1, "largest possible" pairwise-coprime values <= 256, taken
 * greedily downwards from 256; Section 3, the second equation for k_A = k_B evaluated with integers:
 * the largest kappa with k * 4^kappa <= M/2 - 1).
 * moduli_out: host array of num_moduli ints, or NULL.  kappa_out: host int, or NULL; receives -1 when
 * even kappa = 0 breaks the bound.  k >= 1.  Returns 0 or a negative argument code. */
int oz2_get_moduli(int num_moduli, int* moduli_out, int* kappa_out, int64_t k);

/* Smallest number of moduli whose bit budget kappa (same definition as in oz2_get_moduli) reaches `bits` for
 * inner dimension k: with it every entry of a row (column) keeps at least `bits` bits below the row's
 * (column's) largest one under the default shift selection (Section 3.1 works this out for 53 bits: sixteen moduli
 * cover the inner dimensions 1024, 4096 and 16384).  Returns that count, 0 if even oz2_max_moduli() does not reach it, -1 / -2 for k < 1 /
 * bits < 1. */
int oz2_moduli_for_bits(int64_t k, int bits);

/* Workspace size in bytes for a problem, 0 on invalid arguments.  Holds the shift vectors, the INT8
 * residue planes of A and B and the product planes (Algorithm 1, lines 1-7).  oz2_workspace_bytes is enough
 * for either product format (it is the INT32 size); oz2_workspace_bytes_for gives the exact size for one
 * format -- with OZ2_PRODUCT_RESIDUE_U8, the default, about half as much at large sizes (12 instead of 24 GiB at
 * m = n = k = 16384 with 16 moduli).  Calls check the registered size against the format in force. */
size_t oz2_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_moduli);
size_t oz2_workspace_bytes_for(int64_t m, int64_t n, int64_t k, int num_moduli, int product_format);

/* Register a caller-owned device buffer (256-byte aligned) as the workspace for later calls.
 * NULL/0 unregisters.  Returns 0 or -1 (bad alignment or NULL with nonzero size). */
int oz2_set_workspace(void* dev_ptr, size_t bytes);

/* Where each intermediate lives inside the workspace for the product format in force, so that a test can read
 * every stage's output.  This is the layout of the classical form of the products and of the staged entry points;
 * the Strassen form (oz2_set_gemm_algorithm) keeps the small arrays in this order on its own padded extents and
 * holds seven planes of a quarter of the padded area per modulus in each plane region.
 * offsets[0..9] (bytes from the workspace start):
 *   0 rowmax  : m_pad uint64, bit pattern of max_l |a_il| per row of A
 *   1 colmax  : n_pad uint64, same per column of B
 *   2 sa      : m_pad int32 shifts of A's rows      (Algorithm 1 line 1)
 *   3 sb      : n_pad int32 shifts of B's columns
 *   4 A planes: num_moduli x m_pad x k_pad int8 residues of A' (Algorithm 1 line 4), stored in contiguous
 *               blocks of 256 rows x 64 inner-dimension bytes: element (i, l) of plane t at byte
 *               ((t*m_pad + 256*(i/256)) * k_pad) + (l/64)*16384 + (i%256)*64 + (l%64)
 *   5 B planes: num_moduli x n_pad x k_pad int8 residues of B' (line 5), same blocking with the column
 *               index j of B in the place of i and n_pad in the place of m_pad
 *   6 C planes: num_moduli x n_pad x m_pad, plane t element (i,j) at index ((t*n_pad)+j)*m_pad + i; the
 *               elements are int32 products (OZ2_PRODUCT_INT32) or uint8 residues in [0, p_t)
 *               (OZ2_PRODUCT_RESIDUE_U8); the region holds at least 8 bytes per element of one plane
 *   7 rownorm : m_pad uint64, integer norm bound S_i of A's rows (Cauchy-Schwarz shift mode only)
 *   8 colnorm : n_pad uint64, same per column of B
 *   9 flags   : 32 uint64; word 0 is 1 after a stage 1 that found an infinity or a NaN in A or B, else 0
 * dims[0..2] = m_pad, n_pad, k_pad (m, n rounded up to 256, k to 64; padding holds zeros).
 * Returns 0 or a negative argument code. */
int oz2_workspace_layout(int64_t m, int64_t n, int64_t k, int num_moduli, size_t offsets[10], int64_t dims[3]);

/* The whole of Algorithm 1:  C := A*B  with num_moduli INT8 products.
 *   A: m x k, lda >= max(1,m);  B: k x n, ldb >= max(1,k);  C: m x n, ldc >= max(1,m).
 * m == 0 or n == 0: nothing to do.  k == 0: C := 0.  Needs a registered workspace of at least
 * oz2_workspace_bytes_for(m,n,k,num_moduli, format in force); with oz2_workspace_bytes_preferred(m,n,k,num_moduli)
 * large products take the faster Strassen form of line 6 (oz2_set_gemm_algorithm).  Row-major callers pass
 * (n,m,k,B,ldb,A,lda,C,ldc). */
int oz2_dgemm(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
              double* C, int64_t ldc, int num_moduli, void* stream);

/* oz2_dgemm for callers that cannot allocate device memory or register a workspace of their own: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * the same result, bit for bit, as oz2_dgemm under the settings in force; the intermediates (shift vectors,
 * residue planes, product planes) live in a static device array of OZ2_STATIC_SCRATCH_BYTES (64 MiB) that is
 * part of the library's code object, one copy per GPU.  The call allocates and frees nothing (its first use on
 * a device looks up the array's address; oz2_init does that ahead of time) and does not touch the registered
 * workspace.  A problem whose workspace -- oz2_workspace_bytes_for(m, n, k, num_moduli, format in force) --
 * exceeds the array returns OZ2_ERR_STATIC_LIMIT and enqueues nothing: with the default product format that
 * admits m = n = k = 1024 with up to 21 moduli (63 MiB).  The array keeps the last call's
 * contents; every call rewrites all it reads.  All calls on a GPU share the one array: calls that overlap in
 * time on one GPU (two streams, two threads) race -- serialise them.  Always the classical form of line 6. */
int oz2_dgemm_static(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
                     double* C, int64_t ldc, int num_moduli, void* stream);

/* BLAS-style general form:  C := alpha * op(A) * op(B) + beta * C,  op(X) = X for 'N', X^T for 'T' or 'C'.
 *   op(A) is m x k: A is stored m x k (lda >= max(1,m)) for 'N' and k x m (lda >= max(1,k)) otherwise;
 *   op(B) is k x n: B is stored k x n (ldb >= max(1,k)) for 'N' and n x k (ldb >= max(1,n)) otherwise.
 * The product P = op(A) op(B) is formed by Algorithm 1 exactly as in oz2_dgemm; then each element is
 * C_ij := fma(alpha, P_ij, beta * C_ij) (beta * C_ij rounded once; C is not read when beta == 0).  With
 * alpha == 1 and beta == 0 the result is P itself.  alpha == 0 or k == 0: C := beta * C, A and B are not
 * touched.  Argument codes are 1-based over this parameter list. */
int oz2_dgemm_ex(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha, const double* A, int64_t lda,
                 const double* B, int64_t ldb, double beta, double* C, int64_t ldc, int num_moduli, void* stream);

/* Symmetric rank-k update in BLAS form (Section 2.3: for structured products the GEMM of part 2-b becomes the
 * routine that fits, here the SYRK shape):
 *   trans 'N':        C := alpha * A * A^T + beta * C,  A is n x k, lda >= max(1,n);
 *   trans 'T' or 'C': C := alpha * A^T * A + beta * C,  A is k x n, lda >= max(1,k).
 * C is n x n; only its uplo ('L' or 'U') triangle is read and written.  A is converted once and its residue
 * planes serve as both operands; only the tiles of that triangle are multiplied, so stage 1 does half and
 * stage 2 about half of the work of oz2_dgemm_ex on (A, A^T).  Every written element equals what oz2_dgemm_ex
 * gives there (the product of the truncated integers is symmetric).  Workspace: oz2_workspace_bytes(n, n, k,
 * num_moduli).  Argument codes are 1-based over this parameter list. */
int oz2_dsyrk(char uplo, char trans, int64_t n, int64_t k, double alpha, const double* A, int64_t lda, double beta,
              double* C, int64_t ldc, int num_moduli, void* stream);

/* Triangular matrix product in BLAS form (Section 2.3, the TRMM shape), in place:
 *   side 'L': B := alpha * op(A) * B,  A is m x m;   side 'R': B := alpha * B * op(A),  A is n x n;
 * B is m x n (ldb >= max(1,m)), op(A) = A or A^T (transa), A is lower or upper triangular (uplo): only that
 * triangle of the array is read, the rest counts as zero, and with diag 'U' the diagonal is not read and counts
 * as one (diag 'N': it is read).  lda >= max(1, order of A).  The product is formed by Algorithm 1 on the
 * triangular matrix so defined, exactly as oz2_dgemm_ex would on a full array holding those zeros; stage 1
 * masks what is not stored and stage 2 skips the blocks of the inner dimension that are zero by structure
 * (about half).  alpha == 0: B := 0, A is not read.  Workspace: oz2_workspace_bytes(m, n, order of A,
 * num_moduli).  Argument codes are 1-based over this parameter list. */
int oz2_dtrmm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha, const double* A,
              int64_t lda, double* B, int64_t ldb, int num_moduli, void* stream);

/* The three device stages of oz2_dgemm as separate calls (same kernels, same workspace); running them
 * in order is identical to oz2_dgemm.  They exist so that each stage can be tested and timed alone.
 *   oz2_stage1_convert : Algorithm 1 lines 1-5 (shifts, truncation, INT8 residues of A and B)
 *   oz2_stage2_gemm    : line 6 (products of the residue planes, all moduli; with line 7 in its epilogue
 *                        in the default product format)
 *   oz2_stage3_crt     : lines 7-11 (residues of the products, CRT accumulation, mod M, inverse scaling) */
int oz2_stage1_convert(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B,
                       int64_t ldb, int num_moduli, void* stream);
int oz2_stage2_gemm(int64_t m, int64_t n, int64_t k, int num_moduli, void* stream);
int oz2_stage3_crt(int64_t m, int64_t n, int64_t k, double* C, int64_t ldc, int num_moduli, void* stream);

/* Contexts.  The calls above share one process-wide set of settings (shift mode, product format, form of the
 * products, k-block, bit split, non-finite check), one workspace registration and one plan cache: what a call
 * computes depends on settings another thread may change, and two calls that use the one workspace must not overlap.
 * A context is a private copy of all of that: its own settings (at the defaults when created), its own workspace
 * registration, its own lock.  Calls on different contexts, each with a workspace of its own, may be made from
 * different threads and may overlap in time on different streams; calls on one context serialise on its lock and,
 * like the plain calls, must not overlap on the GPU.  A NULL context means the process-wide one, so
 * oz2_context_dgemm(NULL, ...) is oz2_dgemm_ex.  Nothing in the paper corresponds to this; it is how the
 * library keeps Algorithm 1's options out of global state.
 *   oz2_context_create / destroy : host object only, no device memory; destroy does not touch the workspace.
 *   oz2_context_set_workspace    : as oz2_set_workspace, for this context.
 *   oz2_context_set / get        : option = OZ2_OPT_*, value as in the oz2_set_* call of the same name.  Returns 0,
 *                                  -2 for an unknown option, -3 for a value that call rejects.
 *   oz2_context_workspace_bytes  : bytes with which a general product of this shape takes the form this context's
 *                                  settings prefer (oz2_workspace_bytes_preferred for the context).
 *   oz2_context_dgemm / dsyrk / dtrmm : oz2_dgemm_ex / oz2_dsyrk / oz2_dtrmm under this context's settings and
 *                                  workspace; argument codes are 1-based over their own parameter lists (the
 *                                  context is argument 1).
 * The bound of the GEMM's round synchronisation (oz2_set_round_sync), the stage events and the staged entry points
 * belong to the process-wide context only. */
typedef struct oz2_context oz2_context;
#define OZ2_OPT_SHIFT_MODE 0
#define OZ2_OPT_PRODUCT_FORMAT 1
#define OZ2_OPT_GEMM_ALGORITHM 2
#define OZ2_OPT_KBLOCK 3
#define OZ2_OPT_BIT_SPLIT 4
#define OZ2_OPT_NONFINITE_CHECK 5
int oz2_context_create(oz2_context** ctx);
int oz2_context_destroy(oz2_context* ctx);
int oz2_context_set_workspace(oz2_context* ctx, void* dev_ptr, size_t bytes);
int oz2_context_set(oz2_context* ctx, int option, int64_t value);
int oz2_context_get(oz2_context* ctx, int option, int64_t* value);
size_t oz2_context_workspace_bytes(oz2_context* ctx, int64_t m, int64_t n, int64_t k, int num_moduli);
int oz2_context_dgemm(oz2_context* ctx, char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha,
                      const double* A, int64_t lda, const double* B, int64_t ldb, double beta, double* C, int64_t ldc,
                      int num_moduli, void* stream);
int oz2_context_dsyrk(oz2_context* ctx, char uplo, char trans, int64_t n, int64_t k, double alpha, const double* A,
                      int64_t lda, double beta, double* C, int64_t ldc, int num_moduli, void* stream);
int oz2_context_dtrmm(oz2_context* ctx, char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha,
                      const double* A, int64_t lda, double* B, int64_t ldb, int num_moduli, void* stream);

/* Exceptional values (Section 3.1, closing remark: the emulation covers products of finite matrices; NaNs
 * and infinities need detection and a fallback to ordinary FP64 arithmetic).  With the check on (default),
 * stage 1 of oz2_dgemm / oz2_dgemm_ex records in the workspace whether A or B holds an infinity or a NaN
 * (free: the row / column maxima are taken on bit patterns); stage 3 then leaves C alone and an FP64 kernel
 * launched behind it forms C := alpha op(A) op(B) + beta C by the IEEE rules.  The decision is taken on the
 * device, the call does not synchronise; the workspace flag (oz2_workspace_layout, entry 9) tells afterwards
 * which way it went.  Signed zeros are not tracked: an emulated result that is zero is +0.  With the check
 * off the extra launch is skipped and non-finite inputs give unspecified values in C.  The staged entry points
 * (oz2_stage1_convert ...) never fall back.  on: 0 or 1.  Returns 0 or -1. */
int oz2_set_nonfinite_check(int on);

/* What stage 2 leaves in the C planes, for all later calls.  OZ2_PRODUCT_RESIDUE_U8 (default): the GEMM
 * epilogue takes Algorithm 1 line 7 (c'' = c' - floor(c'/p_t) p_t) and stores one byte per element, so that
 * stage 3 reads a quarter of the bytes.  OZ2_PRODUCT_INT32: the INT32 products themselves are stored (exact
 * for k < 2^17; with k-blocking a value congruent to the product modulo p_t) and stage 3 takes line 7.
 * The final C is identical in both formats.  Returns 0 or -1. */
int oz2_set_product_format(int format);

/* How oz2_dgemm / oz2_dgemm_ex form the products of Algorithm 1 line 6, for all later calls.  Line 6 is only used
 * modulo p_t (line 7), and the residues form a ring, so Strassen's identities hold in it exactly: with A'_t, B'_t
 * split into 2 x 2 blocks, seven INT8 products of half the size in each dimension, of block sums and differences
 * reduced modulo p_t again (they still fit INT8), give the four blocks of C''_t.  7/8 of the matrix-core work for
 * 7/4 of the plane bytes in stages 1 and 3; C''_t, and therefore C, is the same as in the classical form, bit
 * for bit.  The form needs UINT8 residue planes (OZ2_PRODUCT_RESIDUE_U8) and applies to the general product only:
 * oz2_dsyrk, oz2_dtrmm and the staged entry points always take the classical form.
 *   OZ2_GEMM_AUTO (default): Strassen form when m and n are at least 8192 and k at least 10240 (below, the extra
 *     bytes cost more than the products save) and the registered workspace holds oz2_workspace_bytes_strassen;
 *     else classical.
 *   OZ2_GEMM_CLASSICAL: never.   OZ2_GEMM_STRASSEN: whenever the form applies, at any size (a workspace below
 *     oz2_workspace_bytes_strassen then gives OZ2_ERR_WORKSPACE).
 * oz2_gemm_algorithm_for tells which form a general product of that shape would take under the settings and the
 * workspace in force (OZ2_GEMM_CLASSICAL or OZ2_GEMM_STRASSEN, or a negative argument code).
 * oz2_workspace_bytes_strassen: bytes the Strassen form needs (0 on invalid arguments): m, n rounded up to 512 and
 * k to 128, seven planes of a quarter of that area per modulus and operand (21 GiB at m = n = k = 16384 with 16
 * moduli).  oz2_workspace_bytes_preferred: bytes with which a general product of that shape takes the form the
 * settings in force prefer (the Strassen size where that form would be chosen, else the size for the product
 * format in force).  Returns of the setter: 0 or -1. */
int oz2_set_gemm_algorithm(int algorithm);
int oz2_gemm_algorithm_for(int64_t m, int64_t n, int64_t k, int num_moduli);
size_t oz2_workspace_bytes_strassen(int64_t m, int64_t n, int64_t k, int num_moduli);
size_t oz2_workspace_bytes_preferred(int64_t m, int64_t n, int64_t k, int num_moduli);

/* How Algorithm 1 line 1 picks the shifts, for all later calls (default OZ2_SHIFT_MAX).
 *   OZ2_SHIFT_MAX: sa_i = kappa - 1 - floor(log2 max_l |a_il|) with the bit budget kappa of Section 3.
 *   OZ2_SHIFT_CAUCHY_SCHWARZ (Section 4.1): (|A||B|)_ij <= ||A(i,:)||_2 ||B(:,j)||_2, and the shifts are the
 *     largest with 2^sa_i nu_i <= 2^beta, 2^sb_j nu_j <= 2^beta, 4^beta <= M/2 - 1, where nu is an integer
 *     upper bound of the 2-norm: e = floor(log2 max |a|), q_l = ceil(|a_l| 2^(19-e)), S = sum q_l^2,
 *     h = min{h : 4^h >= S}, nu = 2^(e-19+h), sa = beta - (e - 19 + h).  One more pass over A and B.
 *   OZ2_SHIFT_INT8_PRODUCT (Section 4.1): |A| <= D'' A'', |B| <= B'' E'' with A''_il = ceil(|a_il| 2^(5-e_i)) and
 *     B''_lj = ceil(|b_lj| 2^(5-f_j)) in [0, 64] (e_i, f_j = floor(log2) of the row / column maximum), P = A''B''
 *     on the matrix cores, R_i = max_j P_ij, C_j = max_i P_ij, t = min{t : 2^t >= R_i (C_j)}, b = max{b : 2^b <=
 *     M/2 - 1}, sa_i = floor((b - t_i)/2) - (e_i - 5), sb_j likewise; then (|A'||B'|)_ij <= 2^b.  One more pass
 *     over A and B, one more INT8 product and a pass over P; needs k (rounded up to 64) below 2^19, else calls
 *     return OZ2_ERR_BUDGET.
 * Returns 0 or -1. */
int oz2_set_shift_mode(int mode);

/* Unequal bit budgets for oz2_dgemm / oz2_dgemm_ex and the staged calls (Section 3: "if the precisions of the
 * matrices A and B differ ... we assume k_A < k_B"), for all later calls.  delta moves that many bits of budget
 * from op(A) to op(B) (negative: the other way); 0 (default) is the equal split k_A = k_B of the paper.  For
 * delta != 0 and the default shift mode: k_A = kappa - delta, k_B = S - k_A with S = max{S : k 2^S <= M/2 - 1},
 * so op(B) also receives the odd bit of S when there is one; in the Cauchy-Schwarz mode the two bounds become
 * 2^(beta - delta) and 2^(b - beta + delta), b = max{b : 2^b <= M/2 - 1}; in the INT8-product mode sa is lowered
 * and sb raised by delta.  Useful when one operand needs fewer bits than the other (e.g. single-precision
 * values of similar magnitude in A: 25 bits suffice) -- fewer moduli then reach a given accuracy.  A call whose
 * budget on either side would fall below 1 bit returns OZ2_ERR_BUDGET.  oz2_dsyrk and oz2_dtrmm always use
 * the equal split.  |delta| <= 100.  Returns 0 or -1. */
int oz2_set_bit_split(int delta);

/* Optional timing hooks for oz2_dgemm: four caller-owned hipEvent_t handles (as void*), recorded on the
 * call's stream before stage 1 and after stages 1, 2 and 3 of every later oz2_dgemm call.  The kernels and
 * their order do not change.  events == NULL switches the hooks off.  Returns 0. */
int oz2_set_stage_events(void* const events[4]);

/* Measurement support: an MFMA-only kernel (v_mfma_i32_32x32x32_i8, no memory traffic) that shows what
 * the matrix cores of the card sustain under its power cap.  `workgroups` x 256 threads each issue
 * iters x 8 MFMAs (65536 INT8 operations per wave and MFMA); random_operands: 0 fills the operand registers with a
 * constant, 1 with random bytes (two fragments per operand, reused by every instruction), 2 with random bytes in
 * eight fragments per operand that meet in changing pairs, as the fragments of a product do (iters should then
 * be a multiple of 8).  sink: device buffer of workgroups*256 ints (written).
 * clocks: device buffer of two int64: shader-clock cycles and 100 MHz reference ticks spent in the loop by
 * workgroup 0.  The caller times the launch itself.  Returns 0, a negative argument code, or OZ2_ERR_HIP. */
int oz2_calibrate_mfma(int workgroups, int iters, int random_operands, int* sink, long long* clocks, void* stream);

/* Inner-dimension block length for line 6.  INT32 accumulation is exact for fewer than 2^17 terms
 * (Section 3.1); longer inner dimensions are processed in blocks and the accumulators are reduced
 * modulo p_t between blocks.  kblock must be a positive multiple of 64 and at most 65536 (the default).
 * With blocking active the INT32 planes hold a value congruent to the exact product modulo p_t.
 * Returns 0 or -1. */
int oz2_set_kblock(int64_t kblock);

/* Tuning and test hook for line 6 (the INT8 products).  For long inner dimensions the workgroups that share an
 * accelerator die start each of their tiles together, so that they read the same part of their shared operand
 * panels at the same time; each such wait is bounded by `spins` polls of a counter (default 4096, about a
 * millisecond).  A workgroup whose wait runs to the bound stops waiting for the rest of the launch: when the
 * workgroups cannot all be resident at once (another kernel holds compute units) a launch loses one bound,
 * not one per tile.  Results never depend on this setting.  spins == 0 switches the synchronisation off;
 * 0 <= spins <= 2^20.  Returns 0 or -1. */
int oz2_set_round_sync(int spins);

/* Host-side evaluation of the device routine for lines 7-10 and the final rounding (same source,
 * compiled for the host), for unit tests of the exact-arithmetic design: given the num_moduli INT32
 * products of one output element it returns the double nearest to X = (sum_t c''_t W_t) mod M and
 * writes nothing else.  No GPU is touched.  Returns 0 or a negative argument code. */
int oz2_host_crt_element(int num_moduli, const int32_t* cprod, double* x_out);

/* The same for the route stage 3 takes with UINT8 residue planes and at most 16 moduli, where the accumulation of
 * line 9 runs on the matrix cores: the weights W_t are brought into the symmetric range modulo M and written in
 * sixteen balanced base-256 digits, the digit sums sum_t c''_t dig_i,t are what one INT8 MFMA delivers (formed
 * here by a plain integer loop), and the same exact tail rounds X.  residues: num_moduli bytes, residues[t] in
 * [0, p_t).  num_moduli <= 16.  Returns 0 or a negative argument code. */
int oz2_host_crt_element_digits(int num_moduli, const uint8_t* residues, double* x_out);

/* Host-side evaluation of the device routine for lines 2-5 on one element: residues of
 * trunc(a * 2^shift) for all moduli (int8, num_moduli entries).  kappa tells the routine which of its
 * two splitting depths to use, as the kernels do.  No GPU is touched. */
int oz2_host_residues(int num_moduli, int kappa, double a, int shift, int8_t* res_out);

const char* oz2_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* OZ2_H */
