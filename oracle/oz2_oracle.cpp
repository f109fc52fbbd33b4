// oz2_oracle.cpp -- plain CPU oracle for Ozaki scheme II FP64 matrix multiplication with INT8
// residues and the Chinese Remainder Theorem (the paper's Algorithm 1 and Sections 2.3, 3, 3.1).
//
// THIS FILE IS TEST INFRASTRUCTURE.  It is slow and obvious on purpose.  Only the tests, the smoke
// check and the benchmark's cpu_baseline leg may load it.  The GPU library never links it, never calls
// it and shares no source, header, table or constant with it.
//
// What it computes, in the paper's order (Algorithm 1):
//   line 1     shifts D, E: one power of two per row of A and per column of B (Section 3, the d_ii / e_jj
//              formulas, read as "governed by the row maximum": sa_i = kappa-1-floor(log2 max_l |a_il|)).
//   lines 2-3  A' = trunc(D A), B' = trunc(B E) as exact integers (round toward zero).
//   lines 4-5  A'_t = A' mod p_t, B'_t = B' mod p_t with the symmetric modulo of Section 2.1.
//   line 6     C'_t = A'_t B'_t in exact integer arithmetic (int64 here, so no wrap for any k).
//   line 7     C''_t = C'_t - floor(C'_t / p_t) p_t in [0, p_t).
//   lines 8-10 Y = sum_t C''_t * (M/p_t) y_t with big integers, X = Y mod M (symmetric), eq. for C in
//              Section 2.3 and the uniqueness range of Section 3.
//   line 11    C = D^-1 X E^-1: one round-to-nearest-even conversion of the integer X, then an exact
//              power-of-two scaling.
// kappa = k_A = k_B follows the second bit-budget equation of Section 3 evaluated with integers:
//   the largest kappa with k * 4^kappa <= M/2 - 1.
// Shift selection has two modes.  Mode 0 is the simple bound of Section 3 described above.  Mode 1 is the
// Cauchy-Schwarz bound of Section 4.1 (the paper's "OS II-fast"): (|A||B|)_ij <= ||A(i,:)||_2 ||B(:,j)||_2, and
// the shifts are chosen so that 2^sa_i ||A(i,:)||_2 <= 2^beta and 2^sb_j ||B(:,j)||_2 <= 2^beta with
// 4^beta <= M/2 - 1, hence (|A'||B'|)_ij < M/2.  To make the choice reproducible bit for bit the norm is
// replaced by an integer upper bound: with e_i = floor(log2 max_l |a_il|), q_il = ceil(|a_il| 2^(19-e_i)) (an
// integer below 2^20), S_i = sum_l q_il^2 and h_i the smallest integer with 4^h_i >= S_i, one has
// ||A(i,:)||_2 <= 2^(e_i-19+h_i) and sa_i = beta - (e_i - 19 + h_i).
// Mode 2 is the INT8-product bound of Section 4.1 (the paper's "OS II-accu"): |A| <= D'' A'', |B| <= B'' E'' with
// non-negative INT8 matrices A'', B'' and power-of-two diagonals, so (|A||B|)_ij <= D''_ii (A''B'')_ij E''_jj.
// Reading taken here (the paper fixes neither the width of A'' nor how D, E follow "in reverse"):
//   e_i = floor(log2 max_l |a_il|), A''_il = ceil(|a_il| 2^(5-e_i)) in [0, 64], D''_ii = 2^(e_i-5); f_j and
//   B''_lj = ceil(|b_lj| 2^(5-f_j)) likewise;  P = A''B'' in exact integers;  R_i = max_j P_ij, C_j = max_i P_ij;
//   t_i = min{t : 2^t >= R_i}, t_j = min{t : 2^t >= C_j};  b = max{b : 2^b <= M/2 - 1};
//   sa_i = floor((b - t_i)/2) - (e_i - 5),  sb_j = floor((b - t_j)/2) - (f_j - 5).
// Since P_ij <= min(R_i, C_j) <= sqrt(R_i C_j) <= 2^((t_i+t_j)/2), this gives
//   (|A'||B'|)_ij <= 2^(sa_i+sb_j) 2^(e_i-5) P_ij 2^(f_j-5) <= 2^b <= M/2 - 1.
// The maxima R_i and C_j run over ALL columns and rows, also when only a subset of outputs is asked for.
// Unequal bit budgets (Section 3: "if the precisions of A and B differ ... k_A < k_B"): an integer delta moves
// delta bits of budget from A to B.  delta = 0 is the paper's equal split in every mode.  For delta != 0:
//   mode 0: k_A = kappa - delta, k_B = S - k_A with S = max{S : k 2^S <= M/2 - 1} (first budget equation; S is
//           2 kappa or 2 kappa + 1, so B also gets the odd bit);
//   mode 1: 2^sa_i nu_i <= 2^(beta - delta), 2^sb_j nu_j <= 2^(b - beta + delta), b = max{b : 2^b <= M/2 - 1};
//   mode 2: sa_i is lowered and sb_j raised by delta.
// In every case the product of the two bounds is unchanged or smaller than M/2 - 1 allows.
// The moduli are the greedy descending pairwise-coprime sequence starting at 256 (Section 3.1 asks for
// the largest possible pairwise-coprime values not above 256); a caller may pass any other list, e.g. the
// sixteen values the paper prints.
//
// Pins (tests/test_oracle_*.py) check this file against Python big-integer / Fraction arithmetic,
// closed forms and the invariants of Sections 2.3 and 3; nothing here is "parity unpinned".
//
// All pointers are host pointers.  Matrices are column-major with leading dimensions (BLAS convention).

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <vector>

namespace {

typedef unsigned __int128 u128;
typedef __int128 i128;

// ---------------------------------------------------------------------------------------------
// Fixed-width unsigned big integer, little-endian 32-bit words.  384 bits hold Y < 2^13 * M for every
// supported number of moduli (M < 2^215 at 28 moduli).
// ---------------------------------------------------------------------------------------------
const int WORDS = 12;

struct BigU {
  uint32_t w[WORDS];
  BigU() { std::memset(w, 0, sizeof(w)); }
  explicit BigU(uint64_t v) {
    std::memset(w, 0, sizeof(w));
    w[0] = (uint32_t)v;
    w[1] = (uint32_t)(v >> 32);
  }
};

bool is_zero(const BigU& a) {
  for (int i = 0; i < WORDS; ++i)
    if (a.w[i]) return false;
  return true;
}

int cmp(const BigU& a, const BigU& b) {
  for (int i = WORDS - 1; i >= 0; --i) {
    if (a.w[i] < b.w[i]) return -1;
    if (a.w[i] > b.w[i]) return 1;
  }
  return 0;
}

BigU add(const BigU& a, const BigU& b) {
  BigU r;
  uint64_t c = 0;
  for (int i = 0; i < WORDS; ++i) {
    uint64_t s = (uint64_t)a.w[i] + b.w[i] + c;
    r.w[i] = (uint32_t)s;
    c = s >> 32;
  }
  return r;
}

// a - b, requires a >= b
BigU sub(const BigU& a, const BigU& b) {
  BigU r;
  int64_t borrow = 0;
  for (int i = 0; i < WORDS; ++i) {
    int64_t d = (int64_t)a.w[i] - (int64_t)b.w[i] - borrow;
    borrow = d < 0;
    if (d < 0) d += ((int64_t)1 << 32);
    r.w[i] = (uint32_t)d;
  }
  return r;
}

BigU mul_small(const BigU& a, uint32_t m) {
  BigU r;
  uint64_t c = 0;
  for (int i = 0; i < WORDS; ++i) {
    uint64_t s = (uint64_t)a.w[i] * m + c;
    r.w[i] = (uint32_t)s;
    c = s >> 32;
  }
  return r;
}

// quotient of a / d for a small divisor; remainder returned through rem
BigU div_small(const BigU& a, uint32_t d, uint32_t* rem) {
  BigU q;
  uint64_t r = 0;
  for (int i = WORDS - 1; i >= 0; --i) {
    uint64_t cur = (r << 32) | a.w[i];
    q.w[i] = (uint32_t)(cur / d);
    r = cur % d;
  }
  if (rem) *rem = (uint32_t)r;
  return q;
}

BigU shl1(const BigU& a) {
  BigU r;
  uint32_t c = 0;
  for (int i = 0; i < WORDS; ++i) {
    r.w[i] = (a.w[i] << 1) | c;
    c = a.w[i] >> 31;
  }
  return r;
}

BigU shr1(const BigU& a) {
  BigU r;
  uint32_t c = 0;
  for (int i = WORDS - 1; i >= 0; --i) {
    r.w[i] = (a.w[i] >> 1) | (c << 31);
    c = a.w[i] & 1u;
  }
  return r;
}

int bit_length(const BigU& a) {
  for (int i = WORDS - 1; i >= 0; --i)
    if (a.w[i]) {
      int b = 32;
      while (!((a.w[i] >> (b - 1)) & 1u)) --b;
      return 32 * i + b;
    }
  return 0;
}

int get_bit(const BigU& a, int pos) { return (a.w[pos / 32] >> (pos % 32)) & 1u; }

// a mod m by binary long division (shift-and-subtract); a < 2^(32*WORDS-1)
BigU mod_big(const BigU& a, const BigU& m) {
  BigU r;
  for (int pos = bit_length(a) - 1; pos >= 0; --pos) {
    r = shl1(r);
    if (get_bit(a, pos)) r.w[0] |= 1u;
    if (cmp(r, m) >= 0) r = sub(r, m);
  }
  return r;
}

// ---------------------------------------------------------------------------------------------
// Section 2.1: symmetric modulo  r = a - p * floor(a/p + 1/2)  on exact integers.
// floor(a/p + 1/2) = floor((2a + p) / (2p)).
// ---------------------------------------------------------------------------------------------
i128 floor_div(i128 num, i128 den) {  // den > 0
  i128 q = num / den;                 // C++ truncates toward zero
  if (num % den != 0 && num < 0) q -= 1;
  return q;
}

int64_t sym_mod(i128 a, int p) { return (int64_t)(a - (i128)p * floor_div(2 * a + p, 2 * (i128)p)); }

// ---------------------------------------------------------------------------------------------
// Section 3.1: moduli.  Greedy: walk down from 256 and keep every value coprime to all kept so far.
// ---------------------------------------------------------------------------------------------
int gcd_int(int a, int b) {
  while (b) {
    int t = a % b;
    a = b;
    b = t;
  }
  return a;
}

int greedy_moduli(int N, int* out) {
  int cnt = 0;
  for (int c = 256; c >= 2 && cnt < N; --c) {
    bool ok = true;
    for (int j = 0; j < cnt; ++j)
      if (gcd_int(c, out[j]) != 1) ok = false;
    if (ok) out[cnt++] = c;
  }
  return cnt == N ? 0 : -1;
}

BigU product(int N, const int* p) {
  BigU M(1);
  for (int t = 0; t < N; ++t) M = mul_small(M, (uint32_t)p[t]);
  return M;
}

// Section 2.3: W_t = M_t * y_t with M_t = M / p_t and M_t y_t = 1 (mod p_t), y_t in [1, p_t).
BigU crt_weight(const BigU& M, int pt) {
  uint32_t rem = 0;
  BigU Mt = div_small(M, (uint32_t)pt, &rem);
  uint32_t r = 0;
  div_small(Mt, (uint32_t)pt, &r);  // r = M_t mod p_t
  int y = 0;
  for (int c = 1; c < pt; ++c)
    if ((r * (uint32_t)c) % (uint32_t)pt == 1u % (uint32_t)pt) {
      y = c;
      break;
    }
  return mul_small(Mt, (uint32_t)y);
}

// Section 3, bit budget with k_A = k_B = kappa: largest kappa with k * 2^(2 kappa) <= M/2 - 1.
int kappa_of(const BigU& M, int64_t k) {
  BigU half = shr1(M);
  if (is_zero(half)) return -1;
  BigU lim = sub(half, BigU(1));
  BigU v((uint64_t)k);  // k * 4^kappa, starting at kappa = 0
  if (cmp(v, lim) > 0) return -1;
  int kappa = 0;
  for (;;) {
    if (bit_length(v) + 2 >= 32 * WORDS - 1) break;
    BigU nxt = shl1(shl1(v));
    if (cmp(nxt, lim) > 0) break;
    v = nxt;
    ++kappa;
  }
  return kappa;
}

// Section 3, first bit-budget equation: the largest S = k_A + k_B with k * 2^S <= M/2 - 1 (-1 if none).
int kappa_sum_of(const BigU& M, int64_t k) {
  BigU half = shr1(M);
  if (is_zero(half)) return -1;
  BigU lim = sub(half, BigU(1));
  BigU v((uint64_t)k);
  if (cmp(v, lim) > 0) return -1;
  int S = 0;
  for (;;) {
    if (bit_length(v) + 1 >= 32 * WORDS - 1) break;
    BigU nxt = shl1(v);
    if (cmp(nxt, lim) > 0) break;
    v = nxt;
    ++S;
  }
  return S;
}

// ---------------------------------------------------------------------------------------------
// FP64 decomposition: |x| = mant * 2^ex exactly, mant < 2^53 (mant = 0 for x = 0).
// ---------------------------------------------------------------------------------------------
void decompose(double x, int* neg, uint64_t* mant, int* ex) {
  uint64_t bits;
  std::memcpy(&bits, &x, 8);
  *neg = (int)(bits >> 63);
  int be = (int)((bits >> 52) & 0x7ff);
  uint64_t frac = bits & ((1ull << 52) - 1);
  if (be == 0) {
    *mant = frac;
    *ex = -1074;
  } else {
    *mant = frac | (1ull << 52);
    *ex = be - 1075;
  }
}

// floor(log2 |x|) for finite nonzero x
int ilog2_abs(double x) {
  int neg, ex;
  uint64_t mant;
  decompose(x, &neg, &mant, &ex);
  int b = 63;
  while (!((mant >> b) & 1ull)) --b;
  return b + ex;
}

// Algorithm 1 lines 2-3: trunc(x * 2^shift) as an exact integer (magnitude < 2^127 required).
i128 scaled_trunc(double x, int shift) {
  int neg, ex;
  uint64_t mant;
  decompose(x, &neg, &mant, &ex);
  if (mant == 0) return 0;
  int sh = ex + shift;
  u128 mag;
  if (sh >= 0)
    mag = (u128)mant << sh;
  else if (-sh >= 64)
    mag = 0;
  else
    mag = (u128)(mant >> (-sh));
  return neg ? -(i128)mag : (i128)mag;
}

// one RNE conversion of an integer magnitude to mant53 * 2^e2
void round_to_53(const BigU& mag, uint64_t* m53, int* e2) {
  int bl = bit_length(mag);
  if (bl <= 53) {
    *m53 = (uint64_t)mag.w[0] | ((uint64_t)mag.w[1] << 32);
    *e2 = 0;
    return;
  }
  int drop = bl - 53;
  uint64_t m = 0;
  for (int b = bl - 1; b >= drop; --b) m = (m << 1) | (uint64_t)get_bit(mag, b);
  int round_bit = get_bit(mag, drop - 1);
  int sticky = 0;
  for (int b = drop - 2; b >= 0; --b) sticky |= get_bit(mag, b);
  if (round_bit && (sticky || (m & 1ull))) m += 1;
  if (m == (1ull << 53)) {
    m >>= 1;
    drop += 1;
  }
  *m53 = m;
  *e2 = drop;
}

// Section 4.1 (Cauchy-Schwarz variant): largest beta with 4^beta <= M/2 - 1
int beta_of(const BigU& M) {
  BigU half = shr1(M);
  if (is_zero(half)) return -1;
  BigU lim = sub(half, BigU(1));
  if (is_zero(lim)) return -1;
  BigU v(1);
  int beta = 0;
  for (;;) {
    BigU nxt = shl1(shl1(v));
    if (cmp(nxt, lim) > 0) break;
    v = nxt;
    ++beta;
  }
  return beta;
}

// ceil(|x| * 2^(19 - e)) for |x| < 2^(e+1): an integer in [0, 2^20]
uint64_t scaled_ceil(double x, int e) {
  int neg, ex;
  uint64_t mant;
  decompose(x, &neg, &mant, &ex);
  if (mant == 0) return 0;
  int sh = ex + 19 - e;  // always negative here: mant has up to 53 bits, the result at most 21
  if (sh >= 0) return mant << sh;
  if (-sh >= 64) return 1;
  uint64_t q = mant >> (-sh);
  if ((q << (-sh)) != mant) q += 1;
  return q;
}

// shift of one vector under the Cauchy-Schwarz bound; x[l*stride], l < k
int fast_shift(const double* x, int64_t k, int64_t stride, int beta) {
  double mx = 0.0;
  for (int64_t l = 0; l < k; ++l) mx = std::fmax(mx, std::fabs(x[l * stride]));
  if (mx == 0.0) return 0;
  int e = ilog2_abs(mx);
  u128 S = 0;
  for (int64_t l = 0; l < k; ++l) {
    u128 q = scaled_ceil(x[l * stride], e);
    S += q * q;
  }
  int h = 0;
  u128 pw = 1;
  while (pw < S) {
    pw <<= 2;
    ++h;
  }
  return beta - (e - 19 + h);
}

// Section 4.1 (INT8-product variant): largest b with 2^b <= M/2 - 1
int log2_budget(const BigU& M) {
  BigU half = shr1(M);
  if (is_zero(half)) return -1;
  BigU lim = sub(half, BigU(1));
  if (is_zero(lim)) return -1;
  return bit_length(lim) - 1;
}

// ceil(|x| * 2^(5 - e)) for |x| < 2^(e+1): an integer in [0, 64]; never 0 for x != 0
int bound6(double x, int e) {
  int neg, ex;
  uint64_t mant;
  decompose(x, &neg, &mant, &ex);
  if (mant == 0) return 0;
  int sh = ex + 5 - e;  // |x| = mant * 2^ex
  if (sh >= 0) return (int)(mant << sh);
  if (-sh >= 64) return 1;
  uint64_t q = mant >> (-sh);
  if ((q << (-sh)) != mant) q += 1;
  return (int)q;
}

// smallest t with 2^t >= v (v >= 1)
int ceil_log2_u64(uint64_t v) {
  int t = 0;
  while (((uint64_t)1 << t) < v) ++t;
  return t;
}

int floor_div2(int x) { return x >= 0 ? x / 2 : -((-x + 1) / 2); }

int validate(int64_t m, int64_t n, int64_t k, int64_t lda, int64_t ldb, int N) {
  if (m < 0 || n < 0 || k < 0) return -1;
  if (lda < (m > 1 ? m : 1) || ldb < (k > 1 ? k : 1)) return -2;
  if (N < 1 || N > 28) return -3;
  return 0;
}

}  // namespace

extern "C" {

int oz2o_words(void) { return WORDS; }

// Greedy moduli table, first N entries.
int oz2o_moduli(int N, int* out) {
  if (N < 1 || N > 28) return -1;
  return greedy_moduli(N, out);
}

// Bit budget of the INT8-product variant for a moduli list: largest b with 2^b <= M/2 - 1.
int oz2o_log2_budget(int N, const int* moduli) {
  if (N < 1 || N > 28) return -1;
  return log2_budget(product(N, moduli));
}

// S = k_A + k_B of the first bit-budget equation of Section 3: largest S with k * 2^S <= M/2 - 1 (-1 if none).
int oz2o_kappa_sum(int N, const int* moduli, int64_t k) {
  if (N < 1 || N > 28 || k < 1) return -1;
  return kappa_sum_of(product(N, moduli), k);
}

// beta of the Cauchy-Schwarz variant for a moduli list: largest beta with 4^beta <= M/2 - 1.
int oz2o_beta(int N, const int* moduli) {
  if (N < 1 || N > 28) return -1;
  return beta_of(product(N, moduli));
}

// kappa for a moduli list and inner dimension k.  -1 when even kappa = 0 violates the bound.
int oz2o_kappa(int N, const int* moduli, int64_t k) {
  if (N < 1 || N > 28 || k < 1) return -1;
  return kappa_of(product(N, moduli), k);
}

// CRT constants as little-endian 32-bit words: M_words[WORDS], W_words[N][WORDS].
int oz2o_crt_constants(int N, const int* moduli, uint32_t* M_words, uint32_t* W_words) {
  if (N < 1 || N > 28) return -1;
  BigU M = product(N, moduli);
  std::memcpy(M_words, M.w, sizeof(M.w));
  for (int t = 0; t < N; ++t) {
    BigU W = crt_weight(M, moduli[t]);
    std::memcpy(W_words + (size_t)t * WORDS, W.w, sizeof(W.w));
  }
  return 0;
}

// Symmetric modulo of Section 2.1 for a 64-bit argument.
int64_t oz2o_sym_mod(int64_t a, int p) { return sym_mod((i128)a, p); }

// The whole of Algorithm 1 on a subset of outputs: rows I[0..nI) of A and columns J[0..nJ) of B
// (I == NULL / J == NULL mean "all rows" / "all columns", then nI = m / nJ = n).
// Every output pointer may be NULL.  Outputs (r = position in I, c = position in J):
//   C_out   [r + c*nI]                 double, final result
//   sa[r], sb[c]                       shifts
//   Ap_sign[r*k + l], Ap_mag[(r*k+l)*4 + w]   A' as sign (0/1) and four little-endian 32-bit words
//   Bp_sign[c*k + l], Bp_mag[...]             B' likewise
//   Ares[(t*nI + r)*k + l]             int8 residues of A' (k contiguous)
//   Bres[(t*nJ + c)*k + l]             int8 residues of B' (k contiguous)
//   Cprod[(t*nJ + c)*nI + r]           int64 exact products C'_t
//   Cres [(t*nJ + c)*nI + r]           uint8 residues C''_t
//   X_sign[r + c*nI], X_mag[(r + c*nI)*WORDS + w]   the integer X
// Returns 0, or a negative code for bad arguments, or 2 when kappa < 1.
int oz2o_dgemm_sub(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
                   int N, int mode, int delta, const int* moduli_in, int64_t nI, const int64_t* I, int64_t nJ,
                   const int64_t* J,
                   double* C_out, int32_t* sa_out, int32_t* sb_out, uint8_t* Ap_sign, uint32_t* Ap_mag,
                   uint8_t* Bp_sign, uint32_t* Bp_mag, int8_t* Ares, int8_t* Bres, int64_t* Cprod, uint8_t* Cres,
                   uint8_t* X_sign, uint32_t* X_mag) {
  int rc = validate(m, n, k, lda, ldb, N);
  if (rc) return rc;
  if (mode != 0 && mode != 1 && mode != 2) return -4;
  if (!I) nI = m;
  if (!J) nJ = n;
  if (nI == 0 || nJ == 0) return 0;

  std::vector<int> p(N);
  if (moduli_in)
    for (int t = 0; t < N; ++t) p[t] = moduli_in[t];
  else if (greedy_moduli(N, p.data()))
    return -3;

  const BigU M = product(N, p.data());
  const BigU halfM = shr1(M);
  std::vector<BigU> W(N);
  for (int t = 0; t < N; ++t) W[t] = crt_weight(M, p[t]);

  if (k == 0) {
    if (C_out)
      for (int64_t e = 0; e < nI * nJ; ++e) C_out[e] = 0.0;
    return 0;
  }
  const int kappa = kappa_of(M, k);
  if (kappa < 1) return 2;
  if (kappa > 120) return -3;
  const int beta = beta_of(M);
  if (mode == 1 && (beta < 1 || beta > 120)) return 2;
  const int budget = log2_budget(M);
  if (mode == 2 && (budget < 2 || budget > 240)) return 2;
  // per-operand budgets (delta == 0: the equal split)
  const int kappa_a = kappa - delta;
  const int kappa_b = delta == 0 ? kappa : kappa_sum_of(M, k) - kappa_a;
  const int beta_a = beta - delta;
  const int beta_b = delta == 0 ? beta : budget - beta_a;
  if (mode == 0 && (kappa_a < 1 || kappa_b < 1 || kappa_a > 120 || kappa_b > 120)) return 2;
  if (mode == 1 && (beta_a < 1 || beta_b < 1 || beta_a > 120 || beta_b > 120)) return 2;

  // line 1: shifts
  std::vector<int32_t> sa(nI), sb(nJ);
  if (mode == 2) {
    // bound matrices for ALL rows and columns (the maxima of P need them), then P row by row
    std::vector<int> ea(m), fb(n);
    std::vector<uint8_t> a2((size_t)m * k), b2((size_t)n * k);  // A''[i*k + l], B''[j*k + l]
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
      double mx = 0.0;
      for (int64_t l = 0; l < k; ++l) mx = std::fmax(mx, std::fabs(A[i + l * lda]));
      ea[i] = mx == 0.0 ? 0 : ilog2_abs(mx);
      for (int64_t l = 0; l < k; ++l) a2[(size_t)i * k + l] = mx == 0.0 ? 0 : (uint8_t)bound6(A[i + l * lda], ea[i]);
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
      double mx = 0.0;
      for (int64_t l = 0; l < k; ++l) mx = std::fmax(mx, std::fabs(B[l + j * ldb]));
      fb[j] = mx == 0.0 ? 0 : ilog2_abs(mx);
      for (int64_t l = 0; l < k; ++l) b2[(size_t)j * k + l] = mx == 0.0 ? 0 : (uint8_t)bound6(B[l + j * ldb], fb[j]);
    }
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nI; ++r) {
      int64_t i = I ? I[r] : r;
      uint64_t R = 0;  // max over all columns j of (A''B'')_ij
      for (int64_t j = 0; j < n; ++j) {
        uint64_t acc = 0;
        for (int64_t l = 0; l < k; ++l) acc += (uint64_t)a2[(size_t)i * k + l] * b2[(size_t)j * k + l];
        if (acc > R) R = acc;
      }
      sa[r] = R == 0 ? 0 : floor_div2(budget - ceil_log2_u64(R)) - delta - (ea[i] - 5);
    }
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < nJ; ++c) {
      int64_t j = J ? J[c] : c;
      uint64_t Cm = 0;  // max over all rows i
      for (int64_t i = 0; i < m; ++i) {
        uint64_t acc = 0;
        for (int64_t l = 0; l < k; ++l) acc += (uint64_t)a2[(size_t)i * k + l] * b2[(size_t)j * k + l];
        if (acc > Cm) Cm = acc;
      }
      sb[c] = Cm == 0 ? 0 : floor_div2(budget - ceil_log2_u64(Cm)) + delta - (fb[j] - 5);
    }
  }
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < nI; ++r) {
    if (mode == 2) continue;
    int64_t i = I ? I[r] : r;
    if (mode == 1) {
      sa[r] = fast_shift(A + i, k, lda, beta_a);
      continue;
    }
    double mx = 0.0;
    for (int64_t l = 0; l < k; ++l) mx = std::fmax(mx, std::fabs(A[i + l * lda]));
    sa[r] = mx == 0.0 ? 0 : kappa_a - 1 - ilog2_abs(mx);
  }
#pragma omp parallel for schedule(static)
  for (int64_t c = 0; c < nJ; ++c) {
    if (mode == 2) continue;
    int64_t j = J ? J[c] : c;
    if (mode == 1) {
      sb[c] = fast_shift(B + j * ldb, k, 1, beta_b);
      continue;
    }
    double mx = 0.0;
    for (int64_t l = 0; l < k; ++l) mx = std::fmax(mx, std::fabs(B[l + j * ldb]));
    sb[c] = mx == 0.0 ? 0 : kappa_b - 1 - ilog2_abs(mx);
  }
  if (sa_out) std::memcpy(sa_out, sa.data(), sizeof(int32_t) * nI);
  if (sb_out) std::memcpy(sb_out, sb.data(), sizeof(int32_t) * nJ);

  // lines 2-5: exact integers A', B' and their symmetric residues
  std::vector<int8_t> ares((size_t)N * nI * k), bres((size_t)N * nJ * k);
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < nI; ++r) {
    int64_t i = I ? I[r] : r;
    for (int64_t l = 0; l < k; ++l) {
      i128 ap = scaled_trunc(A[i + l * lda], sa[r]);
      if (Ap_sign) {
        u128 mag = ap < 0 ? (u128)(-ap) : (u128)ap;
        Ap_sign[r * k + l] = ap < 0;
        for (int w = 0; w < 4; ++w) Ap_mag[(r * k + l) * 4 + w] = (uint32_t)(mag >> (32 * w));
      }
      for (int t = 0; t < N; ++t) ares[((size_t)t * nI + r) * k + l] = (int8_t)sym_mod(ap, p[t]);
    }
  }
#pragma omp parallel for schedule(static)
  for (int64_t c = 0; c < nJ; ++c) {
    int64_t j = J ? J[c] : c;
    for (int64_t l = 0; l < k; ++l) {
      i128 bp = scaled_trunc(B[l + j * ldb], sb[c]);
      if (Bp_sign) {
        u128 mag = bp < 0 ? (u128)(-bp) : (u128)bp;
        Bp_sign[c * k + l] = bp < 0;
        for (int w = 0; w < 4; ++w) Bp_mag[(c * k + l) * 4 + w] = (uint32_t)(mag >> (32 * w));
      }
      for (int t = 0; t < N; ++t) bres[((size_t)t * nJ + c) * k + l] = (int8_t)sym_mod(bp, p[t]);
    }
  }
  if (Ares) std::memcpy(Ares, ares.data(), ares.size());
  if (Bres) std::memcpy(Bres, bres.data(), bres.size());

  // lines 6-11 per output element
#pragma omp parallel for schedule(dynamic, 4) collapse(2)
  for (int64_t c = 0; c < nJ; ++c) {
    for (int64_t r = 0; r < nI; ++r) {
      BigU Y;
      for (int t = 0; t < N; ++t) {
        const int8_t* ar = &ares[((size_t)t * nI + r) * k];
        const int8_t* bc = &bres[((size_t)t * nJ + c) * k];
        int64_t acc = 0;  // line 6
        for (int64_t l = 0; l < k; ++l) acc += (int64_t)ar[l] * (int64_t)bc[l];
        int64_t q = acc / p[t];  // line 7: floor division
        if (acc % p[t] != 0 && acc < 0) q -= 1;
        int64_t res = acc - q * p[t];
        if (Cprod) Cprod[((size_t)t * nJ + c) * nI + r] = acc;
        if (Cres) Cres[((size_t)t * nJ + c) * nI + r] = (uint8_t)res;
        Y = add(Y, mul_small(W[t], (uint32_t)res));  // line 9
      }
      // line 10: X = Y - M floor(Y/M + 1/2); with R = Y mod M this is R - M when 2R >= M, else R
      BigU R = mod_big(Y, M);
      bool negative = cmp(R, halfM) >= 0;  // M is even whenever 256 is a modulus; else 2R >= M <=> R > floor(M/2)
      if ((M.w[0] & 1u) && cmp(R, halfM) == 0) negative = false;
      BigU mag = negative ? sub(M, R) : R;
      if (X_sign) {
        X_sign[r + c * nI] = negative;
        std::memcpy(X_mag + (size_t)(r + c * nI) * WORDS, mag.w, sizeof(mag.w));
      }
      if (C_out) {  // line 11
        uint64_t m53;
        int e2;
        round_to_53(mag, &m53, &e2);
        double v = std::ldexp((double)m53, e2 - sa[r] - sb[c]);
        C_out[r + c * nI] = negative ? -v : v;
      }
    }
  }
  return 0;
}

// BLAS-style update with the product P already formed by Algorithm 1:
//   C_e := alpha * P_e + beta * C_e, evaluated as one rounding of beta * C_e (skipped, and C not read, when
//   beta == 0) followed by one fused multiply-add.
int oz2o_axpby(int64_t count, double alpha, const double* P, double beta, double* C) {
  if (count < 0) return -1;
  for (int64_t e = 0; e < count; ++e) {
    double t = beta == 0.0 ? 0.0 : beta * C[e];
    C[e] = std::fma(alpha, P[e], t);
  }
  return 0;
}

// Ordinary FP64 product for inputs the emulation does not cover (Section 3.1, closing remark: NaNs and
// infinities need detection and a fallback to a native binary64 routine): the textbook triple loop,
// P_ij = sum over l = 0 .. k-1 in that order of a_il * b_lj, every product and every sum rounded to FP64.
// op(A) is m x k, op(B) is k x n; transa / transb != 0 mean the arrays hold the transposes.
int oz2o_native_gemm(int transa, int transb, int64_t m, int64_t n, int64_t k, const double* A, int64_t lda,
                     const double* B, int64_t ldb, double* P) {
  if (m < 0 || n < 0 || k < 0) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t j = 0; j < n; ++j)
    for (int64_t i = 0; i < m; ++i) {
      volatile double acc = 0.0;  // volatile: no fused or reassociated evaluation
      for (int64_t l = 0; l < k; ++l) {
        const double a = transa ? A[l + i * lda] : A[i + l * lda];
        const double b = transb ? B[j + l * ldb] : B[l + j * ldb];
        volatile double prod = a * b;
        acc = acc + prod;
      }
      P[i + j * m] = acc;
    }
  return 0;
}

// 1 when any of the count doubles at X (column-major rows x cols with leading dimension ld) is an infinity or a NaN
int oz2o_has_nonfinite(int64_t rows, int64_t cols, const double* X, int64_t ld) {
  for (int64_t c = 0; c < cols; ++c)
    for (int64_t r = 0; r < rows; ++r)
      if (!std::isfinite(X[r + c * ld])) return 1;
  return 0;
}

// Reference product on the same subset in binary128: every product of two doubles is exact in 113 bits,
// the sum is accumulated in binary128 (relative error about k * 2^-113 of sum |a||b|).
// C_ref = rounded-to-double sum, absAB = sum_l |a_il| |b_lj| rounded to double.
int oz2o_exact_sub(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
                   int64_t nI, const int64_t* I, int64_t nJ, const int64_t* J, double* C_ref, double* absAB) {
  if (m < 0 || n < 0 || k < 0) return -1;
  if (!I) nI = m;
  if (!J) nJ = n;
#pragma omp parallel for schedule(dynamic, 4) collapse(2)
  for (int64_t c = 0; c < nJ; ++c)
    for (int64_t r = 0; r < nI; ++r) {
      int64_t i = I ? I[r] : r, j = J ? J[c] : c;
      __float128 s = 0, sabs = 0;
      for (int64_t l = 0; l < k; ++l) {
        __float128 pr = (__float128)A[i + l * lda] * (__float128)B[l + j * ldb];
        s += pr;
        sabs += pr < 0 ? -pr : pr;
      }
      if (C_ref) C_ref[r + c * nI] = (double)s;
      if (absAB) absAB[r + c * nI] = (double)sabs;
    }
  return 0;
}

}  // extern "C"
