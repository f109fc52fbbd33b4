// Host-side constants of Ozaki scheme II (computed once per (num_moduli, k)):
//   the moduli (Section 3.1), M and the CRT weights W_t = (M/p_t) * ((M/p_t)^-1 mod p_t) (Section 2.3),
//   the bit budget kappa (Section 3, second equation for k_A = k_B) and the FP64 limb tables the
//   kernels use.  Plain integer arithmetic on 256-bit values; nothing here runs on the GPU.
#include <cmath>
#include <cstring>

#include "oz2_internal.h"

namespace {

// 256-bit unsigned, eight 32-bit digits, least significant first.  M < 2^200 for 26 moduli.
struct Wide {
  uint32_t d[8];
};

Wide wide_from(uint64_t v) {
  Wide r;
  std::memset(&r, 0, sizeof(r));
  r.d[0] = (uint32_t)v;
  r.d[1] = (uint32_t)(v >> 32);
  return r;
}

void wide_mul_small(Wide& a, uint32_t f) {
  uint64_t carry = 0;
  for (int i = 0; i < 8; ++i) {
    uint64_t cur = (uint64_t)a.d[i] * f + carry;
    a.d[i] = (uint32_t)cur;
    carry = cur >> 32;
  }
}

// a := a / v, returns the remainder; v up to 64 bits
uint64_t wide_divmod(Wide& a, uint64_t v) {
  unsigned __int128 rem = 0;
  for (int i = 7; i >= 0; --i) {
    unsigned __int128 cur = (rem << 32) | a.d[i];
    a.d[i] = (uint32_t)(cur / v);
    rem = cur % v;
  }
  return (uint64_t)rem;
}

void wide_sub_one(Wide& a) {
  for (int i = 0; i < 8; ++i)
    if (a.d[i]-- != 0) break;
}

int wide_bits(const Wide& a) {
  for (int i = 7; i >= 0; --i)
    if (a.d[i]) return 32 * i + (32 - __builtin_clz(a.d[i]));
  return 0;
}

// bits [lo, lo+40) as an integer-valued double
double wide_limb(const Wide& a, int lo) {
  uint64_t v = 0;
  for (int b = 0; b < OZ2_LIMB_BITS; ++b) {
    int pos = lo + b;
    if (pos < 256 && ((a.d[pos >> 5] >> (pos & 31)) & 1u)) v |= 1ull << b;
  }
  return (double)v;
}

double wide_to_double(const Wide& a) {  // rounded, for reciprocals only
  double v = 0.0;
  for (int i = 7; i >= 0; --i) v = v * 4294967296.0 + (double)a.d[i];
  return v;
}

const int kTableLen = OZ2_MAX_N;

// Greedy descending pairwise-coprime sequence from 256.
void build_table(int* tab) {
  int cnt = 0;
  for (int cand = 256; cand >= 2 && cnt < kTableLen; --cand) {
    bool coprime = true;
    for (int j = 0; j < cnt && coprime; ++j) {
      int x = cand, y = tab[j];
      while (y) {
        int r = x % y;
        x = y;
        y = r;
      }
      coprime = (x == 1);
    }
    if (coprime) tab[cnt++] = cand;
  }
}

Wide product_of(const int* p, int N) {
  Wide M = wide_from(1);
  for (int t = 0; t < N; ++t) wide_mul_small(M, (uint32_t)p[t]);
  return M;
}

int sym_small(int64_t v, int p) {  // representative of v mod p in [-p/2, p/2)
  int r = (int)(((v % p) + p) % p);
  if (2 * r >= p) r -= p;
  return r;
}

int pow2_sym(int e, int p) {
  int64_t r = 1;
  for (int i = 0; i < e; ++i) r = (r * 2) % p;
  return sym_small(r, p);
}

}  // namespace

int oz2_table_moduli(int N, int* out) {
  if (N < 1 || N > kTableLen) return -1;
  int tab[kTableLen];
  build_table(tab);
  for (int t = 0; t < N; ++t) out[t] = tab[t];
  return 0;
}

int oz2_table_kappa(int N, int64_t k) {
  if (N < 1 || N > kTableLen || k < 1) return -1;
  int tab[kTableLen];
  build_table(tab);
  Wide lim = product_of(tab, N);
  wide_divmod(lim, 2);   // M/2
  wide_sub_one(lim);     // M/2 - 1
  wide_divmod(lim, (uint64_t)k);  // floor((M/2-1)/k)
  int bits = wide_bits(lim);
  if (bits == 0) return -1;
  return (bits - 1) / 2;  // largest kappa with 4^kappa <= floor((M/2-1)/k)
}

// largest S with k * 2^S <= M/2 - 1 (-1 if there is none): k_A + k_B of Section 3
int oz2_table_kappa_sum(int N, int64_t k) {
  if (N < 1 || N > kTableLen || k < 1) return -1;
  int tab[kTableLen];
  build_table(tab);
  Wide lim = product_of(tab, N);
  wide_divmod(lim, 2);
  wide_sub_one(lim);
  wide_divmod(lim, (uint64_t)k);  // floor((M/2-1)/k)
  return wide_bits(lim) - 1;
}

// largest b with 2^b <= M/2 - 1 (-1 if there is none); the largest beta with 4^beta <= M/2 - 1 is floor(b/2)
static int table_budget2(const int* moduli, int N) {
  Wide lim = product_of(moduli, N);
  wide_divmod(lim, 2);
  wide_sub_one(lim);
  return wide_bits(lim) - 1;
}

int oz2_build_plan(int N, int64_t k, Oz2Plan* plan) {
  if (N < OZ2_MIN_N || N > OZ2_MAX_N || k < 1) return -1;
  std::memset(plan, 0, sizeof(*plan));
  plan->N = N;
  oz2_table_moduli(N, plan->moduli);
  plan->kappa = oz2_table_kappa(N, k);
  plan->kappa_sum = oz2_table_kappa_sum(N, k);
  plan->budget2 = table_budget2(plan->moduli, N);
  plan->beta = plan->budget2 < 0 ? -1 : plan->budget2 / 2;

  const Wide M = product_of(plan->moduli, N);
  const int mbits = wide_bits(M);
  const int L = (mbits + OZ2_LIMB_BITS - 1) / OZ2_LIMB_BITS;
  if (L > OZ2_MAX_L) return -1;

  Oz2ConvConsts& cv = plan->conv;
  cv.N = N;
  // One-level split x = xh*2^32 + xl keeps |xh*c32 + xl| < 2^51 while kappa <= 75.
  cv.two_level = plan->kappa > 75;
  for (int t = 0; t < N; ++t) {
    int p = plan->moduli[t];
    cv.p[t] = (double)p;
    cv.inv_p[t] = 1.0 / (double)p;
    cv.c32[t] = (double)pow2_sym(32, p);
    cv.c64[t] = (double)pow2_sym(64, p);
  }

  Oz2CrtConsts& cc = plan->crt;
  cc.N = N;
  cc.L = L;
  Wide half = M;
  wide_divmod(half, 2);
  const double Md = wide_to_double(M);
  for (int l = 0; l < OZ2_MAX_L; ++l) {
    cc.mlimb[l] = l < L ? wide_limb(M, OZ2_LIMB_BITS * l) : 0.0;
    cc.mhalf[l] = l < L ? wide_limb(half, OZ2_LIMB_BITS * l) : 0.0;
    cc.rinv[l] = l < L ? std::ldexp(1.0, OZ2_LIMB_BITS * l) / Md : 0.0;
  }
  for (int t = 0; t < N; ++t) {
    int p = plan->moduli[t];
    cc.p[t] = (double)p;
    cc.inv_p[t] = 1.0 / (double)p;
    cc.half_inv_p[t] = 0.5 * cc.inv_p[t];
    Wide Mt = M;
    wide_divmod(Mt, (uint64_t)p);  // M / p_t
    Wide tmp = Mt;
    int r = (int)wide_divmod(tmp, (uint64_t)p);  // (M/p_t) mod p_t
    int y = 0;
    for (int c = 1; c < p; ++c)
      if ((r * c) % p == 1) y = c;
    if (p == 1) y = 0;
    Wide W = Mt;
    wide_mul_small(W, (uint32_t)y);
    for (int l = 0; l < OZ2_MAX_L; ++l) cc.w[t][l] = l < L ? wide_limb(W, OZ2_LIMB_BITS * l) : 0.0;
    if (N <= 16) {
      // balanced base-256 digits of the weight brought into (-M/2, M/2]: two's complement on 128 bits (M < 2^128,
      // |Ws| <= M/2 < 2^127, so the top byte leaves room for the last carry), then digit by digit: a byte of 128
      // or more becomes byte - 256 and carries one into the next
      unsigned __int128 w128 = 0, m128 = 0, h128 = 0;
      for (int i = 3; i >= 0; --i) {
        w128 = (w128 << 32) | W.d[i];
        m128 = (m128 << 32) | M.d[i];
        h128 = (h128 << 32) | half.d[i];
      }
      if (w128 > h128) w128 -= m128;  // wraps: the two's complement of the negative value
      int carry = 0;
      for (int i = 0; i < 16; ++i) {
        int b = (int)((w128 >> (8 * i)) & 0xff) + carry;
        carry = b >= 128 ? 1 : 0;
        plan->digits.dig[i][t] = (int8_t)(b >= 128 ? b - 256 : b);
      }
    }
  }
  plan->digits.valid = N <= 16 ? 1 : 0;
  for (int i = 0; i < 16; ++i) {
    int sum = 0;
    for (int t = 0; t < N && N <= 16; ++t) sum += plan->digits.dig[i][t];
    plan->digits.init[i] = 128 * sum;
  }
  for (int l = 0; l < 4; ++l) {
    double v = 0.0;  // exact: |init| < 2^19, at most eleven digits' worth of them, all far below 2^53 in the limbs in use
    const int first = 5 * l, last = l + 1 < L ? 5 * l + 4 : 15;
    for (int i = last; i >= first && l < L; --i) v = v * 256.0 + (double)plan->digits.init[i];
    plan->digits.sinit[l] = v;
  }
  return plan->kappa < 1 ? 2 : 0;  // 2: the simple bound of Section 3 leaves no bits for this k
}

// c_elem_bytes: 4 for INT32 product planes, 1 for UINT8 residue planes.  The product region always holds at least
// 8 bytes per element of the padded m x n grid: the INT32 product of the INT8-product shift mode and the FP64
// staging buffer of the in-place triangular product live there.
void oz2_make_layout(int64_t m, int64_t n, int64_t k, int N, int c_elem_bytes, Oz2Layout* lay) {
  auto up = [](int64_t v, int64_t a) { return (v + a - 1) / a * a; };
  auto up256 = [](size_t v) { return (v + 255) / 256 * 256; };
  lay->m_pad = up(m > 0 ? m : 1, OZ2_TILE_M);
  lay->n_pad = up(n > 0 ? n : 1, OZ2_TILE_N);
  lay->k_pad = up(k > 0 ? k : 1, OZ2_TILE_K);
  size_t off = 0;
  lay->off_rowmax = off;
  off = up256(off + (size_t)lay->m_pad * 8);
  lay->off_flags = off;  // directly behind the row maxima: one fill clears both
  off += 256;
  lay->off_colmax = off;
  off = up256(off + (size_t)lay->n_pad * 8);
  lay->off_sa = off;
  off = up256(off + (size_t)lay->m_pad * 4);
  lay->off_sb = off;
  off = up256(off + (size_t)lay->n_pad * 4);
  lay->off_a = off;
  off = up256(off + (size_t)N * lay->m_pad * lay->k_pad);
  lay->off_b = off;
  off = up256(off + (size_t)N * lay->n_pad * lay->k_pad);
  lay->off_c = off;
  {
    const size_t per_elem = (size_t)N * c_elem_bytes > 8 ? (size_t)N * c_elem_bytes : 8;
    off = up256(off + per_elem * lay->n_pad * lay->m_pad);
  }
  lay->off_rownorm = off;
  off = up256(off + (size_t)lay->m_pad * 8);
  lay->off_colnorm = off;
  off = up256(off + (size_t)lay->n_pad * 8);
  lay->total = off;
}

void oz2_make_layout_strassen(int64_t m, int64_t n, int64_t k, int N, Oz2Layout* lay) {
  auto up = [](int64_t v, int64_t a) { return (v + a - 1) / a * a; };
  auto up256 = [](size_t v) { return (v + 255) / 256 * 256; };
  const int64_t mh = up(((m > 0 ? m : 1) + 1) / 2, OZ2_TILE_M);
  const int64_t nh = up(((n > 0 ? n : 1) + 1) / 2, OZ2_TILE_N);
  const int64_t kh = up(((k > 0 ? k : 1) + 1) / 2, OZ2_TILE_K);
  lay->m_pad = 2 * mh;
  lay->n_pad = 2 * nh;
  lay->k_pad = 2 * kh;
  size_t off = 0;
  lay->off_rowmax = off;
  off = up256(off + (size_t)lay->m_pad * 8);
  lay->off_flags = off;
  off += 256;
  lay->off_colmax = off;
  off = up256(off + (size_t)lay->n_pad * 8);
  lay->off_sa = off;
  off = up256(off + (size_t)lay->m_pad * 4);
  lay->off_sb = off;
  off = up256(off + (size_t)lay->n_pad * 4);
  // 7 N planes of mh x kh bytes; the single bound plane of the INT8-product shift mode (4 mh kh bytes) fits
  lay->off_a = off;
  off = up256(off + (size_t)7 * N * mh * kh);
  lay->off_b = off;
  off = up256(off + (size_t)7 * N * nh * kh);
  // 7 N product planes of mh x nh bytes, and at least the INT32 bound product (16 mh nh bytes)
  lay->off_c = off;
  off = up256(off + (size_t)(7 * N > 16 ? 7 * N : 16) * mh * nh);
  lay->off_rownorm = off;
  off = up256(off + (size_t)lay->m_pad * 8);
  lay->off_colnorm = off;
  off = up256(off + (size_t)lay->n_pad * 8);
  lay->total = off;
}
