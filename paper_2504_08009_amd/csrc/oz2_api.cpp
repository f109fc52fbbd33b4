// C ABI of liboz2 (see include/oz2.h): argument checks, workspace bookkeeping, stage sequencing.
#include <mutex>
#include <new>

#include "../../include/oz2.h"
#include "oz2_internal.h"

namespace {

struct State {
  std::mutex mu;
  char* ws = nullptr;
  size_t ws_bytes = 0;
  int64_t kblock = 65536;
  int shift_mode = 0;
  int nonfinite_check = 1;
  int bit_split = 0;
  int product_format = OZ2_PRODUCT_RESIDUE_U8;
  int gemm_algorithm = OZ2_GEMM_AUTO;
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  bool ev_on = false;
  Oz2Plan plan;
  int plan_N = 0;
  int64_t plan_k = -1;
  int plan_rc = 0;
};

// The context the calling thread works on: the process-wide default one, or, inside an oz2_context_* call, the
// caller's.  Every entry point below reaches its settings, workspace and plan cache through state().
thread_local State* tl_state = nullptr;
State& state() {
  static State s;
  return tl_state ? *tl_state : s;
}
struct UseContext {
  State* prev;
  explicit UseContext(oz2_context* ctx) : prev(tl_state) { tl_state = reinterpret_cast<State*>(ctx); }
  ~UseContext() { tl_state = prev; }
};

// cached plan for (N, k); caller holds the mutex
int get_plan(State& s, int N, int64_t k, const Oz2Plan** out) {
  if (s.plan_N != N || s.plan_k != k) {
    s.plan_rc = oz2_build_plan(N, k, &s.plan);
    s.plan_N = N;
    s.plan_k = k;
  }
  *out = &s.plan;
  return s.plan_rc;
}

// One-time device set-up of the GEMM kernels, made before any launch under a lock of its own: contexts have
// separate locks, so two of them may reach their first launch together.
std::mutex g_setup_mu;
bool g_setup_done = false;
bool ensure_setup() {
  std::lock_guard<std::mutex> lock(g_setup_mu);
  if (!g_setup_done) g_setup_done = oz2_gemm_setup() == hipSuccess;
  return g_setup_done;
}

bool n_ok(int N) { return N >= OZ2_MIN_N && N <= OZ2_MAX_N; }

// grid dimension limits of the kernels
bool dims_ok(int64_t m, int64_t n, int64_t k) {
  const int64_t lim = (int64_t)1 << 31;
  if (m >= lim - 512 || n >= lim - 512 || k >= lim - 512) return false;
  if ((k + 63) / 64 > 65535) return false;  // second grid dimension of the row-wise kernels
  if ((m + 511) / 512 > 65535) return false;
  return true;
}

// A workspace a call runs in: the registered one, or the library's own static buffer.
struct WsRef {
  char* p;
  size_t bytes;
};

int prepare(State& s, const WsRef& w, int64_t m, int64_t n, int64_t k, int N, const Oz2Plan** plan, Oz2Layout* lay) {
  int rc = get_plan(s, N, k, plan);
  if (rc == 2 && (s.shift_mode == OZ2_SHIFT_MAX || (*plan)->beta < 1)) return OZ2_ERR_BUDGET;
  if (rc == 2) rc = 0;
  if (rc != 0) return -10;
  // unequal budgets must leave at least one bit and at most 110 on each side
  if (s.bit_split != 0) {
    const Oz2Plan& p = **plan;
    int a, b;
    if (s.shift_mode == OZ2_SHIFT_MAX) { a = p.kappa - s.bit_split; b = p.kappa_sum - a; }
    else if (s.shift_mode == OZ2_SHIFT_CAUCHY_SCHWARZ) { a = p.beta - s.bit_split; b = p.budget2 - a; }
    else { a = p.budget2 / 2 - s.bit_split; b = p.budget2 / 2 + s.bit_split; }
    if (a < 1 || b < 1 || a > 110 || b > 110) return OZ2_ERR_BUDGET;
  }
  // the INT8 product of the 6-bit bounds must stay below 2^31
  if (s.shift_mode == OZ2_SHIFT_INT8_PRODUCT && (k + 63) / 64 * 64 >= ((int64_t)1 << 19)) return OZ2_ERR_BUDGET;
  oz2_make_layout(m, n, k, N, s.product_format == OZ2_PRODUCT_INT32 ? 4 : 1, lay);
  if (!w.p || w.bytes < lay->total) return OZ2_ERR_WORKSPACE;
  return ensure_setup() ? OZ2_OK : OZ2_ERR_HIP;
}

int prepare(State& s, int64_t m, int64_t n, int64_t k, int N, const Oz2Plan** plan, Oz2Layout* lay) {
  return prepare(s, WsRef{s.ws, s.ws_bytes}, m, n, k, N, plan, lay);
}

// The Strassen form pays when the matrix-core work it saves (an eighth of 2 m n k N) outweighs the extra plane
// traffic of its conversion and CRT passes (three quarters more bytes per plane) and the lower rate of products
// with a short inner dimension.  Measured on MI355X with 16 moduli, Strassen against classical form on one box:
// even at 8192^3 and at 4096 x 4096 x 32768, -1 % at 6144 x 6144 x 10240, +1 % at 6144 x 6144 x 16384, +2 % at
// 8192 x 8192 x 10240 and 10240^3, +3 % at 8192 x 8192 x 12288, +4 % at 12288 x 12288 x 10240, 8-11 % from 14336^3 on.
bool strassen_pays(int64_t m, int64_t n, int64_t k) { return m >= 8192 && n >= 8192 && k >= 10240; }

// Does a general product of this shape use the Strassen form under the current settings?  It needs UINT8 residue
// planes and, in the INT8-product shift mode, a padded inner dimension below 2^19.  On a yes, *lay is its layout.
bool strassen_applies(const State& s, int64_t m, int64_t n, int64_t k, int N, Oz2Layout* lay) {
  if (s.gemm_algorithm == OZ2_GEMM_CLASSICAL || s.product_format != OZ2_PRODUCT_RESIDUE_U8) return false;
  if (s.gemm_algorithm == OZ2_GEMM_AUTO && !strassen_pays(m, n, k)) return false;
  oz2_make_layout_strassen(m, n, k, N, lay);
  if (s.shift_mode == OZ2_SHIFT_INT8_PRODUCT && lay->k_pad >= ((int64_t)1 << 19)) return false;
  return true;
}

// prepare() for the general product: *strassen tells which form the call takes.  The automatic choice falls back to
// the plain form when the workspace only suffices for that; a forced Strassen form reports the workspace as too small.
int prepare_general(State& s, const WsRef& w, int64_t m, int64_t n, int64_t k, int N, const Oz2Plan** plan, Oz2Layout* lay,
                    bool* strassen) {
  *strassen = false;
  Oz2Layout plain;
  const int rc = prepare(s, w, m, n, k, N, plan, &plain);
  if (rc != OZ2_OK && rc != OZ2_ERR_WORKSPACE) return rc;
  Oz2Layout sl;
  if (strassen_applies(s, m, n, k, N, &sl)) {
    if (w.p && w.bytes >= sl.total) {
      *lay = sl;
      *strassen = true;
      return ensure_setup() ? OZ2_OK : OZ2_ERR_HIP;
    }
    if (s.gemm_algorithm == OZ2_GEMM_STRASSEN) return OZ2_ERR_WORKSPACE;
  }
  *lay = plain;
  return rc;
}

}  // namespace

extern "C" {

int oz2_init(void) {
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  if (!ensure_setup()) return OZ2_ERR_HIP;
  char* p;
  size_t bytes;
  return oz2_static_scratch(&p, &bytes) == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
}

int oz2_min_moduli(void) { return OZ2_MIN_N; }
int oz2_max_moduli(void) { return OZ2_MAX_N; }

int oz2_get_moduli(int num_moduli, int* moduli_out, int* kappa_out, int64_t k) {
  if (!n_ok(num_moduli)) return -1;
  if (k < 1) return -4;
  if (moduli_out) oz2_table_moduli(num_moduli, moduli_out);
  if (kappa_out) *kappa_out = oz2_table_kappa(num_moduli, k);
  return OZ2_OK;
}

int oz2_moduli_for_bits(int64_t k, int bits) {
  if (k < 1) return -1;
  if (bits < 1) return -2;
  for (int N = OZ2_MIN_N; N <= OZ2_MAX_N; ++N)
    if (oz2_table_kappa(N, k) >= bits) return N;
  return 0;
}

size_t oz2_workspace_bytes_for(int64_t m, int64_t n, int64_t k, int num_moduli, int product_format) {
  if (m < 0 || n < 0 || k < 0 || !n_ok(num_moduli) || !dims_ok(m, n, k)) return 0;
  if (product_format != OZ2_PRODUCT_INT32 && product_format != OZ2_PRODUCT_RESIDUE_U8) return 0;
  Oz2Layout lay;
  oz2_make_layout(m, n, k, num_moduli, product_format == OZ2_PRODUCT_INT32 ? 4 : 1, &lay);
  return lay.total;
}

size_t oz2_workspace_bytes(int64_t m, int64_t n, int64_t k, int num_moduli) {
  return oz2_workspace_bytes_for(m, n, k, num_moduli, OZ2_PRODUCT_INT32);
}

size_t oz2_workspace_bytes_strassen(int64_t m, int64_t n, int64_t k, int num_moduli) {
  if (m < 0 || n < 0 || k < 0 || !n_ok(num_moduli) || !dims_ok(m, n, k)) return 0;
  Oz2Layout lay;
  oz2_make_layout_strassen(m, n, k, num_moduli, &lay);
  return lay.total;
}

size_t oz2_workspace_bytes_preferred(int64_t m, int64_t n, int64_t k, int num_moduli) {
  if (m < 0 || n < 0 || k < 0 || !n_ok(num_moduli) || !dims_ok(m, n, k)) return 0;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  Oz2Layout lay;
  if (m > 0 && n > 0 && k > 0 && strassen_applies(s, m, n, k, num_moduli, &lay)) return lay.total;
  oz2_make_layout(m, n, k, num_moduli, s.product_format == OZ2_PRODUCT_INT32 ? 4 : 1, &lay);
  return lay.total;
}

int oz2_set_gemm_algorithm(int algorithm) {
  if (algorithm != OZ2_GEMM_AUTO && algorithm != OZ2_GEMM_CLASSICAL && algorithm != OZ2_GEMM_STRASSEN) return -1;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  s.gemm_algorithm = algorithm;
  return OZ2_OK;
}

int oz2_gemm_algorithm_for(int64_t m, int64_t n, int64_t k, int num_moduli) {
  if (m < 0) return -1;
  if (n < 0) return -2;
  if (k < 0) return -3;
  if (!n_ok(num_moduli)) return -4;
  if (!dims_ok(m, n, k)) return -1;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  Oz2Layout sl;
  if (m == 0 || n == 0 || k == 0 || !strassen_applies(s, m, n, k, num_moduli, &sl)) return OZ2_GEMM_CLASSICAL;
  if (s.gemm_algorithm == OZ2_GEMM_AUTO && !(s.ws && s.ws_bytes >= sl.total)) return OZ2_GEMM_CLASSICAL;
  return OZ2_GEMM_STRASSEN;
}

int oz2_set_workspace(void* dev_ptr, size_t bytes) {
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  if ((!dev_ptr && bytes) || (reinterpret_cast<uintptr_t>(dev_ptr) & 255u)) return -1;
  s.ws = static_cast<char*>(dev_ptr);
  s.ws_bytes = dev_ptr ? bytes : 0;
  return OZ2_OK;
}

int oz2_workspace_layout(int64_t m, int64_t n, int64_t k, int num_moduli, size_t offsets[10], int64_t dims[3]) {
  if (m < 0) return -1;
  if (n < 0) return -2;
  if (k < 0) return -3;
  if (!n_ok(num_moduli)) return -4;
  if (!dims_ok(m, n, k)) return -1;
  if (!offsets) return -5;
  if (!dims) return -6;
  Oz2Layout lay;
  {
    State& s = state();
    std::lock_guard<std::mutex> lock(s.mu);
    oz2_make_layout(m, n, k, num_moduli, s.product_format == OZ2_PRODUCT_INT32 ? 4 : 1, &lay);
  }
  offsets[0] = lay.off_rowmax;
  offsets[1] = lay.off_colmax;
  offsets[2] = lay.off_sa;
  offsets[3] = lay.off_sb;
  offsets[4] = lay.off_a;
  offsets[5] = lay.off_b;
  offsets[6] = lay.off_c;
  offsets[7] = lay.off_rownorm;
  offsets[8] = lay.off_colnorm;
  offsets[9] = lay.off_flags;
  dims[0] = lay.m_pad;
  dims[1] = lay.n_pad;
  dims[2] = lay.k_pad;
  return OZ2_OK;
}

int oz2_set_stage_events(void* const events[4]) {
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  s.ev_on = events != nullptr;
  for (int i = 0; i < 4; ++i) s.ev[i] = events ? static_cast<hipEvent_t>(events[i]) : nullptr;
  return OZ2_OK;
}

int oz2_set_shift_mode(int mode) {
  if (mode != OZ2_SHIFT_MAX && mode != OZ2_SHIFT_CAUCHY_SCHWARZ && mode != OZ2_SHIFT_INT8_PRODUCT) return -1;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  s.shift_mode = mode;
  return OZ2_OK;
}

int oz2_set_nonfinite_check(int on) {
  if (on != 0 && on != 1) return -1;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  s.nonfinite_check = on;
  return OZ2_OK;
}

int oz2_set_bit_split(int delta) {
  if (delta < -100 || delta > 100) return -1;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  s.bit_split = delta;
  return OZ2_OK;
}

int oz2_set_product_format(int format) {
  if (format != OZ2_PRODUCT_INT32 && format != OZ2_PRODUCT_RESIDUE_U8) return -1;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  s.product_format = format;
  return OZ2_OK;
}

int oz2_set_round_sync(int spins) {
  if (spins < 0 || spins > (1 << 20)) return -1;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  oz2_gemm_set_sync_spins(spins);
  return OZ2_OK;
}

int oz2_set_kblock(int64_t kblock) {
  if (kblock < OZ2_TILE_K || kblock > 65536 || kblock % OZ2_TILE_K) return -1;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  s.kblock = kblock;
  return OZ2_OK;
}

int oz2_stage1_convert(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb,
                       int num_moduli, void* stream) {
  if (m < 0) return -1;
  if (n < 0) return -2;
  if (k < 0) return -3;
  if (!dims_ok(m, n, k)) return -1;
  if (lda < (m > 1 ? m : 1)) return -5;
  if (ldb < (k > 1 ? k : 1)) return -7;
  if (!n_ok(num_moduli)) return -8;
  if (m == 0 || n == 0 || k == 0) return OZ2_OK;
  if (!A) return -4;
  if (!B) return -6;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  const Oz2Plan* plan;
  Oz2Layout lay;
  int rc = prepare(s, m, n, k, num_moduli, &plan, &lay);
  if (rc) return rc;
  hipError_t e = oz2_launch_stage1(0, 0, m, n, k, A, lda, B, ldb, 0, 0, *plan, s.shift_mode, s.bit_split, 0, lay, s.ws,
                                   static_cast<hipStream_t>(stream));
  return e == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
}

int oz2_stage2_gemm(int64_t m, int64_t n, int64_t k, int num_moduli, void* stream) {
  if (m < 0) return -1;
  if (n < 0) return -2;
  if (k < 0) return -3;
  if (!dims_ok(m, n, k)) return -1;
  if (!n_ok(num_moduli)) return -4;
  if (m == 0 || n == 0 || k == 0) return OZ2_OK;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  const Oz2Plan* plan;
  Oz2Layout lay;
  int rc = prepare(s, m, n, k, num_moduli, &plan, &lay);
  if (rc) return rc;
  // the counters of the round synchronisation must be zero at launch; in oz2_dgemm stage 1 has cleared them
  hipError_t e = oz2_launch_clear_sync(lay, s.ws, static_cast<hipStream_t>(stream));
  if (e == hipSuccess)
    e = oz2_launch_stage2(*plan, lay, s.ws, s.kblock, s.product_format, 0, OZ2_KRANGE_ALL, 0, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
}

int oz2_stage3_crt(int64_t m, int64_t n, int64_t k, double* C, int64_t ldc, int num_moduli, void* stream) {
  if (m < 0) return -1;
  if (n < 0) return -2;
  if (k < 0) return -3;
  if (!dims_ok(m, n, k)) return -1;
  if (ldc < (m > 1 ? m : 1)) return -5;
  if (!n_ok(num_moduli)) return -6;
  if (m == 0 || n == 0) return OZ2_OK;
  if (!C) return -4;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (k == 0) return oz2_launch_scale_c(m, n, 0.0, C, ldc, 0, st) == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  const Oz2Plan* plan;
  Oz2Layout lay;
  int rc = prepare(s, m, n, k, num_moduli, &plan, &lay);
  if (rc) return rc;
  hipError_t e = oz2_launch_stage3(m, n, 1.0, 0.0, C, ldc, *plan, lay, s.ws, s.product_format, 0, 0, st);
  return e == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
}

namespace {
int trans_code(char c) {
  switch (c) {
    case 'N': case 'n': return 0;
    case 'T': case 't': case 'C': case 'c': return 1;
    default: return -1;
  }
}
}  // namespace

namespace {
// The general product on the registered workspace (static_ws == false) or on the library's static buffer.
int dgemm_ex_impl(bool static_ws, char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha, const double* A,
                  int64_t lda, const double* B, int64_t ldb, double beta, double* C, int64_t ldc, int num_moduli,
                  void* stream) {
  const int ta = trans_code(transa), tb = trans_code(transb);
  if (ta < 0) return -1;
  if (tb < 0) return -2;
  if (m < 0) return -3;
  if (n < 0) return -4;
  if (k < 0) return -5;
  if (!dims_ok(m, n, k)) return -3;
  const int64_t rows_a = ta ? k : m, rows_b = tb ? n : k;
  if (lda < (rows_a > 1 ? rows_a : 1)) return -8;
  if (ldb < (rows_b > 1 ? rows_b : 1)) return -10;
  if (ldc < (m > 1 ? m : 1)) return -13;
  if (!n_ok(num_moduli)) return -14;
  if (m == 0 || n == 0) return OZ2_OK;
  if (!C) return -12;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (k == 0 || alpha == 0.0) {
    if (beta == 1.0) return OZ2_OK;
    return oz2_launch_scale_c(m, n, beta, C, ldc, 0, st) == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
  }
  if (!A) return -7;
  if (!B) return -9;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  WsRef w{s.ws, s.ws_bytes};
  if (static_ws) {
    // the static buffer of the current device; its address is looked up once per device, nothing is allocated
    if (oz2_static_scratch(&w.p, &w.bytes) != hipSuccess) return OZ2_ERR_HIP;
  }
  const Oz2Plan* plan;
  Oz2Layout lay;
  bool strassen;
  int rc = prepare_general(s, w, m, n, k, num_moduli, &plan, &lay, &strassen);
  if (rc == OZ2_ERR_WORKSPACE && static_ws) return OZ2_ERR_STATIC_LIMIT;
  if (rc) return rc;
  char* const ws = w.p;
  auto mark = [&](int i) { return !s.ev_on || hipEventRecord(s.ev[i], st) == hipSuccess; };
  if (!mark(0)) return OZ2_ERR_HIP;
  if (oz2_launch_stage1(ta, tb, m, n, k, A, lda, B, ldb, 0, 0, *plan, s.shift_mode, s.bit_split, strassen ? 1 : 0, lay, ws,
                        st) != hipSuccess ||
      !mark(1))
    return OZ2_ERR_HIP;
  if (strassen) {
    if (oz2_launch_strassen_gemm(*plan, lay, ws, s.kblock, s.nonfinite_check, st) != hipSuccess || !mark(2))
      return OZ2_ERR_HIP;
    if (oz2_launch_strassen_crt(m, n, alpha, beta, C, ldc, *plan, lay, ws, s.nonfinite_check, st) != hipSuccess || !mark(3))
      return OZ2_ERR_HIP;
  } else {
    if (oz2_launch_stage2(*plan, lay, ws, s.kblock, s.product_format, 0, OZ2_KRANGE_ALL, s.nonfinite_check, st) !=
            hipSuccess ||
        !mark(2))
      return OZ2_ERR_HIP;
    // up to 2^18 elements of C the blocks of the fallback ride in the launch of stage 3: one launch less where
    // launches are what the call costs (from 1024 x 1024 on the wider kernel's lower occupancy costs as much)
    if (s.nonfinite_check && s.product_format == OZ2_PRODUCT_RESIDUE_U8 && m * n <= ((int64_t)1 << 18)) {
      if (oz2_launch_stage3_or_fallback(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, *plan, lay, ws, st) !=
              hipSuccess ||
          !mark(3))
        return OZ2_ERR_HIP;
      return OZ2_OK;
    }
    if (oz2_launch_stage3(m, n, alpha, beta, C, ldc, *plan, lay, ws, s.product_format, s.nonfinite_check, 0, st) !=
            hipSuccess ||
        !mark(3))
      return OZ2_ERR_HIP;
  }
  if (s.nonfinite_check &&
      oz2_launch_fallback(reinterpret_cast<const unsigned long long*>(ws + lay.off_flags), ta, tb, m, n, k, alpha, A, lda,
                          B, ldb, beta, C, ldc, 0, 0, 0, st) != hipSuccess)
    return OZ2_ERR_HIP;
  return OZ2_OK;
}

// same argument numbering as oz2_dgemm's declaration: map the codes of the general form
int dgemm_code(int rc) {
  switch (rc) {
    case -3: return -1;
    case -4: return -2;
    case -5: return -3;
    case -7: return -4;
    case -8: return -5;
    case -9: return -6;
    case -10: return -7;
    case -12: return -8;
    case -13: return -9;
    case -14: return -10;
    default: return rc;
  }
}
}  // namespace

int oz2_dgemm_ex(char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha, const double* A, int64_t lda,
                 const double* B, int64_t ldb, double beta, double* C, int64_t ldc, int num_moduli, void* stream) {
  return dgemm_ex_impl(false, transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream);
}

int oz2_dsyrk(char uplo, char trans, int64_t n, int64_t k, double alpha, const double* A, int64_t lda, double beta,
              double* C, int64_t ldc, int num_moduli, void* stream) {
  const int tri = (uplo == 'L' || uplo == 'l') ? 1 : (uplo == 'U' || uplo == 'u') ? 2 : 0;
  const int ta = trans_code(trans);
  if (tri == 0) return -1;
  if (ta < 0) return -2;
  if (n < 0) return -3;
  if (k < 0) return -4;
  if (!dims_ok(n, n, k)) return -3;
  const int64_t rows_a = ta ? k : n;
  if (lda < (rows_a > 1 ? rows_a : 1)) return -7;
  if (ldc < (n > 1 ? n : 1)) return -10;
  if (!n_ok(num_moduli)) return -11;
  if (n == 0) return OZ2_OK;
  if (!C) return -9;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (k == 0 || alpha == 0.0) {
    if (beta == 1.0) return OZ2_OK;
    return oz2_launch_scale_c(n, n, beta, C, ldc, tri, st) == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
  }
  if (!A) return -6;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  const Oz2Plan* plan;
  Oz2Layout lay;
  int rc = prepare(s, n, n, k, num_moduli, &plan, &lay);
  if (rc) return rc;
  auto mark = [&](int i) { return !s.ev_on || hipEventRecord(s.ev[i], st) == hipSuccess; };
  if (!mark(0)) return OZ2_ERR_HIP;
  // op(A) op(A)^T: the columns of the second operand are the rows of the first, so A is converted once and
  // its planes serve as both operands
  if (oz2_launch_stage1(ta, 0, n, n, k, A, lda, nullptr, 0, 0, 0, *plan, s.shift_mode, 0, 0, lay, s.ws, st) != hipSuccess ||
      !mark(1))
    return OZ2_ERR_HIP;
  if (oz2_launch_stage2(*plan, lay, s.ws, s.kblock, s.product_format, tri, OZ2_KRANGE_ALL, s.nonfinite_check, st) != hipSuccess ||
      !mark(2))
    return OZ2_ERR_HIP;
  if (oz2_launch_stage3(n, n, alpha, beta, C, ldc, *plan, lay, s.ws, s.product_format, s.nonfinite_check, tri, st) !=
          hipSuccess ||
      !mark(3))
    return OZ2_ERR_HIP;
  // fallback: op(B) = op(A)^T is A read with the other orientation
  if (s.nonfinite_check &&
      oz2_launch_fallback(reinterpret_cast<const unsigned long long*>(s.ws + lay.off_flags), ta, !ta, n, n, k, alpha, A, lda,
                          A, lda, beta, C, ldc, tri, 0, 0, st) != hipSuccess)
    return OZ2_ERR_HIP;
  return OZ2_OK;
}

int oz2_dtrmm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha, const double* A,
              int64_t lda, double* B, int64_t ldb, int num_moduli, void* stream) {
  const int left = (side == 'L' || side == 'l') ? 1 : (side == 'R' || side == 'r') ? 0 : -1;
  const int lower = (uplo == 'L' || uplo == 'l') ? 1 : (uplo == 'U' || uplo == 'u') ? 0 : -1;
  const int ta = trans_code(transa);
  const int unit = (diag == 'U' || diag == 'u') ? 1 : (diag == 'N' || diag == 'n') ? 0 : -1;
  if (left < 0) return -1;
  if (lower < 0) return -2;
  if (ta < 0) return -3;
  if (unit < 0) return -4;
  if (m < 0) return -5;
  if (n < 0) return -6;
  const int64_t ka = left ? m : n;  // order of A = inner dimension of the product
  if (!dims_ok(m, n, ka)) return -5;
  if (lda < (ka > 1 ? ka : 1)) return -9;
  if (ldb < (m > 1 ? m : 1)) return -11;
  if (!n_ok(num_moduli)) return -12;
  if (m == 0 || n == 0) return OZ2_OK;
  if (!B) return -10;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (alpha == 0.0) return oz2_launch_scale_c(m, n, 0.0, B, ldb, 0, st) == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
  if (!A) return -8;
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  const Oz2Plan* plan;
  Oz2Layout lay;
  int rc = prepare(s, m, n, ka, num_moduli, &plan, &lay);
  if (rc) return rc;
  const int tri = (lower ? 1 : 2) | (unit ? 4 : 0);    // structure of the stored A
  const bool op_lower = (lower != 0) != (ta != 0);     // structure of op(A)
  // the product X * Y with X = op(A), Y = B (left) or X = B, Y = op(A) (right)
  const double* X = left ? A : B;
  const double* Y = left ? B : A;
  const int64_t ldx = left ? lda : ldb, ldy = left ? ldb : lda;
  const int tx = left ? ta : 0, ty = left ? 0 : ta;
  const int trix = left ? tri : 0, triy = left ? 0 : tri;
  const int krange = left ? (op_lower ? OZ2_KRANGE_UPTO_ROW : OZ2_KRANGE_FROM_ROW)
                          : (op_lower ? OZ2_KRANGE_FROM_COL : OZ2_KRANGE_UPTO_COL);
  auto mark = [&](int i) { return !s.ev_on || hipEventRecord(s.ev[i], st) == hipSuccess; };
  if (!mark(0)) return OZ2_ERR_HIP;
  if (oz2_launch_stage1(tx, ty, m, n, ka, X, ldx, Y, ldy, trix, triy, *plan, s.shift_mode, 0, 0, lay, s.ws, st) != hipSuccess ||
      !mark(1))
    return OZ2_ERR_HIP;
  if (oz2_launch_stage2(*plan, lay, s.ws, s.kblock, s.product_format, 0, krange, s.nonfinite_check, st) != hipSuccess || !mark(2))
    return OZ2_ERR_HIP;
  // B is overwritten: stage 1 has read all of it by now (stream order)
  if (oz2_launch_stage3(m, n, alpha, 0.0, B, ldb, *plan, lay, s.ws, s.product_format, s.nonfinite_check, 0, st) !=
          hipSuccess ||
      !mark(3))
    return OZ2_ERR_HIP;
  if (s.nonfinite_check) {
    // the FP64 fallback cannot work in place: it forms the product in the (then unused) product region of the
    // workspace and a second conditional kernel copies it over B
    const unsigned long long* flag = reinterpret_cast<const unsigned long long*>(s.ws + lay.off_flags);
    double* tmp = reinterpret_cast<double*>(s.ws + lay.off_c);
    if (oz2_launch_fallback(flag, tx, ty, m, n, ka, alpha, X, ldx, Y, ldy, 0.0, tmp, m, 0, trix, triy, st) != hipSuccess ||
        oz2_launch_copy_if(flag, m, n, tmp, B, ldb, st) != hipSuccess)
      return OZ2_ERR_HIP;
  }
  return OZ2_OK;
}

int oz2_dgemm(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb, double* C,
              int64_t ldc, int num_moduli, void* stream) {
  return dgemm_code(dgemm_ex_impl(false, 'N', 'N', m, n, k, 1.0, A, lda, B, ldb, 0.0, C, ldc, num_moduli, stream));
}

int oz2_dgemm_static(int64_t m, int64_t n, int64_t k, const double* A, int64_t lda, const double* B, int64_t ldb, double* C,
                     int64_t ldc, int num_moduli, void* stream) {
  return dgemm_code(dgemm_ex_impl(true, 'N', 'N', m, n, k, 1.0, A, lda, B, ldb, 0.0, C, ldc, num_moduli, stream));
}

int oz2_context_create(oz2_context** ctx) {
  if (!ctx) return -1;
  State* s = new (std::nothrow) State();
  if (!s) return OZ2_ERR_HIP;
  *ctx = reinterpret_cast<oz2_context*>(s);
  return OZ2_OK;
}

int oz2_context_destroy(oz2_context* ctx) {
  if (!ctx) return -1;
  delete reinterpret_cast<State*>(ctx);
  return OZ2_OK;
}

int oz2_context_set_workspace(oz2_context* ctx, void* dev_ptr, size_t bytes) {
  UseContext use(ctx);
  return oz2_set_workspace(dev_ptr, bytes);
}

int oz2_context_set(oz2_context* ctx, int option, int64_t value) {
  UseContext use(ctx);
  const bool fits = value >= INT32_MIN && value <= INT32_MAX;
  int rc;
  switch (option) {
    case OZ2_OPT_SHIFT_MODE: rc = fits ? oz2_set_shift_mode((int)value) : -1; break;
    case OZ2_OPT_PRODUCT_FORMAT: rc = fits ? oz2_set_product_format((int)value) : -1; break;
    case OZ2_OPT_GEMM_ALGORITHM: rc = fits ? oz2_set_gemm_algorithm((int)value) : -1; break;
    case OZ2_OPT_KBLOCK: rc = oz2_set_kblock(value); break;
    case OZ2_OPT_BIT_SPLIT: rc = fits ? oz2_set_bit_split((int)value) : -1; break;
    case OZ2_OPT_NONFINITE_CHECK: rc = fits ? oz2_set_nonfinite_check((int)value) : -1; break;
    default: return -2;
  }
  return rc == OZ2_OK ? OZ2_OK : -3;
}

int oz2_context_get(oz2_context* ctx, int option, int64_t* value) {
  if (!value) return -3;
  UseContext use(ctx);
  State& s = state();
  std::lock_guard<std::mutex> lock(s.mu);
  switch (option) {
    case OZ2_OPT_SHIFT_MODE: *value = s.shift_mode; break;
    case OZ2_OPT_PRODUCT_FORMAT: *value = s.product_format; break;
    case OZ2_OPT_GEMM_ALGORITHM: *value = s.gemm_algorithm; break;
    case OZ2_OPT_KBLOCK: *value = s.kblock; break;
    case OZ2_OPT_BIT_SPLIT: *value = s.bit_split; break;
    case OZ2_OPT_NONFINITE_CHECK: *value = s.nonfinite_check; break;
    default: return -2;
  }
  return OZ2_OK;
}

size_t oz2_context_workspace_bytes(oz2_context* ctx, int64_t m, int64_t n, int64_t k, int num_moduli) {
  UseContext use(ctx);
  return oz2_workspace_bytes_preferred(m, n, k, num_moduli);
}

int oz2_context_dgemm(oz2_context* ctx, char transa, char transb, int64_t m, int64_t n, int64_t k, double alpha,
                      const double* A, int64_t lda, const double* B, int64_t ldb, double beta, double* C, int64_t ldc,
                      int num_moduli, void* stream) {
  UseContext use(ctx);
  const int rc = oz2_dgemm_ex(transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, num_moduli, stream);
  return rc < 0 ? rc - 1 : rc;  // argument codes count the context as the first argument
}

int oz2_context_dsyrk(oz2_context* ctx, char uplo, char trans, int64_t n, int64_t k, double alpha, const double* A,
                      int64_t lda, double beta, double* C, int64_t ldc, int num_moduli, void* stream) {
  UseContext use(ctx);
  const int rc = oz2_dsyrk(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, num_moduli, stream);
  return rc < 0 ? rc - 1 : rc;
}

int oz2_context_dtrmm(oz2_context* ctx, char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha,
                      const double* A, int64_t lda, double* B, int64_t ldb, int num_moduli, void* stream) {
  UseContext use(ctx);
  const int rc = oz2_dtrmm(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, num_moduli, stream);
  return rc < 0 ? rc - 1 : rc;
}

int oz2_calibrate_mfma(int workgroups, int iters, int random_operands, int* sink, long long* clocks, void* stream) {
  if (workgroups < 1 || workgroups > 65536) return -1;
  if (iters < 1) return -2;
  if (!sink) return -4;
  if (!clocks) return -5;
  hipError_t e = oz2_launch_mfma_calibration(workgroups, iters, random_operands, sink, clocks,
                                             static_cast<hipStream_t>(stream));
  return e == hipSuccess ? OZ2_OK : OZ2_ERR_HIP;
}

int oz2_host_crt_element(int num_moduli, const int32_t* cprod, double* x_out) {
  if (!n_ok(num_moduli)) return -1;
  if (!cprod) return -2;
  if (!x_out) return -3;
  Oz2Plan plan;
  if (oz2_build_plan(num_moduli, 1, &plan) < 0) return -1;  // the CRT tables do not depend on k
  *x_out = oz2_host_crt_impl(plan.crt, cprod);
  return OZ2_OK;
}

int oz2_host_crt_element_digits(int num_moduli, const uint8_t* residues, double* x_out) {
  if (!n_ok(num_moduli) || num_moduli > 16) return -1;
  if (!residues) return -2;
  if (!x_out) return -3;
  Oz2Plan plan;
  if (oz2_build_plan(num_moduli, 1, &plan) < 0 || !plan.digits.valid) return -1;
  for (int t = 0; t < num_moduli; ++t)
    if (residues[t] >= plan.moduli[t]) return -2;
  *x_out = oz2_host_crt_digits_impl(plan.crt, plan.digits, residues);
  return OZ2_OK;
}

int oz2_host_residues(int num_moduli, int kappa, double a, int shift, int8_t* res_out) {
  if (!n_ok(num_moduli)) return -1;
  if (kappa < 1 || kappa > 110) return -2;
  if (!res_out) return -5;
  Oz2Plan plan;
  if (oz2_build_plan(num_moduli, 1, &plan) < 0) return -1;
  plan.conv.two_level = kappa > 75;  // same rule as the launcher: |x| < 2^kappa
  oz2_host_residues_impl(plan.conv, a, shift, res_out);
  return OZ2_OK;
}

const char* oz2_status_string(int status) {
  switch (status) {
    case OZ2_OK: return "success";
    case OZ2_ERR_WORKSPACE: return "workspace not registered or too small";
    case OZ2_ERR_BUDGET: return "bit budget: moduli product too small for this inner dimension, or a bit split or shift mode it cannot serve";
    case OZ2_ERR_HIP: return "HIP call failed";
    case OZ2_ERR_STATIC_LIMIT: return "problem needs more workspace than the library's static buffer holds (OZ2_STATIC_SCRATCH_BYTES)";
    default: return status < 0 ? "invalid argument" : "unknown status";
  }
}

}  // extern "C"
