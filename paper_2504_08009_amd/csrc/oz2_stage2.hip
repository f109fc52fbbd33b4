// Stage 2 of Ozaki scheme II on gfx950: Algorithm 1 line 6, C'_t = A'_t B'_t for every modulus t with
// INT8 operands and INT32 accumulation on the matrix cores (v_mfma_i32_32x32x32_i8).
//
// Operand layout (written by stage 1): A'_t is m_pad x k_pad with k contiguous, B'_t is n_pad x k_pad with
// k contiguous, both zero padded to the tile sizes, so the kernel has no edge cases.  Output plane t holds
// element (i,j) at (j*m_pad + i), i contiguous.
//
// One workgroup (4 waves, one per SIMD) computes a 256 x 256 tile of one modulus.  Each wave owns a
// 128 x 128 sub-tile = 4 x 4 MFMA tiles of 32 x 32 (256 accumulator registers).  The inner dimension is
// walked in k-tiles of 128 bytes; both operands of a k-tile are copied global -> LDS with 16-byte direct
// loads (no VGPR staging), double buffered, one barrier per k-tile.  LDS rows are 128 bytes; the 16-byte
// chunk index is XOR-swizzled with bits 1..3 of the row so that the 16 rows read together by a
// ds_read_b128 fall on 16 different bank groups.
//
// INT32 accumulation is exact for fewer than 2^17 terms (Section 3.1).  For longer inner dimensions the
// accumulators are reduced modulo p_t every `kblock` bytes of k (kblock <= 65536), which keeps them below
// 2^31 and leaves the residue of the product unchanged.
//
// The 1-D grid is remapped so that each XCD (workgroup id mod 8) walks a contiguous range of tiles, and
// consecutive tiles of that range form 8-tile-tall column groups: the 32 workgroups resident on an XCD
// then share A' and B' panels in that XCD's L2.
#include "oz2_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = OZ2_TILE_M, BN = OZ2_TILE_N, BK = OZ2_TILE_K;
constexpr int kThreads = 256;
constexpr int kStageBytes = (BM + BN) * BK;      // 64 KiB: A tile then B tile
constexpr int kLdsBytes = 2 * kStageBytes;       // double buffered
constexpr int kGroupM = 8;

struct GemmArgs {
  const int8_t* a;
  const int8_t* b;
  int* c;
  int64_t m_pad, n_pad, k_pad;
  int tiles_m, tiles_n, num_moduli;
  int total, chunk;        // work items, and items per XCD
  int ktiles;              // k_pad / BK
  int ktiles_per_block;    // k-tiles between modular reductions of the accumulators
  float p[OZ2_MAX_N];
};

// 16-byte-per-lane direct load global -> LDS.  The wave writes 1024 contiguous bytes starting at the
// LDS byte address in M0; lane l's 16 bytes come from base + its own 32-bit byte offset.  Written as
// inline assembly so that completion is tracked by this file's explicit vmcnt waits (one per k-tile)
// instead of a conservative wait after every load.
__device__ __forceinline__ void load_to_lds_16(const int8_t* base, unsigned voff, unsigned lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(voff), "s"(base), "s"(lds_addr)
      : "memory");
}

// Any representative of c modulo p with |result| <= 3p is enough between k-blocks: the final residue is
// taken in stage 3.  The quotient is estimated in FP32 (error below two units).
__device__ __forceinline__ int reduce_mod(int c, int p, float inv_p) {
  int q = (int)rintf((float)c * inv_p);
  return c - q * p;
}

__global__ void __launch_bounds__(kThreads) gemm_i8_kernel(const GemmArgs g) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  // ---- which tile
  const int wg = blockIdx.x;
  const int idx = wg >> 3;
  const int item = (wg & 7) * g.chunk + idx;
  if (item >= g.total) return;
  const int per_t = g.tiles_m * g.tiles_n;
  const int t = item / per_t;
  const int r = item - t * per_t;
  const int per_group = kGroupM * g.tiles_n;
  const int gid = r / per_group;
  const int first_m = gid * kGroupM;
  const int gsize = g.tiles_m - first_m < kGroupM ? g.tiles_m - first_m : kGroupM;
  const int rr = r - gid * per_group;
  const int tm = first_m + rr % gsize;
  const int tn = rr / gsize;

  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wv >> 1, wn = wv & 1;

  // ---- global -> LDS copy: wave wv fills rows [64 wv, 64 wv + 64) of both tiles, 8 rows per load.
  // Lane l of a load covers row (l >> 3) of its 8-row group and the 16-byte chunk that the swizzle
  // places at physical position (l & 7).
  const size_t kp = (size_t)g.k_pad;
  const int8_t* a_wave = g.a + ((size_t)t * g.m_pad + (size_t)tm * BM + wv * 64) * kp;
  const int8_t* b_wave = g.b + ((size_t)t * g.n_pad + (size_t)tn * BN + wv * 64) * kp;
  const unsigned voff_even = (unsigned)((lane >> 3) * kp) + (((lane & 7) ^ (lane >> 4)) << 4);
  const unsigned voff_odd = (unsigned)(((lane >> 3) + 8) * kp) + (((lane & 7) ^ (4 + (lane >> 4))) << 4);
  const size_t row16 = 16 * kp;

  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds;
  const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds_base + wv * 8192);

  auto issue = [&](int stage, int kt) {
    const unsigned sa = lds_wave + stage * kStageBytes;
    const unsigned sb = sa + BM * BK;
    const int8_t* ga = a_wave + (size_t)kt * BK;
    const int8_t* gb = b_wave + (size_t)kt * BK;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      load_to_lds_16(ga + q * row16, voff_even, sa + (2 * q) * 1024);
      load_to_lds_16(ga + q * row16, voff_odd, sa + (2 * q + 1) * 1024);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      load_to_lds_16(gb + q * row16, voff_even, sb + (2 * q) * 1024);
      load_to_lds_16(gb + q * row16, voff_odd, sb + (2 * q + 1) * 1024);
    }
  };

  // ---- LDS -> fragment addresses
  const int swz = (lane >> 1) & 7;
  const int half = lane >> 5;
  const int a_row_off = (wm * 128 + (lane & 31)) * BK;             // + ti*32*BK
  const int b_row_off = BM * BK + (wn * 128 + (lane & 31)) * BK;   // + tj*32*BK

  v16i acc[4][4];
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int y = 0; y < 4; ++y)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[x][y][e] = 0;

  const int p_int = (int)g.p[t];
  const float inv_pf = 1.0f / g.p[t];

  auto load_frags = [&](const char* base, int s, v4i* af, v4i* bf) {
    const int coff = (((2 * s + half) ^ swz) << 4);
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      af[x] = *reinterpret_cast<const v4i*>(base + a_row_off + x * 32 * BK + coff);
      bf[x] = *reinterpret_cast<const v4i*>(base + b_row_off + x * 32 * BK + coff);
    }
  };

  issue(0, 0);
  for (int kt0 = 0; kt0 < g.ktiles; kt0 += g.ktiles_per_block) {
    const int kt1 = kt0 + g.ktiles_per_block < g.ktiles ? kt0 + g.ktiles_per_block : g.ktiles;
    for (int kt = kt0; kt < kt1; ++kt) {
      const int stage = kt & 1;
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's direct loads have landed in LDS
      __syncthreads();
      if (kt + 1 < g.ktiles) issue(stage ^ 1, kt + 1);
      const char* base = lds + stage * kStageBytes;
      v4i af[2][4], bf[2][4];
      load_frags(base, 0, af[0], bf[0]);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < 4) load_frags(base, s + 1, af[(s + 1) & 1], bf[(s + 1) & 1]);
#pragma unroll
        for (int tj = 0; tj < 4; ++tj)
#pragma unroll
          for (int ti = 0; ti < 4; ++ti)
            acc[tj][ti] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf[s & 1][tj], af[s & 1][ti], acc[tj][ti], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (kt1 < g.ktiles) {  // between k-blocks: bring the accumulators back near zero
#pragma unroll
      for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[x][y][e] = reduce_mod(acc[x][y][e], p_int, inv_pf);
    }
  }

  // ---- epilogue: lane holds i = lane%32 (second operand), registers run over j
  int* c_tile = g.c + ((size_t)t * g.n_pad + (size_t)tn * BN + wn * 128) * g.m_pad + (size_t)tm * BM + wm * 128;
  const unsigned lane_off = (unsigned)(4 * half) * (unsigned)g.m_pad + (lane & 31);
#pragma unroll
  for (int tj = 0; tj < 4; ++tj)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int* row = c_tile + (size_t)(tj * 32 + 8 * (e >> 2) + (e & 3)) * g.m_pad;
#pragma unroll
      for (int ti = 0; ti < 4; ++ti) row[lane_off + ti * 32] = acc[tj][ti][e];
    }
}

}  // namespace

hipError_t oz2_launch_stage2(const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int64_t kblock, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_i8_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  GemmArgs g;
  g.a = reinterpret_cast<const int8_t*>(ws + lay.off_a);
  g.b = reinterpret_cast<const int8_t*>(ws + lay.off_b);
  g.c = reinterpret_cast<int*>(ws + lay.off_c);
  g.m_pad = lay.m_pad;
  g.n_pad = lay.n_pad;
  g.k_pad = lay.k_pad;
  g.tiles_m = (int)(lay.m_pad / BM);
  g.tiles_n = (int)(lay.n_pad / BN);
  g.num_moduli = plan.N;
  const int64_t total = (int64_t)g.tiles_m * g.tiles_n * plan.N;
  if (total > (int64_t)1 << 30) return hipErrorInvalidValue;
  g.total = (int)total;
  g.chunk = (int)((total + 7) / 8);
  g.ktiles = (int)(lay.k_pad / BK);
  g.ktiles_per_block = (int)(kblock / BK);
  for (int t = 0; t < OZ2_MAX_N; ++t) g.p[t] = t < plan.N ? (float)plan.moduli[t] : 1.0f;
  hipLaunchKernelGGL(gemm_i8_kernel, dim3((unsigned)(g.chunk * 8)), dim3(kThreads), kLdsBytes, st, g);
  return hipGetLastError();
}
