// Stage 2 of Ozaki scheme II on gfx950: Algorithm 1 line 6, C'_t = A'_t B'_t for every modulus t with
// INT8 operands and INT32 accumulation on the matrix cores (v_mfma_i32_32x32x32_i8).
//
// Operand layout (written by stage 1): each residue plane is stored in blocks of 256 rows x 64 bytes of
// the inner dimension, every block contiguous (16 KiB): element (row, l) of plane t lives at
//   ((t*rows_pad + 256*(row/256)) * k_pad) + (l/64)*16384 + (row%256)*64 + (l%64).
// Rows and the inner dimension are zero padded to the tile sizes, so the kernel has no edge cases, and
// every global -> LDS copy of a k-tile reads contiguous kilobytes (a row-major plane with a power-of-two
// pitch would hit the same L2 channels with all 256 rows of a tile).  Output plane t holds element (i,j)
// at (j*m_pad + i), i contiguous: either the INT32 product itself, or (RESIDUE_U8) its residue in [0, p_t) as
// one byte (Algorithm 1 line 7 taken in the epilogue; four times less to write here and to read in stage 3).
//
// One workgroup (4 waves, one per SIMD) computes a 256 x 256 tile of one modulus.  Each wave owns a
// 128 x 128 sub-tile = 4 x 4 MFMA tiles of 32 x 32 (256 accumulator registers).  The inner dimension is
// walked in k-tiles of 64 bytes through a ring of four LDS stages (32 KiB each).  Both operands of a
// k-tile are copied global -> LDS with 16-byte direct loads (no VGPR staging).  LDS rows are 64 bytes; the
// 16-byte chunk index is XOR-swizzled with bits 2..3 of the row so that the 16 rows read together by a
// ds_read_b128 fall on 16 different bank groups (measured: no bank conflicts).
//
// Schedule of one k-tile (two MFMA k-steps of 16 MFMAs): during step 0 the fragments of step 1 are read
// from LDS; then one vmcnt wait + barrier makes the NEXT k-tile visible to all waves; during step 1 the
// first fragments of that next tile are read and the 8 direct loads that refill the stage freed by the
// barrier are issued, one LDS read per two MFMAs and one global load per two MFMAs, so that no queue
// fills up and stalls MFMA issue.
//
// INT32 accumulation is exact for fewer than 2^17 terms (Section 3.1).  For longer inner dimensions the
// accumulators are reduced modulo p_t every `kblock` bytes of k (kblock <= 65536), which keeps them below
// 2^31 and leaves the residue of the product unchanged.
//
// The 1-D grid is remapped so that the 32 workgroups resident on an XCD (workgroup id mod 8) form an
// 8 x 4 block of tiles and share A' and B' panels in that XCD's L2.  When the tile grid is a multiple of
// 16 x 16 the eight XCDs additionally work on the eight 8 x 4 sub-blocks of one 16 x 16 super-block at the
// same time, so that panels re-read by several XCDs come from the shared last-level cache instead of HBM
// (measured: same L2 miss count, higher clock under the power cap, +6 % throughput).  Tile grids that are
// multiples of 8 x 4 only (24 x 24, 40 x 40 tiles ...) get the same effect from a list of all 8 x 4 sub-blocks, of
// which the eight XCDs take eight consecutive entries per round (a kernel instantiation of its own, LIST_ORDER,
// so that the tile decoding of the other orders stays as it is; measured: GEMM -2 % at 6144^3, -4 % at 10240^3).
// Otherwise each XCD walks its own contiguous range of tiles in 8-tile-tall column groups.
//
// General products are launched with one workgroup per compute unit; each walks the work indices of its slot in
// launch order (so the mapping above is unchanged).  The ring of LDS stages runs on from tile to tile: every
// iteration of the main loop fetches the k-tile NS - 1 ahead of the one it multiplies, and when that runs past the
// end of the tile it fetches the first k-tiles of the workgroup's next tile, so the copies of a new tile cost no
// time of their own at the tile boundary (measured against issuing them after the main loop, before the
// epilogue: GEMM -9 % at k = 1024, -5 % at 4096^3, -1 % at 8192^3, even at 16384^3 where the power cap decides).
// The loop has one body for every iteration and the same number of copies in flight at every wait: with 256
// accumulator registers per lane, a second variant of the loop body costs register moves between the variants.
//
// Structured products: for the symmetric product op(A) op(A)^T both operands are A's planes and the
// workgroups of the other triangle of tiles return at once; for a triangular operand a tile walks only the
// k-tiles up to or from its diagonal block.
#include <type_traits>

#include "oz2_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = OZ2_TILE_M, BN = OZ2_TILE_N, BK = OZ2_TILE_K;
static_assert(BM == 256 && BN == 256 && BK == 64, "the kernel below is written for 256 x 256 x 64 tiles");
constexpr int kThreads = 256;
constexpr int NS = 4;                            // LDS stages
constexpr int kStageBytes = (BM + BN) * BK;      // 32 KiB: A tile then B tile
constexpr int kLdsBytes = NS * kStageBytes;
constexpr int kLoads = 8;                        // direct loads per wave per k-tile
constexpr int kGroupM = 8;

struct GemmArgs {
  const int8_t* a;
  const int8_t* b;
  int* c;
  int64_t m_pad, n_pad, k_pad;
  int tiles_m, tiles_n, num_moduli;
  int total, chunk;        // work items, and items per XCD
  int superblock;          // 1: tiles_m and tiles_n are multiples of 16, use the super-block order
  int ktiles;              // k_pad / BK
  int ktiles_per_block;    // k-tiles between modular reductions of the accumulators
  int triangle;            // 0: all tiles; 1: only tiles with tm >= tn (lower); 2: only tm <= tn (upper)
  int krange;              // triangular operand: which k-tiles of a tile can be nonzero (see OZ2_KRANGE_*)
  const unsigned long long* skip_flag;  // if not null and nonzero on the device: the products are not needed
  unsigned long long* xcd_sync;         // one counter per XCD (zero at launch), or null: no round sync
  int full_rounds;                      // rounds in which every workgroup slot has a tile
  int xcds;                             // accelerator dies of the chip: workgroup i of a launch runs on die i % xcds
  int sync_spins;                       // bound of one wait of the round synchronisation, in polls of the counter
  float p[OZ2_MAX_PLANES];             // modulus of every plane
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
      : "memory", "m0");
}

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Any representative of c modulo p with |result| <= 3p is enough between k-blocks: the final residue is
// taken in stage 3.  The quotient is estimated in FP32 (error below two units).
__device__ __forceinline__ int reduce_mod(int c, int p, float inv_p) {
  int q = (int)rintf((float)c * inv_p);
  return c - q * p;
}

struct Frag {
  v4i a[4], b[4];
};

// What one workgroup needs to know about a unit of work.
struct Tile {
  int t, tm, tn;
  int ktiles;            // k-tiles this tile walks (may be 0: the tile is then all zeros)
  const int8_t* a_wave;  // first byte this wave copies of the tile's first k-tile of A'
  const int8_t* b_wave;  // same for B'
  bool valid;            // false: nothing to compute for this work index
};

// Work index -> tile.  `slot` counts workgroup slots in launch order: slot % 8 is the XCD a workgroup of a plain
// launch would land on, and the persistent loop keeps that residue (its stride is a multiple of 8).
template <bool LIST_ORDER>
__device__ __forceinline__ Tile decode_tile(const GemmArgs& g, int slot, int wv) {
  Tile T;
  T.valid = false;
  T.ktiles = 0;
  T.a_wave = T.b_wave = nullptr;
  T.t = T.tm = T.tn = 0;
  if (slot >= g.chunk * 8) return T;
  int t, tm, tn;
  if constexpr (LIST_ORDER) {
    // The 8 x 4 sub-blocks of all planes form one list (plane by plane, down the columns of sub-blocks); in a
    // round the eight XCDs take eight consecutive entries, i.e. neighbouring sub-blocks whose A' and B' panels
    // they share through the last-level cache.  g.chunk counts whole rounds of 32 tiles per XCD here.
    const int x = slot & 7, idx = slot >> 3;
    const int rnd = idx >> 5, within = idx & 31;
    const int sub_m = g.tiles_m >> 3, per_plane = sub_m * (g.tiles_n >> 2);
    const int entry = rnd * 8 + x;
    t = entry / per_plane;
    if (t >= g.num_moduli) return T;
    const int r = entry - t * per_plane;
    const int sn = r / sub_m, sm = r - sn * sub_m;
    tm = sm * 8 + (within & 7);
    tn = sn * 4 + (within >> 3);
  } else if (g.superblock) {
    // all eight XCDs work inside one 16 x 16 super-block of tiles at a time; XCD x owns the 8 x 4
    // sub-block (x & 1, x >> 1), so A' and B' panels missed by one L2 are found in the shared cache
    const int x = slot & 7, idx = slot >> 3;
    const int sb = idx >> 5, within = idx & 31;
    const int sbs_m = g.tiles_m >> 4, sbs_n = g.tiles_n >> 4;
    t = sb / (sbs_m * sbs_n);
    const int sr = sb - t * (sbs_m * sbs_n);
    // Structured products: the eight sub-blocks of a super-block hold different amounts of work (tiles beyond
    // the diagonal are skipped, tiles of a triangular operand differ in length), so the sub-block an XCD takes
    // rotates with the super-block and the modulus; over eight moduli every XCD has had every position.
    const int xp = (g.triangle | g.krange) ? ((x + sr + t) & 7) : x;
    // super-block coordinates; with a triangular operand the super-blocks with the longest tiles go first
    // (measured at 16384: 32.0 -> 30.1 ms for the product with a lower triangular first operand)
    int sm = sr % sbs_m, sn = sr / sbs_m;
    if (g.krange == OZ2_KRANGE_UPTO_ROW) { sm = sbs_m - 1 - sr / sbs_n; sn = sr % sbs_n; }
    if (g.krange == OZ2_KRANGE_FROM_ROW) { sm = sr / sbs_n; sn = sr % sbs_n; }
    if (g.krange == OZ2_KRANGE_UPTO_COL) { sn = sbs_n - 1 - sr / sbs_m; }
    tm = sm * 16 + (xp & 1) * 8 + (within & 7);
    tn = sn * 16 + (xp >> 1) * 4 + (within >> 3);
    if (t >= g.num_moduli) return T;
  } else {
    const int item = (slot & 7) * g.chunk + (slot >> 3);
    if (item >= g.total) return T;
    const int per_t = g.tiles_m * g.tiles_n;
    t = item / per_t;
    const int r = item - t * per_t;
    const int per_group = kGroupM * g.tiles_n;
    const int gid = r / per_group;
    const int first_m = gid * kGroupM;
    const int gsize = g.tiles_m - first_m < kGroupM ? g.tiles_m - first_m : kGroupM;
    const int rr = r - gid * per_group;
    tm = first_m + rr % gsize;
    tn = rr / gsize;
  }
  // symmetric product: the other triangle of tiles is never needed
  if ((g.triangle == 1 && tm < tn) || (g.triangle == 2 && tm > tn)) return T;
  // Triangular operand (TRMM shape): op(A)(i, l) vanishes for l > i (lower) or l < i (upper), so the tile only
  // needs the k-tiles up to / from its diagonal block; which index (tm or tn) counts depends on the side.
  int kt_begin = 0, kt_end = g.ktiles;
  {
    const int per = BM / BK;  // k-tiles per diagonal block
    if (g.krange == OZ2_KRANGE_UPTO_ROW) kt_end = min(g.ktiles, (tm + 1) * per);
    if (g.krange == OZ2_KRANGE_FROM_ROW) kt_begin = min(g.ktiles, tm * per);
    if (g.krange == OZ2_KRANGE_UPTO_COL) kt_end = min(g.ktiles, (tn + 1) * per);
    if (g.krange == OZ2_KRANGE_FROM_COL) kt_begin = min(g.ktiles, tn * per);
  }
  const size_t kp = (size_t)g.k_pad;
  T.t = t;
  T.tm = tm;
  T.tn = tn;
  T.ktiles = kt_end - kt_begin;
  T.a_wave = g.a + ((size_t)t * g.m_pad + (size_t)tm * BM) * kp + wv * 64 * BK + (size_t)kt_begin * (BM * BK);
  T.b_wave = g.b + ((size_t)t * g.n_pad + (size_t)tn * BN) * kp + wv * 64 * BK + (size_t)kt_begin * (BN * BK);
  T.valid = true;
  return T;
}

// EARLY_ARRIVAL: a workgroup counts itself into the next round of the XCD synchronisation before its epilogue
// instead of after it (see the launcher).
// KBLOCKED: the inner dimension of a tile is walked in several k-blocks with a modular reduction of the
// accumulators between them (inner dimensions beyond the INT32 exactness bound, or a smaller block on request).
// A kernel of its own: the reduction's 256 x 8 instructions need so many registers at once that the compiler parks
// 48 accumulators in scratch memory around it, on the path of every tile, and the instantiation without it does not.
template <bool RESIDUE_U8, bool LIST_ORDER, bool EARLY_ARRIVAL, bool KBLOCKED>
__global__ void __launch_bounds__(kThreads) gemm_i8_kernel(const GemmArgs g) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  // stage 1 found an infinity or a NaN: the FP64 fallback forms C, these products would be thrown away
  if (g.skip_flag != nullptr && *g.skip_flag != 0ull) return;

  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wv >> 1, wn = wv & 1;

  // ---- which tiles: a workgroup takes the work indices blockIdx.x, blockIdx.x + gridDim.x, ...  With one
  // index per workgroup (gridDim.x = number of indices) this is a plain launch; with gridDim.x = number of
  // workgroup slots of the chip the loop keeps the launch order and lets the first copies of the next tile
  // fly while the current tile's epilogue runs.
  int slot = blockIdx.x;
  Tile cur = decode_tile<LIST_ORDER>(g, slot, wv);
  while (!cur.valid && slot < g.chunk * 8) {
    slot += gridDim.x;
    cur = decode_tile<LIST_ORDER>(g, slot, wv);
  }
  if (!cur.valid) return;

  // ---- global -> LDS copy: wave wv fills rows [64 wv, 64 wv + 64) of both tiles, 16 rows (1 KiB) per
  // load.  Lane l covers row (l >> 2) of the group and the chunk that the swizzle puts at position (l & 3).
  const unsigned voff = (unsigned)((lane >> 2) * BK) + (((lane & 3) ^ (lane >> 4)) << 4);
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds;
  const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds_base + wv * (64 * BK));

  // direct load q in 0..7 of a k-tile (pa, pb: this wave's first bytes of its A' and B' parts) into `stage`
  auto gl = [&](const int8_t* pa, const int8_t* pb, int stage, int q) {
    const unsigned sa = lds_wave + stage * kStageBytes;
    if (q < 4)
      load_to_lds_16(pa + q * 1024, voff, sa + q * 1024);
    else
      load_to_lds_16(pb + (q - 4) * 1024, voff, sa + BM * BK + (q - 4) * 1024);
  };
  // k-tiles 0 .. NS-2 of a tile on their way into the stages from `base` on (the ring of stages runs on across tiles)
  // (a tile with fewer k-tiles fetches its k-tile 0 again in the place of those it lacks: every wait below can
  // then count on the same number of copies in flight)
  auto prologue_loads = [&](const Tile& T, int base) {
#pragma unroll
    for (int pth = 0; pth < NS - 1; ++pth) {
      const int st = base + pth >= NS ? base + pth - NS : base + pth;
      const int src = pth < T.ktiles ? pth : 0;
#pragma unroll
      for (int q = 0; q < kLoads; ++q) gl(T.a_wave + (size_t)src * (BM * BK), T.b_wave + (size_t)src * (BN * BK), st, q);
    }
  };

  // ---- LDS -> fragments: lane reads row (lane & 31) of a 32-row group, k-chunk (2 s + lane/32)
  const int swz = (lane >> 2) & 3;
  const int half = lane >> 5;
  const int a_row_off = (wm * 128 + (lane & 31)) * BK;
  const int b_row_off = BM * BK + (wn * 128 + (lane & 31)) * BK;
  const int off_s0 = ((0 + half) ^ swz) << 4, off_s1 = ((2 + half) ^ swz) << 4;
  auto rd = [&](Frag& F, const char* base, int coff, int q) {  // read q in 0..7, ordered by first use
    if (q == 0)
      F.b[0] = *reinterpret_cast<const v4i*>(base + b_row_off + coff);
    else if (q <= 4)
      F.a[q - 1] = *reinterpret_cast<const v4i*>(base + a_row_off + (q - 1) * 32 * BK + coff);
    else
      F.b[q - 4] = *reinterpret_cast<const v4i*>(base + b_row_off + (q - 4) * 32 * BK + coff);
  };

  v16i acc[4][4];

// Operand roles of v_mfma_i32_32x32x32_i8: the rows of the first operand run over the result registers
// (lane l, register e: row 8 (e / 4) + 4 (l / 32) + e % 4), the rows of the second over the lanes (row l % 32).
//   INT32 export: first = B' (columns j over registers), second = A' (rows i over lanes): every register is
//   stored as 2 x 128 contiguous bytes of a column of C'.
//   UINT8 export: first = A', second = B': each group of four registers holds four consecutive rows i of
//   one column, i.e. the four bytes of one 32-bit store.
#define OZ2_MFMA(F, q)                                                                                        \
  acc[(q)&3][(q) >> 2] =                                                                                      \
      RESIDUE_U8 ? __builtin_amdgcn_mfma_i32_32x32x32_i8(F.a[(q)&3], F.b[(q) >> 2], acc[(q)&3][(q) >> 2], 0, 0, 0) \
                 : __builtin_amdgcn_mfma_i32_32x32x32_i8(F.b[(q) >> 2], F.a[(q)&3], acc[(q)&3][(q) >> 2], 0, 0, 0)

  prologue_loads(cur, 0);
  bool first = true;
  int round = 0;
  int stage = 0;  // stage that holds k-tile 0 of the current tile
  const int xcd = blockIdx.x % g.xcds;
  for (;;) {
  const int ktiles = cur.ktiles;
  const int t = cur.t, tm = cur.tm, tn = cur.tn;
  // ---- the next tile of this workgroup, if any.  Every iteration of the main loop below fetches one k-tile, NS - 1
  // ahead of the one it multiplies.  When that runs past the end of this tile and both tiles are at least NS - 1
  // k-tiles long, it fetches the first k-tiles of the next tile: its copies then cost no time of their own at the
  // tile boundary.  Otherwise the slot fetches this tile's k-tile 0 once more into a stage nobody reads again (one
  // loop body for every iteration, the same number of copies in flight at every wait).
  Tile nxt;
  nxt.valid = false;
  do {
    slot += gridDim.x;
    nxt = decode_tile<LIST_ORDER>(g, slot, wv);
  } while (!nxt.valid && slot < g.chunk * 8);
  const bool across = nxt.valid && ktiles >= NS - 1 && nxt.ktiles >= NS - 1;
  const int8_t* const over_a = across ? nxt.a_wave : cur.a_wave;
  const int8_t* const over_b = across ? nxt.b_wave : cur.b_wave;
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int y = 0; y < 4; ++y)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[x][y][e] = RESIDUE_U8 ? (int)0x80000000 : 0;
  // (the residue epilogue works on c' + 2^31 as an unsigned word: the accumulators start there, modulo 2^32)

  // ---- k-tiles 0 .. NS-2 are in flight: make tile 0 visible, its first fragments in registers.  After the
  // first tile of the loop the previous epilogue's stores are outstanding as well and cannot be told apart
  // from loads by the counter, so everything is waited for (the loads were issued before that epilogue).
  if (first)
    wait_vmcnt<(NS - 2) * kLoads>();
  else
    wait_vmcnt<0>();
  first = false;
  if (g.xcd_sync != nullptr && round < g.full_rounds && threadIdx.x == 0) {
    // The workgroups of an XCD start their tiles of a round together.  The wait is bounded (about a millisecond).
    // If it runs to its bound, the workgroups of this XCD are not all resident at once (another kernel holds
    // compute units) or the counters were not cleared: the counter is then pushed beyond every target of this
    // launch, so that no workgroup of the XCD waits again -- the launch loses one bound, not one per round.
    // (A flag kept in a register instead would live across the main loop, where no register is free.)
    unsigned long long* c = g.xcd_sync + xcd;
    if (!EARLY_ARRIVAL || round == 0) atomicAdd(c, 1ull);
    const unsigned long long target = (unsigned long long)(gridDim.x / g.xcds) * (unsigned long long)(round + 1);
    bool arrived = false;
    for (int spins = 0; spins < g.sync_spins; ++spins) {
      if (__hip_atomic_load(c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) {
        arrived = true;
        break;
      }
      __builtin_amdgcn_s_sleep(8);
    }
    if (!arrived) {
      atomicAdd(c, 1ull << 40);
      wait_vmcnt<0>();
    }
  }
  ++round;
  __syncthreads();
  Frag F0, F1;
#pragma unroll
  for (int q = 0; q < 8; ++q) rd(F0, lds + stage * kStageBytes, off_s0, q);

  // fa, fb: where the next fetch reads (k-tile kt + NS - 1 of this tile while that exists)
  const int8_t* fa = NS - 1 < ktiles ? cur.a_wave + (size_t)(NS - 1) * (BM * BK) : cur.a_wave;
  const int8_t* fb = NS - 1 < ktiles ? cur.b_wave + (size_t)(NS - 1) * (BN * BK) : cur.b_wave;
  auto body = [&](int kt) {
    const char* base = lds + stage * kStageBytes;
    const int nstage = stage + 1 == NS ? 0 : stage + 1;
    const char* nbase = lds + nstage * kStageBytes;
    const int lstage = stage == 0 ? NS - 1 : stage - 1;  // stage of tile kt-1 == stage of tile kt+NS-1
    // step 0: MFMAs on F0, fetch F1 = (tile kt, step 1)
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      OZ2_MFMA(F0, q);
      if ((q & 1) == 0) rd(F1, base, off_s1, q >> 1);
      if (q == 1 && kt + NS - 1 == ktiles) {  // the fetches run past the end of this tile from here on
        fa = over_a;
        fb = over_b;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // k-tile kt+1 must be complete in LDS for every wave before anyone reads it; passing this barrier
    // also means every wave has finished reading k-tile kt-1, whose stage is refilled below
    wait_vmcnt<(NS - 3) * kLoads>();
    __syncthreads();
    // step 1: MFMAs on F1, fetch F0 = (tile kt+1, step 0), issue the loads of tile kt+NS-1
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      OZ2_MFMA(F1, q);
      if ((q & 1) == 0) rd(F0, nbase, off_s0, q >> 1);
      if ((q & 1) == 1) gl(fa, fb, lstage, q >> 1);
      if (q == 15 && (kt + NS - 1 < ktiles || across)) {
        fa += BM * BK;
        fb += BN * BK;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    stage = nstage;
  };

  const int p_int = (int)g.p[t];
  const float inv_pf = 1.0f / g.p[t];
  if constexpr (KBLOCKED) {
    for (int kt0 = 0; kt0 < ktiles; kt0 += g.ktiles_per_block) {
      const int kt1 = kt0 + g.ktiles_per_block < ktiles ? kt0 + g.ktiles_per_block : ktiles;
      int kt = kt0;
      for (; kt < kt1; ++kt) body(kt);
      if (kt1 < ktiles) {  // between k-blocks: bring the accumulators back near zero
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
          for (int y = 0; y < 4; ++y)
#pragma unroll
            for (int e = 0; e < 16; ++e)
              acc[x][y][e] = RESIDUE_U8 ? (reduce_mod(acc[x][y][e] ^ (int)0x80000000, p_int, inv_pf) ^ (int)0x80000000)
                                        : reduce_mod(acc[x][y][e], p_int, inv_pf);
      }
    }
  } else {
    for (int kt = 0; kt < ktiles; ++kt) body(kt);
  }

  // ---- a next tile whose first copies were not fetched by the main loop above: they fly during the epilogue
  // below.  The barrier makes sure that every wave has left the main loop (all LDS reads of this tile issued) before
  // stages refill.  `stage` is by now the stage after this tile's last k-tile, where the next tile starts.
  if (nxt.valid) {
    if (!across) {
      __syncthreads();
      prologue_loads(nxt, stage);
    }
    if constexpr (EARLY_ARRIVAL) {
      // count in for the next round now: the others then wait for this workgroup's main loop only, not for its
      // epilogue, and the counter's round trip overlaps the epilogue
      if (g.xcd_sync != nullptr && round < g.full_rounds && threadIdx.x == 0)
        atomicAdd(g.xcd_sync + xcd, 1ull);
    }
  }

  // ---- epilogue
  if (RESIDUE_U8) {
    // Algorithm 1 line 7 here: c'' = c' mod p in [0, p), four residues per 32-bit store.  Lane holds column
    // j = lane % 32 of a 32 x 32 tile, each group of four registers four consecutive rows i.
    //   u = c' + 2^31 as an unsigned word with bytes b3..b0;  r1 = sum_i b_i (2^(8i) mod p) + ((-2^31) mod p)
    //   is congruent to c' and below 2^18 (one v_dot4_u32_u8), hence exact in FP32.  floor((r1 + 1/2)/p)
    //   == floor(r1/p), and (r1 + 1/2)/p stays 2^-9 away from every integer while the FP32 evaluation errs
    //   by less than 2^-12 (quotient below 2^11), so the floor and the remainder are exact.
    const unsigned pu = (unsigned)p_int;
    const unsigned k1 = 256u % pu, k2 = (k1 * k1) % pu, k3 = (k2 * k1) % pu;
    const unsigned kpack = 1u | (k1 << 8) | (k2 << 16) | (k3 << 24);
    const unsigned two31 = (((k3 * 128u) % pu));            // 2^31 = 2^24 * 2^7
    const unsigned bias = (pu - two31) % pu;
    const float pf = g.p[t], ipf = 1.0f / pf, hipf = 0.5f / pf;
    // the wave's corner of the tile (uniform over the wave) and the lane's own offset from it (column lane % 32,
    // rows 16 half ..: below 2^32, m_pad is below 2^27)
    uint8_t* const corner = reinterpret_cast<uint8_t*>(g.c) + (size_t)t * g.n_pad * g.m_pad +
                            ((size_t)tn * BN + wn * 128) * g.m_pad + (size_t)tm * BM + wm * 128;
    // (formed again for every tile from the lane number as the hardware counts it: a value kept across the main
    // loop, where no register is free, would be parked in scratch memory and fetched per tile)
    unsigned start = 0u;
    asm volatile("" : "+s"(start));  // opaque zero: the count below is taken here, in every tile
    const unsigned lane_now = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, start));
    const unsigned lane_off = (lane_now & 31u) * (unsigned)g.m_pad + 16u * (lane_now >> 5);
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
      // w[ti][a]: rows ti*32 + 8a + 4*half + (0..3) of column j, one byte each
      unsigned w[4][4];
#pragma unroll
      for (int ti = 0; ti < 4; ++ti)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          unsigned v = 0;
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const unsigned u = (unsigned)acc[ti][tj][4 * a + b];
            const float x = (float)__builtin_amdgcn_udot4(u, kpack, bias, false);
            const float q = floorf(fmaf(x, ipf, hipf));
            v = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(-q, pf, x), b, v);
          }
          w[ti][a] = v;
        }
      // Lanes l and l + 32 hold the two interleaved halves of the same 32 rows.  Swapping the upper half
      // of w[ti][a] with the lower half of w[ti][a+2] leaves lane l with rows 0..15 and lane l + 32 with
      // rows 16..31 of the 32-row group, 16 contiguous bytes each: one 16-byte store per lane and group,
      // issued together so that the cache lines of the column are complete at once.
      uint8_t* cj = corner + (size_t)(tj * 32) * g.m_pad;  // uniform; + ti*32 + lane_off below
#pragma unroll
      for (int ti = 0; ti < 4; ++ti) {
        const auto s0 = __builtin_amdgcn_permlane32_swap(w[ti][0], w[ti][2], false, false);
        const auto s1 = __builtin_amdgcn_permlane32_swap(w[ti][1], w[ti][3], false, false);
        v4i o = {(int)s0[0], (int)s0[1], (int)s1[0], (int)s1[1]};
        *reinterpret_cast<v4i*>(cj + ti * 32 + lane_off) = o;
      }
    }
  } else {
    // lane holds row i = lane % 32 of a 32 x 32 tile, register e column 8 (e / 4) + 4 (lane / 32) + e % 4
    const size_t row = (size_t)tm * BM + wm * 128 + (lane & 31);       // + ti*32
    const size_t col0 = (size_t)tn * BN + wn * 128 + 4 * half;         // + tj*32 + 8*(e/4) + e%4
    int* plane = g.c + (size_t)t * g.n_pad * g.m_pad + row;
#pragma unroll
    for (int tj = 0; tj < 4; ++tj)
#pragma unroll
      for (int ti = 0; ti < 4; ++ti)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          plane[(col0 + tj * 32 + 8 * (e >> 2) + (e & 3)) * g.m_pad + ti * 32] = acc[ti][tj][e];
  }
  if (!nxt.valid) {
    wait_vmcnt<0>();  // the copies fetched beyond the end of the last tile must have landed before the LDS is given back
    break;
  }
  cur = nxt;
  }  // loop over this workgroup's tiles
#undef OZ2_MFMA
}

__global__ void clear_sync_kernel(unsigned long long* counters, int count) {
  if ((int)threadIdx.x < count) counters[threadIdx.x] = 0ull;
}

}  // namespace

namespace {

// Once per process: the kernels' dynamic LDS limit and the number of compute units (a multiple of 8, one
// workgroup slot each).  Callers hold the library's lock.
int g_cus = 0;
// The tile orders above are written for the eight accelerator dies (XCDs) of the MI355X, on which the hardware
// places workgroup i of a launch on die i % 8.
constexpr int kXcds = 8;
int g_sync_spins = 4096;  // polls per wait of the round synchronisation (each followed by a short sleep); 0: off
hipError_t gemm_setup() {
  if (g_cus) return hipSuccess;
#define OZ2_BOTH(U8, LIST, EARLY)                                              \
  reinterpret_cast<const void*>(gemm_i8_kernel<U8, LIST, EARLY, false>),       \
      reinterpret_cast<const void*>(gemm_i8_kernel<U8, LIST, EARLY, true>)
  const void* kernels[12] = {OZ2_BOTH(false, false, false), OZ2_BOTH(true, false, false), OZ2_BOTH(false, true, false),
                             OZ2_BOTH(true, true, false),   OZ2_BOTH(true, false, true),  OZ2_BOTH(true, true, true)};
#undef OZ2_BOTH
  hipError_t e = hipSuccess;
  for (int i = 0; i < 12 && e == hipSuccess; ++i)
    e = hipFuncSetAttribute(kernels[i], hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  if (e != hipSuccess) return e;
  int dev = 0, n = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  g_cus = n / 8 * 8 < 8 ? 8 : n / 8 * 8;
  return hipSuccess;
}

// num_moduli planes of A' (off_a) times planes of B' (off_b) -> planes of C' (off_c); moduli[t] = modulus of plane t
// b_is_a: the second operand's planes are the first operand's (symmetric product; m_pad == n_pad)
hipError_t launch_gemm(const Oz2Layout& lay, char* ws, int num_moduli, const int* moduli, int64_t kblock, int residue_u8,
                       int triangle, int krange, bool b_is_a, bool check_flag, hipStream_t st) {
  hipError_t e = gemm_setup();
  if (e != hipSuccess) return e;
  if (num_moduli < 1 || num_moduli > OZ2_MAX_PLANES) return hipErrorInvalidValue;
  GemmArgs g;
  g.a = reinterpret_cast<const int8_t*>(ws + lay.off_a);
  g.b = reinterpret_cast<const int8_t*>(ws + (b_is_a ? lay.off_a : lay.off_b));
  if (b_is_a && lay.m_pad != lay.n_pad) return hipErrorInvalidValue;
  g.triangle = triangle;
  g.krange = krange;
  g.skip_flag = check_flag ? reinterpret_cast<const unsigned long long*>(ws + lay.off_flags) : nullptr;
  g.c = reinterpret_cast<int*>(ws + lay.off_c);
  g.m_pad = lay.m_pad;
  g.n_pad = lay.n_pad;
  g.k_pad = lay.k_pad;
  if (lay.m_pad >= ((int64_t)1 << 27)) return hipErrorInvalidValue;  // the epilogue's lane offsets: 31 m_pad + 16 in 32 bits
  g.tiles_m = (int)(lay.m_pad / BM);
  g.tiles_n = (int)(lay.n_pad / BN);
  g.num_moduli = num_moduli;
  const int64_t total = (int64_t)g.tiles_m * g.tiles_n * num_moduli;
  if (total > (int64_t)1 << 30) return hipErrorInvalidValue;
  g.total = (int)total;
  g.chunk = (int)((total + 7) / 8);
  g.superblock = (g.tiles_m % 16 == 0 && g.tiles_n % 16 == 0) ? 1 : 0;
  // list order of the 8 x 4 sub-blocks: general products whose tile grid is a multiple of 8 x 4 but not of 16 x 16
  // (and at least eight rounds of them: with a handful of sub-blocks the range order spreads the tiles better)
  const bool list_order = !g.superblock && triangle == 0 && krange == OZ2_KRANGE_ALL && g.tiles_m % 8 == 0 &&
                          g.tiles_n % 4 == 0 && total / 32 >= 64;
  if (list_order) g.chunk = (int)((total / 32 + 7) / 8) * 32;  // whole rounds of 32 tiles per XCD
  g.ktiles = (int)(lay.k_pad / BK);
  g.ktiles_per_block = (int)(kblock / BK);
  for (int t = 0; t < OZ2_MAX_PLANES; ++t) g.p[t] = t < num_moduli ? (float)moduli[t] : 1.0f;
  // General products: one workgroup per compute unit (each holds one: 128 KiB of LDS, 512 registers per lane),
  // every workgroup walks the work indices of its slot in launch order.  Structured products have tiles of
  // unequal length (or none): there the hardware's dynamic placement of one workgroup per index balances better.
  unsigned grid = (unsigned)(g.chunk * 8);
  g.xcd_sync = nullptr;
  g.full_rounds = 0;
  g.xcds = kXcds;
  g.sync_spins = g_sync_spins;
  if (triangle == 0 && krange == OZ2_KRANGE_ALL) {
    if (grid > (unsigned)g_cus) grid = (unsigned)g_cus;
    // General products: the workgroups of an XCD start the tiles of a round together, which keeps them
    // on the same k-tiles of their shared panels (measured: L2 misses 48.7 GiB per launch every time instead of
    // 50-54 GiB, and 83 GiB in some runs).  The counters are words 8..15 of the flag words that stage 1 clears.
    // Only for inner dimensions above 6144: shorter panels stay in the L2 anyway and the wait for the slowest
    // workgroup of every round costs more than it saves (measured without it: -10 % at k = 1024, -6 % at 2048,
    // -4 % at 4096, -3 % at 6144, -1.5 % at 8192 with 64 rounds but +1 % at 8192 with 448 rounds).
    if (num_moduli > 1 && g.ktiles > 96 && g_sync_spins > 0) {
      g.xcd_sync = reinterpret_cast<unsigned long long*>(ws + lay.off_flags) + 8;
      // rounds in which each of the grid / 8 workgroup slots of every XCD has a tile: all of them in the
      // super-block order (its work count is a multiple of 256); otherwise XCD 7 runs out first
      const int per_xcd = (int)grid / 8;
      const int last = g.total - 7 * g.chunk;  // work items of XCD 7
      g.full_rounds = g.superblock ? (g.chunk * 8) / (int)grid : (last > 0 ? last / per_xcd : 0);
      // list order: the rounds in which all eight XCDs have a sub-block, when a round of the launch (32 workgroups
      // per XCD) is a round of the list
      if (list_order) g.full_rounds = per_xcd == 32 ? (int)(total / 256) : 0;
    }
  }
  // Early arrival at the round synchronisation: with tiles of up to 128 k-tiles (measured at 8192: -1 % of the
  // GEMM time with 448 rounds, -1.5 % with 64); with longer tiles the tighter form keeps the workgroups closer
  // together on their panels and is the faster one.  UINT8 epilogue only.
  const bool early = residue_u8 && g.xcd_sync != nullptr && g.ktiles <= 128;
  const dim3 grd(grid), thr(kThreads);
  // tiles walked in one k-block (the usual case) take the instantiation without the reduction between k-blocks
  const bool kblocked = g.ktiles_per_block < g.ktiles;
#define OZ2_GEMM(U8, LIST, EARLY)                                                                   \
  do {                                                                                              \
    if (kblocked)                                                                                   \
      hipLaunchKernelGGL((gemm_i8_kernel<U8, LIST, EARLY, true>), grd, thr, kLdsBytes, st, g);      \
    else                                                                                            \
      hipLaunchKernelGGL((gemm_i8_kernel<U8, LIST, EARLY, false>), grd, thr, kLdsBytes, st, g);     \
  } while (0)
  if (!residue_u8 && list_order)
    OZ2_GEMM(false, true, false);
  else if (!residue_u8)
    OZ2_GEMM(false, false, false);
  else if (list_order && early)
    OZ2_GEMM(true, true, true);
  else if (list_order)
    OZ2_GEMM(true, true, false);
  else if (early)
    OZ2_GEMM(true, false, true);
  else
    OZ2_GEMM(true, false, false);
#undef OZ2_GEMM
  return hipGetLastError();
}

}  // namespace

hipError_t oz2_gemm_setup() { return gemm_setup(); }

void oz2_gemm_set_sync_spins(int spins) { g_sync_spins = spins; }

// The round synchronisation counts on counters that are zero at launch.  Stage 1 clears them with the row
// maxima; a GEMM launched without a stage 1 before it (the staged entry point called again) clears them here.
hipError_t oz2_launch_clear_sync(const Oz2Layout& lay, char* ws, hipStream_t st) {
  hipLaunchKernelGGL(clear_sync_kernel, dim3(1), dim3(64), 0, st,
                     reinterpret_cast<unsigned long long*>(ws + lay.off_flags) + 8, kXcds);
  return hipGetLastError();
}

hipError_t oz2_launch_stage2(const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int64_t kblock, int residue_u8,
                             int triangle, int krange, int check_flag, hipStream_t st) {
  return launch_gemm(lay, ws, plan.N, plan.moduli, kblock, residue_u8, triangle, krange, triangle != 0, check_flag != 0, st);
}

// The seven products per modulus of the Strassen form: 7 N planes of half the extents of lay, plane 7 t + s
// reduced modulo p_t in the epilogue (UINT8 residues).
hipError_t oz2_launch_strassen_gemm(const Oz2Plan& plan, const Oz2Layout& lay, char* ws, int64_t kblock, int check_flag,
                                    hipStream_t st) {
  Oz2Layout half = lay;
  half.m_pad = lay.m_pad / 2;
  half.n_pad = lay.n_pad / 2;
  half.k_pad = lay.k_pad / 2;
  if (half.m_pad % BM || half.n_pad % BN || half.k_pad % BK) return hipErrorInvalidValue;
  int moduli[OZ2_MAX_PLANES];
  for (int t = 0; t < plan.N; ++t)
    for (int s = 0; s < 7; ++s) moduli[7 * t + s] = plan.moduli[t];
  return launch_gemm(half, ws, 7 * plan.N, moduli, kblock, 1, 0, OZ2_KRANGE_ALL, false, check_flag != 0, st);
}

// One plain INT8 product with INT32 output and no modular reduction between k-blocks: the caller guarantees
// k_pad * 64 * 64 < 2^31.
hipError_t oz2_launch_bound_gemm(const Oz2Layout& lay, char* ws, bool symmetric, hipStream_t st) {
  const int one = 1;
  return launch_gemm(lay, ws, 1, &one, lay.k_pad, 0, 0, OZ2_KRANGE_ALL, symmetric, false, st);
}
