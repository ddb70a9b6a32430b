// Kernel template of the bf16 MFMA GEMM family (gfx950) and its per-tile-shape launcher.  Each
// tile shape is instantiated in a translation unit of its own (gemm_bf16_<shape>.hip) so that the
// shapes compile in parallel; gemm_bf16.hip chooses among them.
//
// Design (MI355X):
//   * a workgroup computes a BM x BN tile of C, K advanced BK at a time; every wavefront owns a
//     (32 TM) x 64 part as TM x 2 accumulators of v_mfma_f32_32x32x16_bf16 (TM = 4: 128 x 64, the
//     shape with the fewest LDS bytes per FLOP that fits the register file, or TM = 2);
//   * WK > 1 ("k-groups"): WK sets of wavefronts share one tile position and split the k-steps of
//     every k-tile among them; their accumulators are summed through LDS at the end in a fixed
//     order.  This gives a narrow tile (256 x 128: twice as many tiles for a given C) the full
//     128 x 64 wave shape with eight wavefronts per CU;
//   * operand tiles go global -> LDS directly (global_load_lds_dwordx4, 16 B per lane, no VGPR
//     staging) into a ring of kStages k-tiles;
//   * because those loads place lane i's 16 B at slot i of a 1 KiB run, bank-conflict avoidance
//     is done by permuting WHICH 16-byte chunk each lane fetches (XOR swizzle), not by padding;
//   * a k-contiguous operand is read back with ds_read_b128 (8 consecutive k for one row);
//     an m/n-contiguous operand is read with ds_read_b64_tr_b16, the LDS transpose load, so no
//     operand is ever transposed in memory or registers;
//   * the MFMA is issued with its operands exchanged (B-fragment as the instruction's A), which
//     leaves every lane holding 4 consecutive n of one row m; the epilogue transposes 32x64 slabs
//     through LDS so that global stores (and aux / old-C loads) are contiguous 256 B row pieces;
//   * fragments are fetched from LDS ahead of the MFMAs that use them, in an order pinned by
//     scheduling barriers, and the fetch-ahead runs across k-tile boundaries (the barrier that
//     publishes the next k-tile stands where a wave has fetched its last fragment of this one);
//   * ragged M / N: rows past the edge are clamped to the last row at load time (they only reach
//     outputs that are not stored); ragged K: chunks past K are zero-filled in LDS;
//   * one launch can sum up to 3 (A, B, K) segments into one C, or run up to 4 independent
//     problems (grouped launch), so that small outputs still fill the chip;
//   * workgroup ids are dealt round-robin to the 8 XCDs by hardware, so ids are remapped to make
//     each XCD (own L2) work on a compact patch of C.
#pragma once
#include <algorithm>
#include <cstdio>
#include <type_traits>

#include "gemm_bf16.h"
#include "timing.h"

namespace mtf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// BM x BN tile, WM x WN wave positions, WK k-groups, k-tiles of BK, L2 patches of GROUP_M tile
// rows, STAGES k-tiles resident in LDS.
template <int BM_, int BN_, int WM_, int WN_, int WK_, int BK_, int GROUP_M_, int STAGES_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, WK = WK_, BK = BK_;
  static constexpr int kPositions = WM * WN;  // wave positions in the tile
  static constexpr int kWaves = kPositions * WK, kThreads = kWaves * 64;
  static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;  // 32x32 accumulators per wave
  static constexpr int kATile = BM * BK * 2, kBTile = BN * BK * 2, kStage = kATile + kBTile;  // bytes
  static constexpr int kGroupM = GROUP_M_;  // tile rows per L2 patch
  static constexpr int kStages = STAGES_;   // k-tiles resident in LDS (one computing, the rest in flight)
  static constexpr int kSteps = BK / 16 / WK;  // k-steps (of 16) a wave runs per k-tile
  // k-steps of fragments fetched ahead; kFragAhead + 1 must divide kSteps
  static constexpr int kFragAhead = (TM * TN >= 8 || kSteps < 4) ? 1 : 3;
  // register budget: two wavefronts per SIMD where the LDS lets two workgroups of 4 waves (or one
  // of 8) share a CU, else one
  static constexpr int kWavesPerSimd = (kWaves == 4 && kStages * kStage > 80 * 1024) ? 1 : 2;
  static_assert(BK == 32 || BK == 64, "k-tile of 32 or 64");
  static_assert(WK == 1 || WK == 2, "one or two k-groups");
  static_assert(kSteps >= 2 && TN == 2, "wave tiles are 64 columns wide, at least two k-steps per k-tile");
  static_assert(WK == 1 || TM % 2 == 0, "k-groups split the wave tile's rows between them at the end");
};

// Slot p * nseg + s of A/B/K is k-segment s of problem p (one problem unless the launch is
// grouped; every problem of a group has nseg segments and its own M, N, C and leading dims).
struct GemmArgs {
  const bf16_t* A[kMaxSlots];
  const bf16_t* B[kMaxSlots];
  int K[kMaxSlots];
  int nseg, ngroup;
  int M[kMaxGroup], N[kMaxGroup];
  int64_t lda[kMaxGroup], ldb[kMaxGroup], ldc[kMaxGroup];
  void* C[kMaxGroup];
  const bf16_t* aux;
  const bf16_t* bias;
  const float* row_scale;
  float alpha;
  int accumulate;
  int tiles_m[kMaxGroup], tiles_n[kMaxGroup];
  int xcds_per_problem;  // grouped launch: > 0 when every XCD works on one problem only, else 0
  int batch1;
  int64_t sA0, sA1, sB0, sB1, sC0, sC1;
};

// Direct global -> LDS load of 16 bytes per lane: lane i's bytes land at lds_addr + 16*i.
// Written as inline assembly on purpose: through the compiler's builtin, every later LDS read
// is made to wait for ALL outstanding loads of this kind (it cannot tell the two stages apart
// once more than a handful of such loads exist), which would serialise load and compute.  Here
// the waits are placed by hand (wait_for_tile below).  m0 carries the LDS address; nothing else in
// these kernels uses m0.
__device__ __forceinline__ void load16_to_lds(const char* uniform_base, uint32_t lane_offset,
                                              uint32_t lds_addr_uniform) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2\n"
      :
      : "s"(lds_addr_uniform), "v"(lane_offset), "s"(uniform_base)
      : "memory", "m0");
}

__device__ __forceinline__ uint32_t lds_address(const char* p) {
  return (uint32_t)(uintptr_t)LDS_PTR(const char, p);
}

// Chunk permutation of a k-contiguous operand tile: LDS row = one m (or n) = BK * 2 bytes.  The
// 16 lanes a ds_read_b128 serves together read consecutive rows at one chunk index; rows whose
// starts are a multiple of 256 B apart would hit the same banks, so the chunk is XORed with the
// row's index among those.
template <int BK>
__device__ __forceinline__ int kc_swizzle(int r) {
  return BK == 64 ? (r >> 1) & 7 : (r >> 2) & 3;
}

// One operand tile (ROWS of the M/N index x BK of k) global -> LDS, in 1 KiB runs (one wave-wide
// load each).
//   k-contiguous: LDS row = one m (or n), BK*2 B = BK/8 chunks; chunk c of row r sits at c ^ kc_swizzle(r)
//   mn-contiguous: LDS row = one k, 2*ROWS B; chunk c of row k sits at c ^ ((k&3)<<2)
// TileLoader keeps, per lane, the loop-invariant byte offsets of its chunks relative to the tile's
// first element (rows / columns beyond the matrix edge are clamped to the last valid one: they
// only feed C elements that are never stored); the tile origin itself is wave-uniform.
template <bool KCONTIG, int ROWS, int NWAVES, int BK>
struct TileLoader {
  static constexpr int NL = ROWS * BK * 2 / 1024 / NWAVES;  // loads per lane per tile
  static constexpr int CPK = BK / 8;                        // k-contiguous: chunks per row
  static constexpr int RPK = 64 / CPK;                      // k-contiguous: rows per run
  static constexpr int CPR = ROWS / 8;                      // mn-contiguous: 16-byte chunks per k-row
  static constexpr int RPR = 64 / CPR;                      // mn-contiguous: k-rows per run
  static_assert(NL >= 1 && NL * NWAVES * 1024 == ROWS * BK * 2, "whole runs per wave");
  uint32_t off[NL];  // byte offset of this lane's chunk i from the tile origin (k0 = 0)
  int kpos[NL];      // k of the chunk (k-contiguous) or k-row (mn-contiguous), relative to k0

  __device__ __forceinline__ void init(int64_t ld, int mn0, int mn_limit, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int run = i * NWAVES + wave;
      if (KCONTIG) {
        const int r = run * RPK + lane / CPK;
        const int c = (lane % CPK) ^ kc_swizzle<BK>(r);
        const int mn = min(mn0 + r, mn_limit - 1) - mn0;
        off[i] = (uint32_t)((int64_t)mn * ld * 2 + c * 16);
        kpos[i] = c * 8;
      } else {
        const int kr = run * RPR + lane / CPR;
        const int c = (lane % CPR) ^ ((kr & 3) << 2);
        const int mn = min(mn0 + c * 8, mn_limit - 8) - mn0;
        off[i] = (uint32_t)((int64_t)kr * ld * 2 + mn * 2);
        kpos[i] = kr;
      }
    }
  }

  // A tile that lies entirely inside K.
  __device__ __forceinline__ void issue_full(const char* origin, char* tile, int wave) const {
#pragma unroll
    for (int i = 0; i < NL; ++i)
      load16_to_lds(origin, off[i], lds_address(tile) + (i * NWAVES + wave) * 1024);
  }

  // origin: address of element (mn0, k0) of the operand (wave-uniform).
  __device__ __forceinline__ void issue(const char* origin, char* tile, int wave, int lane,
                                        int k_left) const {
    if (k_left >= BK) {
#pragma unroll
      for (int i = 0; i < NL; ++i)
        load16_to_lds(origin, off[i], lds_address(tile) + (i * NWAVES + wave) * 1024);
    } else {  // ragged last k-tile: chunks past K become zeros
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        char* run = tile + (i * NWAVES + wave) * 1024;
        if (kpos[i] < k_left)
          load16_to_lds(origin, off[i], lds_address(run));
        else
          *LDS_PTR(u32x4, run + lane * 16) = u32x4{0u, 0u, 0u, 0u};
      }
    }
  }
};

// MFMA operand fragment for 32 consecutive m (or n) starting at mn_base and the 16 k of step ks
// (counted within the k-tile): lane l gets index mn_base + l%32 and k = ks*16 + (l/32)*8 + 0..7.
template <bool KCONTIG, int ROWS, int BK>
__device__ __forceinline__ bf16x8 read_fragment(const char* tile, int mn_base, int ks, int lane) {
  if (KCONTIG) {
    const int r = mn_base + (lane & 31);
    const int c = ks * 2 + (lane >> 5);
    return *LDS_PTR(const bf16x8, tile + r * (BK * 2) + ((c ^ kc_swizzle<BK>(r)) << 4));
  } else {
    // Transpose load: in each group of 16 lanes, lane j points at 4 consecutive n of k-row j/4;
    // the hardware hands lane i the 4 k-values of column i.
    constexpr int kPitch = ROWS * 2;
    const int g = lane >> 4, j = lane & 15;
    const int n = mn_base + (g & 1) * 16 + (j & 3) * 4;
    const int krow = ks * 16 + (g >> 1) * 8 + (j >> 2);
    const int chunk = (n >> 3) ^ ((j >> 2) << 2);  // (krow & 3) == j >> 2
    const char* p = tile + krow * kPitch + (chunk << 4) + (n & 7) * 2;
    union {
      s16x4 h[2];
      bf16x8 v;
    } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p + 4 * kPitch));
    return u.v;
  }
}

template <class Cfg, bool A_K, bool B_K, int EPI, bool OUT_BF16>
__global__ void __launch_bounds__(Cfg::kThreads, Cfg::kWavesPerSimd) gemm_bf16_kernel(GemmArgs g) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, TM = Cfg::TM, TN = Cfg::TN, BK = Cfg::BK, WK = Cfg::WK;
  // Ring of kStages k-tiles: one being computed on, the others in flight.
  constexpr int NS = Cfg::kStages;
  __shared__ __attribute__((aligned(1024))) char ring[NS * Cfg::kStage];

  // ---- which tile: XCD-aware remap, then patches of kGroupM tile rows
  // Workgroups go to the 8 XCDs round-robin in dispatch order (gridDim.x is a multiple of 8), and
  // each XCD has an L2 of its own.  One problem: XCD x takes a contiguous run of the tile order
  // below.  A group of equally sized problems, 1, 2 or 4 XCDs per problem: an XCD takes tiles of
  // one problem only, so that it fetches that problem's operands and nobody else's (with every
  // problem spread over all XCDs, each XCD fetched the narrow operand of every problem).
  // Otherwise blockIdx.y picks the problem and each problem is spread over all XCDs.
  int grp, t;
  if (g.xcds_per_problem > 0) {
    const int flat = blockIdx.y * gridDim.x + blockIdx.x, xcd = flat & 7, slot = flat >> 3;
    const int per_xcd = (gridDim.x * g.ngroup) >> 3;
    grp = xcd / g.xcds_per_problem;
    t = (xcd % g.xcds_per_problem) * per_xcd + slot;
  } else {
    grp = g.ngroup > 1 ? blockIdx.y : 0;
    t = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  }
  const int M = g.M[grp], N = g.N[grp], tiles_m = g.tiles_m[grp], tiles_n = g.tiles_n[grp];
  const int64_t lda = g.lda[grp], ldb = g.ldb[grp], ldc = g.ldc[grp];
  if (t >= tiles_m * tiles_n) return;
  const int per_group = Cfg::kGroupM * tiles_n;
  const int first_m = (t / per_group) * Cfg::kGroupM;
  const int rows = min(tiles_m - first_m, Cfg::kGroupM);
  const int tile_m = first_m + (t % per_group) % rows;
  const int tile_n = (t % per_group) / rows;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int zb = g.ngroup > 1 ? 0 : blockIdx.y;
  const int z0 = zb / g.batch1, z1 = zb % g.batch1;
  const int64_t offA = z0 * g.sA0 + z1 * g.sA1, offB = z0 * g.sB0 + z1 * g.sB1,
                offC = z0 * g.sC0 + z1 * g.sC1;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kg = wave / Cfg::kPositions;   // k-group of this wave (0 when WK == 1)
  const int pos = wave % Cfg::kPositions;  // its position in the tile
  const int wm = pos / Cfg::WN, wn = pos % Cfg::WN;  // this wave's (32*TM) x (32*TN) part
  const int wave_m = wm * (32 * TM), wave_n = wn * (32 * TN);
  const int ks0 = kg * Cfg::kSteps;  // first k-step (within a k-tile) this wave computes

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  TileLoader<A_K, BM, Cfg::kWaves, BK> load_a;
  TileLoader<B_K, BN, Cfg::kWaves, BK> load_b;
  load_a.init(lda, m0, M, wave, lane);
  load_b.init(ldb, n0, N, wave, lane);
  const int64_t a_tile0 = A_K ? (int64_t)m0 * lda : m0, a_kstep = A_K ? 1 : lda;
  const int64_t b_tile0 = B_K ? (int64_t)n0 * ldb : n0, b_kstep = B_K ? 1 : ldb;

  // k-tiles of all segments, in order.  Everything the per-tile issue needs is brought into
  // scalar registers once (indexing the kernel arguments inside the loop costs a scalar memory
  // load and a wait per k-tile) and then advanced incrementally.
  const char* seg_a[kMaxSegments];
  const char* seg_b[kMaxSegments];
  int seg_k[kMaxSegments];
  int total_tiles = 0;
#pragma unroll
  for (int s = 0; s < kMaxSegments; ++s) {
    const int slot = min(grp * g.nseg + s, kMaxSlots - 1);
    seg_a[s] = reinterpret_cast<const char*>(g.A[slot] + offA + a_tile0);
    seg_b[s] = reinterpret_cast<const char*>(g.B[slot] + offB + b_tile0);
    seg_k[s] = s < g.nseg ? g.K[slot] : 0;
    total_tiles += (seg_k[s] + BK - 1) / BK;
  }
  const int64_t a_tile_bytes = a_kstep * (BK * 2), b_tile_bytes = b_kstep * (BK * 2);
  const char *next_a = seg_a[0], *next_b = seg_b[0];  // operand origins of the next tile to issue
  int next_seg = 0, next_left = seg_k[0];             // its segment and the k still ahead in it
  uint32_t full_hist = 0;                             // bit i: the (i+1)-th latest issued tile was full

  auto issue_next = [&](char* st) {
    // The common case first, under one branch: a full k-tile of the segment in progress.  (This
    // runs once per k-tile in every wave, between MFMAs; the general path below is some hundred
    // scalar instructions and a dozen branches.)
    if (next_left >= BK) {
      load_a.issue_full(next_a, st, wave);
      load_b.issue_full(next_b, st + Cfg::kATile, wave);
      full_hist = (full_hist << 1) | 1u;
    } else {
      // skip exhausted (or empty) segments
#pragma unroll
      for (int q = 0; q < kMaxSegments - 1; ++q)
        if (next_left <= 0 && next_seg == q) {
          next_seg = q + 1;
          next_a = seg_a[q + 1];
          next_b = seg_b[q + 1];
          next_left = seg_k[q + 1];
        }
      load_a.issue(next_a, st, wave, lane, next_left);
      load_b.issue(next_b, st + Cfg::kATile, wave, lane, next_left);
      full_hist = (full_hist << 1) | (next_left >= BK ? 1u : 0u);
    }
    next_a += a_tile_bytes;
    next_b += b_tile_bytes;
    next_left -= BK;
  };
  // A wave runs kSteps steps of 16 per k-tile (its k-group's share).  LDS->register latency is
  // several hundred cycles, more than the MFMAs of one step take, so fragments are fetched kAhead
  // steps ahead into a rotating set of kAhead+1 register buffers (one LDS read slotted in front of
  // each of the first TM+TN MFMAs of a step) - and the fetch-ahead runs across k-tile boundaries:
  // the barrier that publishes tile kt+1 stands kAhead steps before the end of tile kt, right
  // where this wave has fetched the last fragment of tile kt.  The MFMAs still to do on tile kt
  // then cover both the latency of the first fragments of tile kt+1 and the issue of the loads of
  // a further tile.
  constexpr int kAhead = Cfg::kFragAhead;
  constexpr int kSteps = Cfg::kSteps;
  constexpr bool kStaggerIssue = Cfg::kWaves == 8 && Cfg::kWavesPerSimd == 2;
  static_assert(kSteps % (kAhead + 1) == 0, "fragment buffers must rotate back at a tile boundary");
  static_assert(kAhead < kSteps, "fetch-ahead of at most one k-tile");
  bf16x8 af[kAhead + 1][TM], bf[kAhead + 1][TN];
  auto fetch = [&](const char* st, int ks, bf16x8* a_dst, bf16x8* b_dst, int which) {
    // ks: step within this wave's share; which: 0..TN-1 -> B fragment, TN..TN+TM-1 -> A fragment
    if (which < TN)
      b_dst[which] = read_fragment<B_K, BN, BK>(st + Cfg::kATile, wave_n + which * 32, ks0 + ks, lane);
    else
      a_dst[which - TN] = read_fragment<A_K, BM, BK>(st, wave_m + (which - TN) * 32, ks0 + ks, lane);
  };
  // Loads complete in issue order, so "tile kt has landed" = at most the loads of the newer tiles
  // are still outstanding.  A ragged tile may issue fewer than the usual number of loads per wave,
  // so only full newer tiles are counted (a smaller allowance only waits longer).
  constexpr int kLoadsPerTile =
      TileLoader<A_K, BM, Cfg::kWaves, BK>::NL + TileLoader<B_K, BN, Cfg::kWaves, BK>::NL;
  // Waits until at most n of this wave's loads are outstanding (n rounded down to one of the
  // counts that occur: the immediate of s_waitcnt is a compile-time constant).
  auto wait_vmcnt = [&](int n) {
#define MTF_VMCNT_CASE(v)                                         \
  if (n >= (v)) {                                                 \
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(v) : "memory");      \
    return;                                                       \
  }
    if (NS >= 3) {
      MTF_VMCNT_CASE(2 * kLoadsPerTile)
    }
    MTF_VMCNT_CASE(kLoadsPerTile)
#undef MTF_VMCNT_CASE
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };
  // Loads still allowed in flight when tile kt must have landed: those of the `newer` tiles issued
  // after it (only whole tiles are counted).
  auto wait_for_tile = [&](int kt) {
    const int newer = min(NS - 2, total_tiles - 1 - kt);  // tiles issued after tile kt
    const int allowed = newer > 0 ? __builtin_popcount(full_hist & ((1u << newer) - 1u)) : 0;
    wait_vmcnt(allowed * kLoadsPerTile);
    // Passing the barrier also means every wave has fetched its last fragment of the tile being
    // computed on (the barrier waits for the wave's own LDS reads first), so that tile's stage
    // may be overwritten by the next issue.
    __syncthreads();
  };
  // MFMAs of tile kt (in stage `st`); HAS_NEXT: tile kt+1 exists (in `st_next`), and `fill`
  // (or nullptr) is the stage - the one tile kt occupies when NS == 2 - a further tile goes to.
  auto compute = [&](auto has_next, int kt, const char* st, const char* st_next, char* fill) {
    constexpr bool HAS_NEXT = decltype(has_next)::value;
#pragma unroll
    for (int ks = 0; ks < kSteps; ++ks) {
      const int cur = ks % (kAhead + 1), nxt = (ks + kAhead) % (kAhead + 1);
      const bool crosses = ks + kAhead >= kSteps;  // the fetch of this step reads the next tile
      // The two waves of a SIMD (w and w + 4) pass the barrier together; were both to issue their
      // loads of the further tile right away, the matrix pipe would idle meanwhile.  The second
      // one does this step's MFMAs first (any time after the barrier is safe for the stage, and
      // the loads have a whole k-tile to land).
      const bool issue_late = kStaggerIssue && wave >= 4;
      if (HAS_NEXT && ks + kAhead == kSteps) {
        wait_for_tile(kt + 1);
        if (fill && !issue_late) issue_next(fill);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int slot = i * TN + j;  // MFMA number within the step
          if (slot < TM + TN) {
            if (!crosses)
              fetch(st, ks + kAhead, af[nxt], bf[nxt], slot);
            else if (HAS_NEXT)
              fetch(st_next, ks + kAhead - kSteps, af[nxt], bf[nxt], slot);
          }
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
          // keep this read-then-MFMA order: left alone, the scheduler sinks every read to just
          // before its first use (fewer live registers) and the overlap is lost
          __builtin_amdgcn_sched_barrier(0);
        }
      if (HAS_NEXT && ks + kAhead == kSteps && fill && issue_late) {
        issue_next(fill);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  // Prologue: fill the ring (NS == 2: both stages are free, so two tiles go out at once), wait
  // for tile 0 and fetch its first kAhead steps.
#pragma unroll
  for (int p = 0; p < NS; ++p)
    if (p < total_tiles) issue_next(ring + p * Cfg::kStage);
  if (total_tiles > 0) {
    {
      // tiles 1 .. NS-1 were issued after tile 0
      const int newer = min(NS - 1, total_tiles - 1);
      const int allowed = newer > 0 ? __builtin_popcount(full_hist & ((1u << newer) - 1u)) : 0;
      wait_vmcnt(allowed * kLoadsPerTile);
      __syncthreads();
    }
#pragma unroll
    for (int p = 0; p < kAhead; ++p)
#pragma unroll
      for (int w = 0; w < TM + TN; ++w) fetch(ring, p, af[p], bf[p], w);
    // Tile kt sits in stage kt % NS.  At the boundary inside compute(kt) the stage of tile kt is
    // released and refilled with tile kt+NS.
    int stage = 0;
    for (int kt = 0; kt + 1 < total_tiles; ++kt) {
      const int nstage = stage + 1 == NS ? 0 : stage + 1;
      compute(std::true_type{}, kt, ring + stage * Cfg::kStage, ring + nstage * Cfg::kStage,
              kt + NS < total_tiles ? ring + stage * Cfg::kStage : nullptr);
      stage = nstage;
    }
    compute(std::false_type{}, total_tiles - 1, ring + stage * Cfg::kStage, nullptr, nullptr);
  }

  // The epilogue stores the wave tile as 32-row slabs; with k-groups a wave stores its group's
  // half of them.  The mask operand of a slab (the only global read on the epilogue's critical
  // path) is requested one slab ahead, the first slab's before the barrier below - from clamped,
  // always valid addresses, so that the loads need no branch around them.
  auto my_slab = [&](int i) { return WK == 1 || (i / (TM / 2)) == kg; };
  // Read-back shape: a lane handles kW consecutive columns of one row, 16 bytes of the output
  // (4 fp32 or 8 bf16), so that every global access is 16 bytes per lane whatever the output type.
  constexpr int kW = OUT_BF16 ? 8 : 4;          // columns per lane
  constexpr int kLanesPerRow = 64 / kW;         // 16 or 8
  constexpr int kRowsPerIt = 64 / kLanesPerRow; // rows a wave covers per instruction: 4 or 8
  constexpr int kIts = 32 / kRowsPerIt;         // instructions per 32-row slab: 8 or 4
  struct alignas(kW * 2) AuxVec {
    uint32_t w[kW / 2];  // kW bf16 values
  };
  AuxVec aux_v[2][kIts];
  auto request_mask = [&](int i) {
    const int out_row_ = lane / kLanesPerRow, out_col_ = (lane % kLanesPerRow) * kW;
#pragma unroll
    for (int it = 0; it < kIts; ++it) {
      const int mc = min(m0 + wave_m + i * 32 + it * kRowsPerIt + out_row_, M - 1);
      const int nc = min(n0 + wave_n + out_col_, N - kW);  // N % 8 == 0
      aux_v[i & 1][it] = *reinterpret_cast<const AuxVec*>(g.aux + offC + (int64_t)mc * ldc + nc);
    }
  };
  if (EPI == MTF_EPI_MASK_GT0) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
      if (my_slab(i) && (i == 0 || !my_slab(i - 1))) request_mask(i);
  }
  __syncthreads();  // everyone is done reading the last k-tile: the ring is free
  // ---- k-groups: the two waves at one tile position hold partial sums over disjoint k.  They
  // exchange halves through LDS (one 32-row slab per wave and round, lane-major so that every
  // access is a conflict-free 1 KiB run): group 0 ends with the complete upper TM/2 slabs, group 1
  // with the lower ones.  own + partner's, a fixed order.
  if (WK == 2) {
    constexpr int H = TM / 2;
    char* mine = ring + wave * (TN * 4 * 1024);
    const char* theirs = ring + (wave ^ Cfg::kPositions) * (TN * 4 * 1024);
    static_assert(Cfg::kWaves * TN * 4 * 1024 <= NS * Cfg::kStage, "exchange area fits the ring");
#pragma unroll
    for (int r = 0; r < (WK == 2 ? H : 0); ++r) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v;
          if (kg == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[H + r][j][q * 4 + e];
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[r][j][q * 4 + e];
          }
          *LDS_PTR(f32x4, mine + ((j * 4 + q) * 64 + lane) * 16) = v;
        }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v = *LDS_PTR(const f32x4, theirs + ((j * 4 + q) * 64 + lane) * 16);
          if (kg == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[r][j][q * 4 + e] += v[e];
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[H + r][j][q * 4 + e] += v[e];
          }
        }
      __syncthreads();
    }
  }
  // ---- epilogue.  A lane holds, per accumulator, one row m and 4 x 4 consecutive n: stored
  // directly that would be 16-byte pieces scattered over 32 rows per instruction.  Instead each
  // wave passes its 32 x 64 accumulator slabs through a private LDS area (the operand ring is
  // free now) and reads them back row-wise, so every global access is 16 lanes x 16 B = one
  // contiguous 256 B row segment; aux / old-C reads of the fused epilogues get the same shape.
  constexpr int kPitch = 64 * 4 + 16;  // fp32 row + 16 B: row-to-row bank shift of 4
  static_assert(Cfg::kWaves * 32 * kPitch <= NS * Cfg::kStage, "slab area fits the ring");
  char* slab = ring + wave * (32 * kPitch);
  const int lane_m = lane & 31, lane_h = lane >> 5;
  const int out_row = lane / kLanesPerRow, out_col = (lane % kLanesPerRow) * kW;
  void* const Cg = g.C[grp];
  // a lane reads back the same kW columns of every slab: its bias values are loaded once
  float biasv[kW];
#pragma unroll
  for (int e = 0; e < kW; ++e) biasv[e] = 0.f;
  if (g.bias && n0 + wave_n + out_col < N) {
#pragma unroll
    for (int e = 0; e < kW; e += 2) {
      const uint32_t b2 = *reinterpret_cast<const uint32_t*>(g.bias + n0 + wave_n + out_col + e);
      biasv[e] = __uint_as_float(b2 << 16);
      biasv[e + 1] = __uint_as_float(b2 & 0xffff0000u);
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (!my_slab(i)) continue;  // the other k-group stores this slab
    if (EPI == MTF_EPI_MASK_GT0 && i + 1 < TM && my_slab(i + 1)) request_mask(i + 1);
    // The old C of an accumulating store is requested for the whole slab before anything waits on
    // it (clamped addresses again): one memory round trip per slab, hidden behind the slab's pass
    // through LDS, instead of one per row group.
    AuxVec old_bf[kIts];
    float4 old_f[kIts];
    if (g.accumulate) {
#pragma unroll
      for (int it = 0; it < kIts; ++it) {
        const int mc = min(m0 + wave_m + i * 32 + it * kRowsPerIt + out_row, M - 1);
        const int nc = min(n0 + wave_n + out_col, N - kW);  // N % 8 == 0
        const int64_t idc = offC + (int64_t)mc * ldc + nc;
        if (OUT_BF16)
          old_bf[it] = *reinterpret_cast<const AuxVec*>(static_cast<const bf16_t*>(Cg) + idc);
        else
          old_f[it] = *reinterpret_cast<const float4*>(static_cast<const float*>(Cg) + idc);
      }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = g.alpha * acc[i][j][q * 4 + e];
        *LDS_PTR(f32x4, slab + lane_m * kPitch + (j * 32 + q * 8 + lane_h * 4) * 4) = v;
      }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < kIts; ++it) {
      const int r = it * kRowsPerIt + out_row;
      float v[kW];
#pragma unroll
      for (int h4 = 0; h4 < kW / 4; ++h4) {
        const f32x4 t = *LDS_PTR(const f32x4, slab + r * kPitch + (out_col + h4 * 4) * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[h4 * 4 + e] = t[e];
      }
      const int m = m0 + wave_m + i * 32 + r;
      const int n = n0 + wave_n + out_col;
      if (m >= M || n >= N) continue;
      const int64_t idx = offC + (int64_t)m * ldc + n;
      if (g.row_scale) {
        const float rs = g.row_scale[(int64_t)zb * M + m];
#pragma unroll
        for (int e = 0; e < kW; ++e) v[e] *= rs;
      }
      if (g.accumulate) {
        if (OUT_BF16) {
#pragma unroll
          for (int e = 0; e < kW; e += 2) {
            v[e] += __uint_as_float(old_bf[it].w[e / 2] << 16);
            v[e + 1] += __uint_as_float(old_bf[it].w[e / 2] & 0xffff0000u);
          }
        } else {
          v[0] += old_f[it].x;
          v[1] += old_f[it].y;
          v[2] += old_f[it].z;
          v[3] += old_f[it].w;
        }
      }
#pragma unroll
      for (int e = 0; e < kW; ++e) v[e] += biasv[e];
      if (EPI == MTF_EPI_RELU) {
#pragma unroll
        for (int e = 0; e < kW; ++e) v[e] = fmaxf(v[e], 0.f);
      } else if (EPI == MTF_EPI_MASK_GT0) {
        // bf16 > 0  <=>  sign bit clear and magnitude non-zero
        const AuxVec mk = aux_v[i & 1][it];
#pragma unroll
        for (int e = 0; e < kW; ++e) {
          const uint32_t w = (e & 1) ? (mk.w[e / 2] >> 16) : (mk.w[e / 2] & 0xffffu);
          v[e] = (w != 0u && w < 0x8000u) ? v[e] : 0.f;
        }
      }
      if (OUT_BF16) {
        AuxVec o;
#pragma unroll
        for (int e = 0; e < kW; e += 2) o.w[e / 2] = pack_bf16x2(v[e], v[e + 1]);
        *reinterpret_cast<AuxVec*>(static_cast<bf16_t*>(Cg) + idx) = o;
      } else {
        *reinterpret_cast<float4*>(static_cast<float*>(Cg) + idx) = make_float4(v[0], v[1], v[2], v[3]);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

template <class Cfg, bool A_K, bool B_K, int EPI, bool OUT_BF16>
int launch_instance(const GemmArgs& a, int batch, hipStream_t stream) {
  // name as a profiler prints the instantiation
  struct Name {
    char text[96];  // fits mtf_kernel_time::kernel
    Name() {
      std::snprintf(text, sizeof text, "gemm_bf16_kernel<TileCfg<%d, %d, %d, %d, %d, %d, %d, %d>, %s, %s, %d, %s>",
                    Cfg::BM, Cfg::BN, Cfg::WM, Cfg::WN, Cfg::WK, Cfg::BK, Cfg::kGroupM, Cfg::kStages,
                    A_K ? "true" : "false", B_K ? "true" : "false", EPI, OUT_BF16 ? "true" : "false");
    }
  };
  static const Name name_once;  // initialised once, also when two host threads launch at the same time
  const char* name = name_once.text;
  GemmArgs args = a;
  int64_t tiles = 0;
  double flops = 0, bytes = 0;
  for (int p = 0; p < a.ngroup; ++p) {
    args.tiles_m[p] = (int)ceil_div(a.M[p], Cfg::BM);
    args.tiles_n[p] = (int)ceil_div(a.N[p], Cfg::BN);
    tiles = std::max<int64_t>(tiles, (int64_t)args.tiles_m[p] * args.tiles_n[p]);
    double ktot = 0;
    for (int s = 0; s < a.nseg; ++s) ktot += a.K[p * a.nseg + s];
    flops += 2.0 * a.M[p] * a.N[p] * ktot * batch;
    bytes += batch * (2.0 * ktot * (a.M[p] + a.N[p]) + (double)a.M[p] * a.N[p] * (OUT_BF16 ? 2 : 4));
  }
  if (tiles > (1 << 28)) return fail(MTF_ERR_UNSUPPORTED, "too many tiles");
  bool same_count = true;
  for (int p = 1; p < a.ngroup; ++p)
    same_count = same_count && args.tiles_m[p] * args.tiles_n[p] == args.tiles_m[0] * args.tiles_n[0];
  args.xcds_per_problem = (a.ngroup > 1 && 8 % a.ngroup == 0 && same_count) ? 8 / a.ngroup : 0;
  dim3 grid((unsigned)(ceil_div(tiles, 8) * 8), (unsigned)(a.ngroup > 1 ? a.ngroup : batch), 1);
  LaunchTimer timer(name, flops, bytes, stream);
  gemm_bf16_kernel<Cfg, A_K, B_K, EPI, OUT_BF16><<<grid, Cfg::kThreads, 0, stream>>>(args);
  return launch_status("gemm_bf16_kernel");
}

template <class Cfg, bool A_K, bool B_K>
int launch_layout(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s) {
  if (d.out_bf16) {
    switch (d.epi) {
      case MTF_EPI_NONE: return launch_instance<Cfg, A_K, B_K, MTF_EPI_NONE, true>(a, batch, s);
      case MTF_EPI_RELU: return launch_instance<Cfg, A_K, B_K, MTF_EPI_RELU, true>(a, batch, s);
      default: return launch_instance<Cfg, A_K, B_K, MTF_EPI_MASK_GT0, true>(a, batch, s);
    }
  }
  switch (d.epi) {
    case MTF_EPI_NONE: return launch_instance<Cfg, A_K, B_K, MTF_EPI_NONE, false>(a, batch, s);
    case MTF_EPI_RELU: return launch_instance<Cfg, A_K, B_K, MTF_EPI_RELU, false>(a, batch, s);
    default: return launch_instance<Cfg, A_K, B_K, MTF_EPI_MASK_GT0, false>(a, batch, s);
  }
}

// All instantiations of one tile shape: operand layouts x epilogues x output dtypes.
template <class Cfg>
int launch_cfg(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s) {
  if (d.a_kcontig && d.b_kcontig) return launch_layout<Cfg, true, true>(d, a, batch, s);
  if (d.a_kcontig) return launch_layout<Cfg, true, false>(d, a, batch, s);
  if (d.b_kcontig) return launch_layout<Cfg, false, true>(d, a, batch, s);
  return launch_layout<Cfg, false, false>(d, a, batch, s);
}

// The tile shapes.  Each launch_<shape> lives in gemm_bf16_<shape>.hip.
using LargeTile = TileCfg<256, 256, 2, 4, 1, 64, 4, 2>;      // 8 waves, 128 KiB LDS, one workgroup per CU
using SmallTile = TileCfg<128, 128, 2, 2, 1, 64, 8, 2>;      // 4 waves, 64 KiB LDS, two workgroups per CU
using SmallDeepTile = TileCfg<128, 128, 2, 2, 1, 64, 8, 4>;  // 128 KiB LDS: for outputs with at most one
                                                             // small tile per CU, a longer load pipeline
using SplitTile = TileCfg<256, 128, 2, 2, 2, 64, 4, 3>;      // 8 waves in two k-groups, 144 KiB LDS, one per CU

int launch_large(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s);
int launch_small(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s);
int launch_small_deep(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s);
int launch_split(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s);

}  // namespace mtf
