// bf16 x bf16 -> fp32-accumulate GEMM on the gfx950 matrix cores, with fused component-wise
// epilogues.  Every contraction of the Transformer-layer path lowers to this kernel (section
// "Performance Comparison": the einsums are where the computation time goes).
//
// Design (MI355X):
//   * large tile: one workgroup = 8 wavefronts (2 per SIMD) computes 256x256 of C, K advanced 64
//     at a time; each wave owns 128x64 as 4x2 accumulators of v_mfma_f32_32x32x16_bf16;
//     small tile (outputs with too few large tiles to fill 256 CUs): 128x128 by 4 waves of 64x64,
//     two workgroups per CU;
//   * operand tiles go global -> LDS directly (global_load_lds_dwordx4, 16 B per lane, no VGPR
//     staging), double-buffered: large 2 x (32 + 32) KiB = 128 of the CU's 160 KiB, small 64 KiB;
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
#include "gemm_bf16.h"

#include <type_traits>

#include "timing.h"

#include <cstdio>

namespace mtf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

namespace {

constexpr int BK = 64;

template <int BM_, int BN_, int WM_, int WN_, int GROUP_M_, int STAGES_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int kWaves = WM * WN, kThreads = kWaves * 64;
  static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;  // 32x32 accumulators per wave
  static constexpr int kATile = BM * BK * 2, kBTile = BN * BK * 2, kStage = kATile + kBTile;  // bytes
  static constexpr int kGroupM = GROUP_M_;  // tile rows per L2 patch
  static constexpr int kStages = STAGES_;   // k-tiles resident in LDS (one computing, the rest in flight)
  // k-steps (of 16) of fragments fetched ahead; kFragAhead + 1 must divide the steps per k-tile
  static constexpr int kFragAhead = TM * TN >= 8 ? 1 : 3;
  // register budget: two wavefronts per SIMD where the LDS lets two workgroups of 4 waves (or one
  // of 8) share a CU, else one
  static constexpr int kWavesPerSimd = (kWaves == 4 && kStages * kStage > 80 * 1024) ? 1 : 2;
};
using LargeTile = TileCfg<256, 256, 2, 4, 4, 2>;      // 128 KiB LDS, one workgroup per CU
using SmallTile = TileCfg<128, 128, 2, 2, 8, 2>;      // 64 KiB LDS, two workgroups per CU
using SmallDeepTile = TileCfg<128, 128, 2, 2, 8, 4>;  // 128 KiB LDS: for outputs with at most one
                                                      // small tile per CU, a longer load pipeline

// Slot s of A/B/K is k-segment s of one problem (ngroup == 1) or, in a grouped launch, the
// operands of problem s (then every problem has one segment and its own M, N, C and leading dims).
struct GemmArgs {
  const bf16_t* A[kMaxGroup];
  const bf16_t* B[kMaxGroup];
  int K[kMaxGroup];
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
  int batch1;
  int64_t sA0, sA1, sB0, sB1, sC0, sC1;
};

// Direct global -> LDS load of 16 bytes per lane: lane i's bytes land at lds_addr + 16*i.
// Written as inline assembly on purpose: through the compiler's builtin, every later LDS read
// is made to wait for ALL outstanding loads of this kind (it cannot tell the two stages apart
// once more than a handful of such loads exist), which would serialise load and compute.  Here
// the waits are placed by hand (tile_ready below).  m0 carries the LDS address; nothing else in
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

// One operand tile (ROWS of the M/N index x 64 of k) global -> LDS, in 1 KiB runs (one wave-wide
// load each), ROWS/8/NWAVES loads per lane.
//   k-contiguous: LDS row = one m (or n), 128 B = 8 chunks; chunk c of row r sits at c ^ ((r>>1)&7)
//   mn-contiguous: LDS row = one k, 2*ROWS B; chunk c of row k sits at c ^ ((k&3)<<2)
// TileLoader keeps, per lane, the loop-invariant byte offsets of its chunks relative to the tile's
// first element (rows / columns beyond the matrix edge are clamped to the last valid one: they
// only feed C elements that are never stored); the tile origin itself is wave-uniform.
template <bool KCONTIG, int ROWS, int NWAVES>
struct TileLoader {
  static constexpr int NL = ROWS / 8 / NWAVES;   // loads per lane per tile
  static constexpr int CPR = ROWS / 8;           // mn-contiguous: 16-byte chunks per k-row
  static constexpr int RPR = 64 / CPR;           // mn-contiguous: k-rows per run
  uint32_t off[NL];  // byte offset of this lane's chunk i from the tile origin (k0 = 0)
  int kpos[NL];      // k of the chunk (k-contiguous) or k-row (mn-contiguous), relative to k0

  __device__ __forceinline__ void init(int64_t ld, int mn0, int mn_limit, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int run = i * NWAVES + wave;
      if (KCONTIG) {
        const int r = run * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
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

// MFMA operand fragment for 32 consecutive m (or n) starting at mn_base and the 16 k of step ks:
// lane l gets index mn_base + l%32 and k = ks*16 + (l/32)*8 + 0..7.
template <bool KCONTIG, int ROWS>
__device__ __forceinline__ bf16x8 read_fragment(const char* tile, int mn_base, int ks, int lane) {
  if (KCONTIG) {
    const int r = mn_base + (lane & 31);
    const int c = ks * 2 + (lane >> 5);
    return *LDS_PTR(const bf16x8, tile + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
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
  constexpr int BM = Cfg::BM, BN = Cfg::BN, TM = Cfg::TM, TN = Cfg::TN;
  // Ring of kStages k-tiles: one being computed on, the others in flight.
  constexpr int NS = Cfg::kStages;
  __shared__ __attribute__((aligned(1024))) char ring[NS * Cfg::kStage];

  // ---- which tile: XCD-aware remap, then patches of kGroupM tile rows
  const int grp = g.ngroup > 1 ? blockIdx.y : 0;  // grouped launch: blockIdx.y picks the problem
  const int M = g.M[grp], N = g.N[grp], tiles_m = g.tiles_m[grp], tiles_n = g.tiles_n[grp];
  const int64_t lda = g.lda[grp], ldb = g.ldb[grp], ldc = g.ldc[grp];
  const int per_xcd = gridDim.x >> 3;
  const int t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
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
  const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;  // this wave's (32*TM) x (32*TN) part
  const int wave_m = wm * (32 * TM), wave_n = wn * (32 * TN);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  TileLoader<A_K, BM, Cfg::kWaves> load_a;
  TileLoader<B_K, BN, Cfg::kWaves> load_b;
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
    const int slot = min(grp + s, kMaxGroup - 1);  // grp > 0 only with nseg == 1
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
    next_a += a_tile_bytes;
    next_b += b_tile_bytes;
    next_left -= BK;
  };
  // One k-tile = BK/16 steps of 16.  LDS->register latency is several hundred cycles, more than
  // the MFMAs of one step take, so fragments are fetched kAhead steps ahead into a rotating set
  // of kAhead+1 register buffers (one LDS read slotted in front of each of the first TM+TN MFMAs
  // of a step) - and the fetch-ahead runs across k-tile boundaries: the barrier that publishes
  // tile kt+1 stands kAhead steps before the end of tile kt, right where this wave has fetched
  // the last fragment of tile kt.  The MFMAs still to do on tile kt then cover both the latency
  // of the first fragments of tile kt+1 and the issue of the loads of a further tile.
  constexpr int kAhead = Cfg::kFragAhead;
  constexpr int kSteps = BK / 16;
  static_assert(kSteps % (kAhead + 1) == 0, "fragment buffers must rotate back at a tile boundary");
  static_assert(kAhead < kSteps, "fetch-ahead of at most one k-tile");
  bf16x8 af[kAhead + 1][TM], bf[kAhead + 1][TN];
  auto fetch = [&](const char* st, int ks, bf16x8* a_dst, bf16x8* b_dst, int which) {
    // which: 0..TN-1 -> B fragment, TN..TN+TM-1 -> A fragment
    if (which < TN)
      b_dst[which] = read_fragment<B_K, BN>(st + Cfg::kATile, wave_n + which * 32, ks, lane);
    else
      a_dst[which - TN] = read_fragment<A_K, BM>(st, wave_m + (which - TN) * 32, ks, lane);
  };
  // Loads complete in issue order, so "tile kt has landed" = at most the loads of the newer tiles
  // are still outstanding.  A ragged tile may issue fewer than the usual number of loads per wave,
  // so only full newer tiles are counted (a smaller allowance only waits longer).
  constexpr int kLoadsPerTile = TileLoader<A_K, BM, Cfg::kWaves>::NL + TileLoader<B_K, BN, Cfg::kWaves>::NL;
  auto wait_for_tile = [&](int kt) {
    const int newer = min(NS - 2, total_tiles - 1 - kt);  // tiles issued after tile kt
    const int allowed = newer > 0 ? __builtin_popcount(full_hist & ((1u << newer) - 1u)) : 0;
    if (NS >= 4 && allowed >= 2)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kLoadsPerTile) : "memory");
    else if (NS >= 3 && allowed >= 1)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerTile) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
      if (HAS_NEXT && ks + kAhead == kSteps) {
        wait_for_tile(kt + 1);
        if (fill) issue_next(fill);
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
      if (allowed >= NS - 1 && NS == 2)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerTile) : "memory");
      else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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

  // ---- epilogue.  A lane holds, per accumulator, one row m and 4 x 4 consecutive n: stored
  // directly that would be 16-byte pieces scattered over 32 rows per instruction.  Instead each
  // wave passes its 32 x 64 accumulator slabs through a private LDS area (the operand ring is
  // free now) and reads them back row-wise, so every global access is 16 lanes x 16 B = one
  // contiguous 256 B row segment; aux / old-C reads of the fused epilogues get the same shape.
  static_assert(TN == 2, "epilogue staging assumes 64-column wave tiles");
  constexpr int kPitch = 64 * 4 + 16;  // fp32 row + 16 B: row-to-row bank shift of 4
  __syncthreads();                     // everyone is done reading the last k-tile
  char* slab = ring + wave * (32 * kPitch);
  const int lane_m = lane & 31, lane_h = lane >> 5;
  const int out_row = lane >> 4, out_col = (lane & 15) * 4;  // read-back: 4 rows per instruction
  void* const Cg = g.C[grp];
  // a lane reads back the same 4 columns of every slab: its bias values are loaded once
  float bias4[4] = {0.f, 0.f, 0.f, 0.f};
  if (g.bias && n0 + wave_n + out_col < N) {
    const uint2 b2 = *reinterpret_cast<const uint2*>(g.bias + n0 + wave_n + out_col);
    bias4[0] = __uint_as_float(b2.x << 16);
    bias4[1] = __uint_as_float(b2.x & 0xffff0000u);
    bias4[2] = __uint_as_float(b2.y << 16);
    bias4[3] = __uint_as_float(b2.y & 0xffff0000u);
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
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
    for (int it = 0; it < 8; ++it) {
      const int r = it * 4 + out_row;
      const f32x4 t = *LDS_PTR(const f32x4, slab + r * kPitch + out_col * 4);
      const int m = m0 + wave_m + i * 32 + r;
      const int n = n0 + wave_n + out_col;
      if (m >= M || n >= N) continue;
      const int64_t idx = offC + (int64_t)m * ldc + n;
      float v[4] = {t[0], t[1], t[2], t[3]};
      if (g.row_scale) {
        const float rs = g.row_scale[(int64_t)zb * M + m];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] *= rs;
      }
      if (g.accumulate) {
        if (OUT_BF16) {
          uint2 old = *reinterpret_cast<const uint2*>(static_cast<const bf16_t*>(Cg) + idx);
          v[0] += __uint_as_float(old.x << 16);
          v[1] += __uint_as_float(old.x & 0xffff0000u);
          v[2] += __uint_as_float(old.y << 16);
          v[3] += __uint_as_float(old.y & 0xffff0000u);
        } else {
          float4 old = *reinterpret_cast<const float4*>(static_cast<const float*>(Cg) + idx);
          v[0] += old.x;
          v[1] += old.y;
          v[2] += old.z;
          v[3] += old.w;
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += bias4[e];
      if (EPI == MTF_EPI_RELU) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
      } else if (EPI == MTF_EPI_MASK_GT0) {
        uint2 a = *reinterpret_cast<const uint2*>(g.aux + idx);
        // bf16 > 0  <=>  sign bit clear and magnitude non-zero
        const uint32_t w[4] = {a.x & 0xffffu, a.x >> 16, a.y & 0xffffu, a.y >> 16};
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (w[e] != 0u && w[e] < 0x8000u) ? v[e] : 0.f;
      }
      if (OUT_BF16)
        *reinterpret_cast<uint2*>(static_cast<bf16_t*>(Cg) + idx) =
            make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
      else
        *reinterpret_cast<float4*>(static_cast<float*>(Cg) + idx) = make_float4(v[0], v[1], v[2], v[3]);
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
      std::snprintf(text, sizeof text, "gemm_bf16_kernel<TileCfg<%d, %d, %d, %d, %d, %d>, %s, %s, %d, %s>", Cfg::BM,
                    Cfg::BN, Cfg::WM, Cfg::WN, Cfg::kGroupM, Cfg::kStages, A_K ? "true" : "false",
                    B_K ? "true" : "false", EPI, OUT_BF16 ? "true" : "false");
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
    if (a.ngroup > 1) ktot = a.K[p];
    else for (int s = 0; s < a.nseg; ++s) ktot += a.K[s];
    flops += 2.0 * a.M[p] * a.N[p] * ktot * batch;
    bytes += batch * (2.0 * ktot * (a.M[p] + a.N[p]) + (double)a.M[p] * a.N[p] * (OUT_BF16 ? 2 : 4));
  }
  if (tiles > (1 << 28)) return fail(MTF_ERR_UNSUPPORTED, "too many tiles");
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

template <class Cfg>
int launch_cfg(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s) {
  if (d.a_kcontig && d.b_kcontig) return launch_layout<Cfg, true, true>(d, a, batch, s);
  if (d.a_kcontig) return launch_layout<Cfg, true, false>(d, a, batch, s);
  if (d.b_kcontig) return launch_layout<Cfg, false, true>(d, a, batch, s);
  return launch_layout<Cfg, false, false>(d, a, batch, s);
}

}  // namespace

// The tile loaders keep per-lane byte offsets relative to the tile origin in 32 bits: up to
// (tile rows - 1) * ld * 2 + 128 for a k-contiguous operand (256-row tile) and 63 * ld * 2 +
// 2 * tile columns for an mn-contiguous one.  Leading dims beyond this would wrap.
static bool ld_fits_32bit_offsets(int64_t ld, bool kcontig) {
  const int64_t worst = kcontig ? 255 * ld * 2 + 128 : 63 * ld * 2 + 512;
  return ld >= 0 && ld < (INT64_C(1) << 40) && worst <= (int64_t)UINT32_MAX;
}

bool gemm_bf16_supported(const GemmDesc& d) {
  if (d.nseg < 1 || d.nseg > kMaxSegments) return false;
  if (!ld_fits_32bit_offsets(d.lda, d.a_kcontig) || !ld_fits_32bit_offsets(d.ldb, d.b_kcontig)) return false;
  for (int p = 0; p < d.nextra && p < kMaxGroup - 1; ++p)
    if (!ld_fits_32bit_offsets(d.extra[p].lda, d.a_kcontig) || !ld_fits_32bit_offsets(d.extra[p].ldb, d.b_kcontig))
      return false;
  if (d.M <= 0 || d.N <= 0 || d.M > INT32_MAX || d.N > INT32_MAX) return false;
  if (d.lda % 8 || d.ldb % 8 || d.ldc % 4 || d.N % 8) return false;
  if (!d.a_kcontig && d.M % 8) return false;
  if (d.sA0 % 8 || d.sA1 % 8 || d.sB0 % 8 || d.sB1 % 8 || d.sC0 % 4 || d.sC1 % 4) return false;
  for (int s = 0; s < d.nseg; ++s) {
    if (d.K[s] < 0 || d.K[s] > INT32_MAX) return false;
    if ((d.a_kcontig || d.b_kcontig) && d.K[s] % 8) return false;
    if (!aligned16(d.A[s]) || !aligned16(d.B[s])) return false;
  }
  if (!aligned16(d.C) || (d.epi == MTF_EPI_MASK_GT0 && (!d.aux || !aligned16(d.aux)))) return false;
  if (d.bias && (((uintptr_t)d.bias & 7) || d.nextra > 0)) return false;
  if (d.row_scale && d.nextra > 0) return false;
  if (d.batch0 * d.batch1 > 65535) return false;
  if (d.nextra < 0 || d.nextra > kMaxGroup - 1) return false;
  if (d.nextra > 0 && (d.nseg != 1 || d.batch0 * d.batch1 != 1 || d.accumulate || d.epi != MTF_EPI_NONE))
    return false;
  for (int p = 0; p < d.nextra; ++p) {
    const GemmDesc::Extra& e = d.extra[p];
    if (e.M <= 0 || e.N <= 0 || e.K < 0 || e.M > INT32_MAX || e.N > INT32_MAX || e.K > INT32_MAX) return false;
    if (e.lda % 8 || e.ldb % 8 || e.ldc % 4 || e.N % 8 || (!d.a_kcontig && e.M % 8)) return false;
    if ((d.a_kcontig || d.b_kcontig) && e.K % 8) return false;
    if (!e.A || !e.B || !e.C || !aligned16(e.A) || !aligned16(e.B) || !aligned16(e.C)) return false;
  }
  return true;
}

int gemm_bf16_launch(const GemmDesc& d, hipStream_t stream) {
  if (!gemm_bf16_supported(d)) return fail(MTF_ERR_UNSUPPORTED, "GEMM shape/alignment");
  GemmArgs a;
  for (int s = 0; s < kMaxGroup; ++s) {
    a.A[s] = s < d.nseg ? d.A[s] : d.A[0];
    a.B[s] = s < d.nseg ? d.B[s] : d.B[0];
    a.K[s] = s < d.nseg ? (int)d.K[s] : 0;
    a.M[s] = (int)d.M;
    a.N[s] = (int)d.N;
    a.lda[s] = d.lda;
    a.ldb[s] = d.ldb;
    a.ldc[s] = d.ldc;
    a.C[s] = d.C;
    a.tiles_m[s] = a.tiles_n[s] = 0;
  }
  a.nseg = d.nseg;
  a.ngroup = 1 + d.nextra;
  for (int p = 0; p < d.nextra; ++p) {
    const GemmDesc::Extra& e = d.extra[p];
    a.A[p + 1] = e.A; a.B[p + 1] = e.B; a.C[p + 1] = e.C;
    a.M[p + 1] = (int)e.M; a.N[p + 1] = (int)e.N; a.K[p + 1] = (int)e.K;
    a.lda[p + 1] = e.lda; a.ldb[p + 1] = e.ldb; a.ldc[p + 1] = e.ldc;
  }
  a.aux = d.aux;
  a.bias = d.bias;
  a.row_scale = d.row_scale;
  a.alpha = d.alpha;
  a.accumulate = d.accumulate ? 1 : 0;
  a.batch1 = (int)d.batch1;
  a.sA0 = d.sA0; a.sA1 = d.sA1; a.sB0 = d.sB0; a.sB1 = d.sB1; a.sC0 = d.sC0; a.sC1 = d.sC1;
  const int batch = (int)(d.batch0 * d.batch1);
  // Tile choice: the large tile moves half the bytes per flop, but needs enough tiles to occupy
  // the 256 CUs; below that the small tile (4x the tiles, two workgroups per CU) wins.
  int64_t large_tiles = ceil_div(d.M, LargeTile::BM) * ceil_div(d.N, LargeTile::BN) * batch;
  for (int p = 0; p < d.nextra; ++p)
    large_tiles += ceil_div(d.extra[p].M, LargeTile::BM) * ceil_div(d.extra[p].N, LargeTile::BN);
  int64_t small_tiles = ceil_div(d.M, SmallTile::BM) * ceil_div(d.N, SmallTile::BN) * batch;
  for (int p = 0; p < d.nextra; ++p)
    small_tiles += ceil_div(d.extra[p].M, SmallTile::BM) * ceil_div(d.extra[p].N, SmallTile::BN);
  // rounds of tiles over 256 CUs (large: one workgroup per CU, 4 work units each; small: two
  // per CU, 1 unit each, at ~0.8 of the large tile's rate)
  const double cost_large = (double)ceil_div(large_tiles, 256) * 4.0;
  const double cost_small = (double)ceil_div(small_tiles, 512) * 2.0 / 0.8;
  int tile = d.tile;
  if (tile == 0) tile = cost_large <= cost_small ? 2 : (small_tiles <= 256 ? 3 : 1);
  if (tile == 2) return launch_cfg<LargeTile>(d, a, batch, stream);
  if (tile == 3) return launch_cfg<SmallDeepTile>(d, a, batch, stream);
  return launch_cfg<SmallTile>(d, a, batch, stream);
}

}  // namespace mtf
