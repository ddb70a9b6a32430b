// Fused softmax attention for one processor's heads: the two attention einsums
//   logits[b,h,l,m] = einsum(q[b,l,h,k], k_[b,m,h,k])      ctx[b,l,h,v] = einsum(p[b,h,l,m], v_[b,m,h,v])
// with the row softmax between them, forward and backward, without materialising [l,m] tensors.
// The memory_length dim is never split (softmax needs the whole row locally), heads are.
//
// All matrix products run on v_mfma_f32_32x32x16_bf16.  Orientation trick used throughout: the
// first product is computed TRANSPOSED relative to the second one's needs, so that the fp32
// accumulator a lane holds (one column, 16 rows in the order (j/4)*8 + (lane/32)*4 + j%4) can be
// packed to bf16 and fed straight back as the next MFMA's B operand; the other operand of that
// second product is read with the LDS transpose load using the same row order.  No shuffles, no
// round trip through LDS for the probabilities.
//
// The kernels are templates on the head width HD = d_k = d_v: 128 (the translation models of the
// paper's experiments) and 256 (its language models).  LDS tiles are 64 rows x HD (2*HD bytes per
// row), filled by direct global->LDS loads.  One XOR swizzle of the 16-byte chunk index serves both
// access patterns (row-wise ds_read_b128 and transposed ds_read_b64_tr_b16).
//
// Work decomposition: a wave owns 32 query rows (forward, dq) or 32 memory rows (dk/dv) and keeps
// their operand fragments in registers for the whole kernel; those fragments arrive, and the
// results leave, through wave-private LDS slabs so that global memory sees whole 256-byte rows.
// Under the causal mask an 8-wave workgroup pairs a late with an early block of query rows, and
// grids put heads fastest, so that every SIMD and every XCD gets the same amount of work.
// The softmax keeps the vector ALU work per logit at one fma, one exp2 and one add (scale folded
// into the fma, running maximum raised lazily, masking only on ragged / diagonal tiles).
#include "attention.h"

#include "timing.h"

namespace mtf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

namespace {

constexpr int kTileRows = 64;
// Sizes that follow from the head width.
template <int HD>
struct Geo {
  static_assert(HD == 128 || HD == 256, "head width 128 or 256");
  static constexpr int kRowBytes = HD * 2;
  static constexpr int kTileBytes = kTileRows * kRowBytes;  // 16 / 32 KiB
  static constexpr int kSlabBytes = 32 * kRowBytes;         // 8 / 16 KiB
  static constexpr int kKS = HD / 16;                       // k-steps of 16 over d
  static constexpr int kBlk = HD / 32;                      // 32-column blocks over d
  static constexpr int kCPR = HD / 8;                       // 16-byte chunks per row
  static constexpr int kRPR = 64 / kCPR;                    // rows per 1 KiB run (one wave-wide load)
  static constexpr int kTileRuns = kTileBytes / 1024;
  static constexpr int kSlabRuns = kSlabBytes / 1024;
};
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
  const bf16_t *q, *k, *v, *ctx, *dctx;
  bf16_t *out0, *out1;  // fwd: ctx | dq kernel: dq | dkv kernel: dk, dv
  const float *lse_in, *delta_in;
  float *lse_out, *delta_out;
  int batch, length, heads;
  float scale;
  int causal;
};

__device__ __forceinline__ uint32_t lds_address(const char* p) {
  return (uint32_t)(uintptr_t)LDS_PTR(const char, p);
}

// 16 bytes per lane, global -> LDS, lane i to lds_addr + 16*i (inline asm: the waits are placed
// by hand; m0 carries the LDS address and is used by nothing else here).
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

__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ void wait_loads_then_barrier() {
  wait_loads();
  __syncthreads();
}

// The compiler's bookkeeping of outstanding loads does not see the asm tile loads.  A value it
// loaded itself and first uses inside the tile loop would get its s_waitcnt vmcnt(n) there, on
// every trip, and that wait also drains the asynchronous loads of the next tile - the whole
// load latency lands in every step.  Naming the value here makes it settle the load before the
// loop instead.
template <class T>
__device__ __forceinline__ void settle(T& v) {
  asm volatile("" : "+v"(v));
}

// chunk c of row r is stored at chunk c ^ swz(r): a bijection over any 16 consecutive rows (row
// reads of 16 lanes hit 16 different chunks) whose upper two bits differ over any aligned group
// of 4 rows (transpose reads of 4 rows hit 4 different 64-byte bank groups).
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// Tile <- rows row0 .. row0+ROWS-1 (clamped to row_limit-1) of head h of a [*, rows, heads, HD] tensor.
// base: address of element (b, 0, h, 0).
template <int HD, int NWAVES, int ROWS = kTileRows>
__device__ __forceinline__ void load_tile(const bf16_t* base, uint32_t row_stride_bytes, int row0,
                                          int row_limit, char* tile, int wave, int lane) {
  using G = Geo<HD>;
  static_assert((ROWS * G::kRowBytes / 1024) % NWAVES == 0, "whole runs per wave");
#pragma unroll
  for (int i = 0; i < ROWS * G::kRowBytes / 1024 / NWAVES; ++i) {
    const int run = i * NWAVES + wave;
    const int row = run * G::kRPR + lane / G::kCPR;
    const int c = (lane % G::kCPR) ^ swz(row);
    const int src = min(row0 + row, row_limit - 1);
    load16_to_lds(reinterpret_cast<const char*>(base), (uint32_t)src * row_stride_bytes + c * 16,
                  lds_address(tile) + run * 1024);
  }
}

// Operand fragment with the tile's rows as the MFMA's outer (M or N) index and d as k:
// lane l -> row row_base + l%32, d = ks*16 + (l/32)*8 + 0..7.
template <int HD>
__device__ __forceinline__ bf16x8 rows_frag(const char* tile, int row_base, int ks, int lane) {
  const int r = row_base + (lane & 31);
  const int c = ks * 2 + (lane >> 5);
  return *LDS_PTR(const bf16x8, tile + r * Geo<HD>::kRowBytes + ((c ^ swz(r)) << 4));
}

// Operand fragment with d as the MFMA's outer index (32 columns from d_base) and the tile's rows
// as k, in accumulator row order: k-slot e of lane-half hf is row row_base + (e/4)*8 + hf*4 + e%4.
template <int HD>
__device__ __forceinline__ bf16x8 cols_frag(const char* tile, int d_base, int row_base, int lane) {
  const int g = lane >> 4, j = lane & 15;
  const int d = d_base + (g & 1) * 16 + (j & 3) * 4;
  const int row = row_base + (g >> 1) * 4 + (j >> 2);
  union {
    s16x4 h[2];
    bf16x8 v;
  } u;
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2) {
    const int r = row + h2 * 8;
    const char* p = tile + r * Geo<HD>::kRowBytes + (((d >> 3) ^ swz(r)) << 4) + (d & 7) * 2;
    u.h[h2] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p));
  }
  return u.v;
}

// Same row-operand fragment straight from global memory (kept in registers for the whole kernel).
__device__ __forceinline__ bf16x8 global_rows_frag(const bf16_t* base, int64_t row_stride, int row,
                                                   int ks, int lane) {
  return *reinterpret_cast<const bf16x8*>(base + (int64_t)row * row_stride + ks * 16 + (lane >> 5) * 8);
}

__device__ __forceinline__ bf16x8 pack8(const float* v) {
  union {
    uint32_t w[4];
    bf16x8 v;
  } u;
#pragma unroll
  for (int i = 0; i < 4; ++i) u.w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
  return u.v;
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

// Row of an accumulator value: value jj of a lane in half hf sits at row (jj/4)*8 + hf*4 + jj%4.
__device__ __forceinline__ int acc_row(int jj, int hf) { return (jj >> 2) * 8 + hf * 4 + (jj & 3); }

// A slab = 32 rows of 2*HD bytes private to one wave, same chunk swizzle as a tile.  The fragments a
// wave keeps in registers for the whole kernel, and the rows it stores at the end, pass through
// it so that global memory sees whole 256-byte rows (a fragment taken straight from global
// memory is 32-byte pieces of 32 different rows per instruction).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// slab <- rows row0 .. row0+31 (clamped to row_limit-1); asynchronous, completes with the wave's
// other tile loads (s_waitcnt vmcnt).
template <int HD>
__device__ __forceinline__ void load_slab(const bf16_t* base, uint32_t row_stride_bytes, int row0,
                                          int row_limit, char* slab, int lane) {
  using G = Geo<HD>;
#pragma unroll
  for (int run = 0; run < G::kSlabRuns; ++run) {
    const int row = run * G::kRPR + lane / G::kCPR;
    const int c = (lane % G::kCPR) ^ swz(row);
    const int src = min(row0 + row, row_limit - 1);
    load16_to_lds(reinterpret_cast<const char*>(base), (uint32_t)src * row_stride_bytes + c * 16,
                  lds_address(slab) + run * 1024);
  }
}

// Stores a [32 x HD]^T accumulator set (lane = one row of the output, 4 consecutive d per group)
// as bf16 rows row0 .. row0+31 (those below row_limit) of a [*, rows, heads, HD] tensor.  Only
// this wave touches `slab`.
template <int HD>
__device__ __forceinline__ void store_rows_bf16(bf16_t* base, int64_t row_stride, int row0,
                                                int row_limit, const f32x16* acc, float mul,
                                                char* slab, int lane) {
  // keeps the compiler from preparing the addresses of these stores before the tile loop and
  // carrying them through it in registers it does not have
  asm volatile("" : "+v"(lane));
  using G = Geo<HD>;
  const int hf = lane >> 5, r = lane & 31;
#pragma unroll
  for (int blk = 0; blk < G::kBlk; ++blk)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int d = blk * 32 + q4 * 8 + hf * 4;
      u32x2 w;
      w[0] = pack_bf16x2(acc[blk][q4 * 4 + 0] * mul, acc[blk][q4 * 4 + 1] * mul);
      w[1] = pack_bf16x2(acc[blk][q4 * 4 + 2] * mul, acc[blk][q4 * 4 + 3] * mul);
      *LDS_PTR(u32x2, slab + r * G::kRowBytes + (((d >> 3) ^ swz(r)) << 4) + (d & 7) * 2) = w;
    }
  __builtin_amdgcn_wave_barrier();  // LDS operations of a wave complete in order
#pragma unroll
  for (int run = 0; run < G::kSlabRuns; ++run) {
    const int row = run * G::kRPR + lane / G::kCPR, c = lane % G::kCPR;
    const u32x4 v = *LDS_PTR(const u32x4, slab + row * G::kRowBytes + ((c ^ swz(row)) << 4));
    if (row0 + row < row_limit)
      *reinterpret_cast<u32x4*>(base + (int64_t)(row0 + row) * row_stride + c * 8) = v;
  }
}

// Query rows of a workgroup.  With 8 waves the workgroup takes two blocks of 128 query rows, one
// from each end of the sequence (waves 0-3 the later block, waves 4-7 the earlier one): under the
// causal mask a late block sees many memory tiles and an early one few, and a wave of each kind
// lands on every SIMD (wave w runs on SIMD w % 4), so all SIMDs of all CUs get the same work.
// Smaller workgroups take NWAVES*32 consecutive rows, later blocks first.
struct QueryRows {
  int wave_row0;  // first query row of this wave
  int last_row;   // last query row of the workgroup (bounds the memory tiles a causal pass needs)
  bool active;    // false: this wave has no rows (odd number of blocks, middle block)
};
template <int NWAVES>
__device__ __forceinline__ QueryRows query_rows(int length, bool causal, int wave) {
  QueryRows r;
  if (NWAVES == 8) {
    const int nblk = (length + 127) / 128;
    const int late = nblk - 1 - (int)blockIdx.z, early = (int)blockIdx.z;
    r.wave_row0 = (wave < 4 ? late : early) * 128 + (wave & 3) * 32;
    r.last_row = late * 128 + 127;
    r.active = wave < 4 || early != late;
  } else {
    const int q0 = (causal ? gridDim.z - 1 - blockIdx.z : blockIdx.z) * (NWAVES * 32);
    r.wave_row0 = q0 + wave * 32;
    r.last_row = q0 + NWAVES * 32 - 1;
    r.active = true;
  }
  return r;
}

// ------------------------------------------------------------------------------------ forward
// Shape of the forward / dq kernels at a head width.  At 128 a wave keeps its row-operand
// fragments (q; q and dctx) in registers for the whole kernel, K/V tiles have 64 rows, and two
// wavefronts share a SIMD.  At 256 those fragments alone would fill the vector registers a wave
// can address, so one of them stays in the wave's LDS slab and is fetched like the tile operands,
// the K/V tiles shrink to 32 rows (the slabs need the LDS), and one wavefront has the SIMD.
template <int HD, int NWAVES, bool ROWS_IN_LDS>
struct RowKernelShape {
  static constexpr bool kRowsInLds = ROWS_IN_LDS;
  static constexpr int kTR = HD == 256 ? 32 : kTileRows;  // rows of a K/V tile
  static constexpr int kWavesPerSimd = (HD == 128 && NWAVES >= 4) ? 2 : 1;
  // Slabs get LDS of their own when they stay in use (rows in LDS) or when, with 8 waves, they
  // need as much as both stages; otherwise they borrow stage 1, which the pipeline first writes at
  // the barrier of step 0 and last reads before the barrier that precedes the final stores.
  static constexpr bool kOwnSlabs = kRowsInLds || NWAVES == 8;
  static constexpr int kTileBytes = kTR * Geo<HD>::kRowBytes;
  static constexpr int kTileLoads = 2 * (kTileBytes / 1024 / NWAVES);  // loads per wave of one K + V tile
  static_assert(kOwnSlabs || NWAVES * Geo<HD>::kSlabBytes <= 2 * kTileBytes, "borrowed slabs fit stage 1");
  static constexpr int kLdsBytes = 4 * kTileBytes + (kOwnSlabs ? NWAVES * Geo<HD>::kSlabBytes : 0);
};

// Flips the sign of every element of a slab's rows in place (each lane its own fragments).
template <int HD>
__device__ __forceinline__ void negate_slab(char* slab, int lane) {
  const int r = lane & 31;
#pragma unroll
  for (int ks = 0; ks < Geo<HD>::kKS; ++ks) {
    const int c = ks * 2 + (lane >> 5);
    char* p = slab + r * Geo<HD>::kRowBytes + ((c ^ swz(r)) << 4);
    u32x4 v = *LDS_PTR(u32x4, p);
    v ^= u32x4{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
    *LDS_PTR(u32x4, p) = v;
  }
}

// One workgroup: NWAVES*32 query rows of one (batch, head); each wave owns 32 of them.
template <int HD, int NWAVES>
__global__ void __launch_bounds__(NWAVES * 64, (RowKernelShape<HD, NWAVES, false>::kWavesPerSimd)) attn_fwd_kernel(AttnArgs a) {
  using G = Geo<HD>;
  using S = RowKernelShape<HD, NWAVES, false>;
  __shared__ __attribute__((aligned(1024))) char lds[S::kLdsBytes];
  constexpr int kTR = S::kTR, kTileBytes = S::kTileBytes, kSlabBytes = G::kSlabBytes, kKS = G::kKS, kBlk = G::kBlk;
  constexpr bool kQInLds = S::kRowsInLds;
  char* const stage0 = lds;                     // K tile, V tile
  char* const stage1 = lds + 2 * kTileBytes;
  char* const slabs = lds + 4 * kTileBytes;     // only with kOwnSlabs
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* slab = (S::kOwnSlabs ? slabs : stage1) + wave * kSlabBytes;
  const int L = a.length, H = a.heads;
  const int b = blockIdx.y, h = blockIdx.x;
  const QueryRows qr = query_rows<NWAVES>(L, a.causal, wave);
  const int q0w = qr.wave_row0;
  const int64_t rs = (int64_t)H * HD;
  const int64_t head0 = ((int64_t)b * L) * rs + (int64_t)h * HD;
  const bf16_t *qb = a.q + head0, *kb = a.k + head0, *vb = a.v + head0;

  const int q_lane = q0w + (lane & 31);  // this lane's query row
  const int kv_end = a.causal ? min(L, qr.last_row + 1) : L;
  const int n_tiles = (kv_end + kTR - 1) / kTR;
  // Tiles this wave takes part in: under the causal mask its rows see nothing past their own
  // position.  The rest of the workgroup's tiles it only helps to load, in a loop of their own: a
  // bypass inside the processing loop would make the compiler carry the accumulators through
  // copies around every tile.
  const int my_tiles = !qr.active ? 0 : a.causal ? min(n_tiles, (q0w + 31) / kTR + 1) : n_tiles;
  auto issue = [&](int t, char* st) {
    load_tile<HD, NWAVES, kTR>(kb, (uint32_t)(rs * 2), t * kTR, L, st, wave, lane);
    load_tile<HD, NWAVES, kTR>(vb, (uint32_t)(rs * 2), t * kTR, L, st + kTileBytes, wave, lane);
  };
  // this wave's query rows and the first K/V tile travel together
  load_slab<HD>(qb, (uint32_t)(rs * 2), q0w, L, slab, lane);
  issue(0, stage0);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(S::kTileLoads) : "memory");  // the slab has landed
  // The running maximum works on s * c with c >= 0.  A negative scale is moved into q (sign
  // bits flipped: logits come out negated); a zero scale becomes a tiny positive one (logits
  // of order 1e-30 instead of 0), which keeps -inf * c = -inf for hidden positions.
  bf16x8 qf[kQInLds ? 1 : kKS];
  if (kQInLds) {
    if (a.scale < 0.f) negate_slab<HD>(slab, lane);
  } else {
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) qf[ks] = rows_frag<HD>(slab, 0, ks, lane);
    if (a.scale < 0.f) {
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) {
        union {
          bf16x8 v;
          uint32_t w[4];
        } u;
        u.v = qf[ks];
#pragma unroll
        for (int i = 0; i < 4; ++i) u.w[i] ^= 0x80008000u;
        qf[ks] = u.v;
      }
    }
  }

  f32x16 o[kBlk];
#pragma unroll
  for (int i = 0; i < kBlk; ++i) o[i] = zero16();
  float m2 = -INFINITY, lsum = 0.f;  // running max (log2 units) and row sum
  const float c2 = fmaxf(fabsf(a.scale) * kLog2e, 1e-30f);

  auto process = [&](int t, const char* st) {
    const int kv0 = t * kTR;
    const char *kt_ = st, *vt_ = st + kTileBytes;
    // Operand fragments are fetched from LDS kDepth MFMAs ahead of their use, through rings of
    // kDepth + 1 register buffers, and a scheduling barrier after each MFMA keeps that order: left
    // alone, the scheduler either sinks each read to just before its MFMA (which then waits out a
    // full LDS round trip; for most of a causal pass a wave has no partner on its SIMD to cover
    // it) or, with registers to spare, hoists them all and spills.  Consecutive MFMAs go to
    // different accumulators where there are several.
    constexpr int kDepth = 2, kRing = kDepth + 1;
    constexpr int kKvb = kTR / 32;            // 32-row blocks of the tile
    constexpr int kT = kTR / 16;              // 16-row k-steps of the second product
    constexpr int kItems1 = kKvb * kKS;       // first product, item n = ks*kKvb + kvb: K rows kvb*32.., k-step ks
    constexpr int kItems2 = kT * kBlk;        // second product, item n = t*kBlk + blk: V columns blk*32.., rows t*16..
    bf16x8 fk[kRing], fq[kQInLds ? kRing : 1], fv[kRing];
    auto fetch_k = [&](int n) {
      fk[n % kRing] = rows_frag<HD>(kt_, (n % kKvb) * 32, n / kKvb, lane);
      if (kQInLds) fq[n % kRing] = rows_frag<HD>(slab, 0, n / kKvb, lane);
    };
    auto fetch_v = [&](int n) { fv[n % kRing] = cols_frag<HD>(vt_, (n % kBlk) * 32, (n / kBlk) * 16, lane); };
#pragma unroll
    for (int n = 0; n < kDepth; ++n) fetch_k(n);
    // logits^T: rows = memory positions of the tile, column = this lane's query
    f32x16 s[kKvb];
#pragma unroll
    for (int kvb = 0; kvb < kKvb; ++kvb) s[kvb] = zero16();
#pragma unroll
    for (int n = 0; n < kItems1; ++n) {
      if (n + kDepth < kItems1)
        fetch_k(n + kDepth);
      else
        fetch_v(n + kDepth - kItems1);  // the last steps already bring in the second product's operands
      s[n % kKvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[n % kRing], kQInLds ? fq[n % kRing] : qf[n / kKvb],
                                                            s[n % kKvb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // Softmax bookkeeping, kept cheap on the vector ALU (it competes with the matrix cores):
    //  * masking only on tiles that can contain a hidden position for this wave (wave-uniform);
    //  * the scale is folded into one fma per logit: p = exp2(s * c2 - m);
    //  * the running maximum m2 is only raised (and O, lsum rescaled) when some row's maximum
    //    exceeds it by more than kSlack: until then p <= 2^kSlack, harmless in fp32 / bf16.
    const bool need_mask = kv0 + kTR > L || (a.causal && kv0 + kTR - 1 > q0w);
    if (need_mask) {
#pragma unroll
      for (int kvb = 0; kvb < kKvb; ++kvb)
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
          const int kv = kv0 + kvb * 32 + acc_row(jj, hf);
          const bool vis = kv < L && (!a.causal || kv <= q_lane);
          s[kvb][jj] = vis ? s[kvb][jj] : -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kvb = 0; kvb < kKvb; ++kvb)
#pragma unroll
      for (int jj = 0; jj < 16; ++jj) mx = fmaxf(mx, s[kvb][jj]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));  // the other half-wave holds the rest of this query's row
    mx *= c2;  // c2 > 0, so a fully hidden row stays at -inf
    constexpr float kSlack = 8.f;
    if (__builtin_expect(__any(mx > m2 + kSlack), 0)) {  // first tile: m2 = -inf, always taken; position 0 is visible
      const float m_new = fmaxf(m2, mx);
      const float alpha = __builtin_amdgcn_exp2f(m2 - m_new);
      lsum *= alpha;
      m2 = m_new;
      if (HD == 256) {
        // One wavefront per SIMD: the accumulators live in the accumulation registers, which the
        // vector ALU cannot multiply in place.  Written as plain C++ the compiler carries them
        // through ordinary registers around every tile's matrix instructions for the sake of this
        // rare block; here each element makes the round trip inside the block instead.  The s_nops
        // cover the matrix-core-to-ALU and ALU-to-matrix-core register hazards, which the compiler
        // cannot see through the asm (the logits products already separate the two by far more).
        asm volatile("s_nop 15\n\ts_nop 15");
#pragma unroll
        for (int blk = 0; blk < kBlk; ++blk)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float acc = o[blk][e], tmp;
            asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\ts_nop 0\n\tv_accvgpr_write_b32 %0, %1"
                         : "+a"(acc), "=&v"(tmp)
                         : "v"(alpha));
            o[blk][e] = acc;
          }
        asm volatile("s_nop 7");
      } else {
#pragma unroll
        for (int blk = 0; blk < kBlk; ++blk)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[blk][e] *= alpha;
      }
    }
    float psum = 0.f;
    bf16x8 pf[kT];
#pragma unroll
    for (int kvb = 0; kvb < kKvb; ++kvb) {
      float p[16];
#pragma unroll
      for (int jj = 0; jj < 16; ++jj) {
        p[jj] = __builtin_amdgcn_exp2f(fmaf(s[kvb][jj], c2, -m2));  // hidden: exp2(-inf) = 0
        psum += p[jj];
      }
      pf[kvb * 2 + 0] = pack8(p);
      pf[kvb * 2 + 1] = pack8(p + 8);
    }
    psum += __shfl_xor(psum, 32);
    lsum += psum;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int n = 0; n < kItems2; ++n) {
      if (n + kDepth < kItems2) fetch_v(n + kDepth);
      o[n % kBlk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[n % kRing], pf[n / kBlk], o[n % kBlk], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Two stages: the tile after the one being processed is in flight.  Passing the barrier means
  // everyone has the current tile and is done with the stage the next issue() overwrites.
  for (int t = 0; t < my_tiles; ++t) {
    char* cur = (t & 1) ? stage1 : stage0;
    char* nxt = (t & 1) ? stage0 : stage1;
    wait_loads_then_barrier();
    if (t + 1 < n_tiles) issue(t + 1, nxt);
    process(t, cur);
  }
  for (int t = my_tiles; t < n_tiles; ++t) {  // tiles only later waves of the workgroup can see
    wait_loads_then_barrier();
    if (t + 1 < n_tiles) issue(t + 1, (t & 1) ? stage0 : stage1);
  }
  if (!S::kOwnSlabs) __syncthreads();  // stage 1 may still be read by a slower wave
  if (!qr.active) return;
  store_rows_bf16<HD>(a.out0 + head0, rs, q0w, L, o, 1.f / lsum, slab, lane);
  if (q_lane < L && hf == 0)
    a.lse_out[((int64_t)b * H + h) * L + q_lane] = (m2 + __log2f(lsum)) * kLn2;
}

// ------------------------------------------------------------------------------------ backward
// dq: one workgroup per NWAVES*32 query rows; loops over memory tiles.  Also produces
// delta[b,h,l] = sum_d dctx[b,l,h,d] * ctx[b,l,h,d] (= sum_m p * dp of the softmax Jacobian) for
// its rows, which the dk/dv kernel launched after it reads.
template <int HD, int NWAVES>
__global__ void __launch_bounds__(NWAVES * 64, (RowKernelShape<HD, NWAVES, HD == 256>::kWavesPerSimd)) attn_dq_kernel(AttnArgs a) {
  using G = Geo<HD>;
  using S = RowKernelShape<HD, NWAVES, HD == 256>;
  constexpr int kTR = S::kTR, kTileBytes = S::kTileBytes, kSlabBytes = G::kSlabBytes, kKS = G::kKS, kBlk = G::kBlk;
  constexpr bool kDoInLds = S::kRowsInLds;  // the dctx rows stay in the slab (q is kept in registers)
  __shared__ __attribute__((aligned(1024))) char stage0[2 * kTileBytes];  // K tile, V tile
  __shared__ __attribute__((aligned(1024))) char stage1[2 * kTileBytes];
  __shared__ __attribute__((aligned(1024))) char slabs[S::kOwnSlabs ? NWAVES * kSlabBytes : 16];
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* slab = (S::kOwnSlabs ? slabs : stage1) + wave * kSlabBytes;
  const int L = a.length, H = a.heads;
  const int b = blockIdx.y, h = blockIdx.x;
  const QueryRows qr = query_rows<NWAVES>(L, a.causal, wave);
  const int q0w = qr.wave_row0;
  const int64_t rs = (int64_t)H * HD;
  const int64_t head0 = ((int64_t)b * L) * rs + (int64_t)h * HD;
  const bf16_t *qb = a.q + head0, *kb = a.k + head0, *vb = a.v + head0, *dob = a.dctx + head0;

  const int q_lane = q0w + (lane & 31);
  const int q_load = min(q_lane, L - 1);
  const int kv_end = a.causal ? min(L, qr.last_row + 1) : L;
  const int n_tiles = (kv_end + kTR - 1) / kTR;
  // Tiles this wave takes part in: under the causal mask its rows see nothing past their own
  // position.  The rest of the workgroup's tiles it only helps to load, in a loop of their own: a
  // bypass inside the processing loop would make the compiler carry the accumulators through
  // copies around every tile.
  const int my_tiles = !qr.active ? 0 : a.causal ? min(n_tiles, (q0w + 31) / kTR + 1) : n_tiles;
  auto issue = [&](int t, char* st) {
    load_tile<HD, NWAVES, kTR>(kb, (uint32_t)(rs * 2), t * kTR, L, st, wave, lane);
    load_tile<HD, NWAVES, kTR>(vb, (uint32_t)(rs * 2), t * kTR, L, st + kTileBytes, wave, lane);
  };
  const int64_t stat = ((int64_t)b * H + h) * L + q_load;
  float lse2 = a.lse_in[stat] * kLog2e;
  settle(lse2);  // before any asynchronous load is in flight
  // This wave's rows of q and of dctx pass through its slab, one after the other; the operand
  // that is kept in registers goes first, the one that stays in the slab (width 256: dctx) last.
  // The ctx rows (used once, for delta) come straight from global memory alongside the first slab
  // and the first K/V tile.
  bf16x8 qf[kKS], dof[kDoInLds ? 1 : kKS], of[kKS];
#pragma unroll
  for (int ks = 0; ks < kKS; ++ks) of[ks] = global_rows_frag(a.ctx + head0, rs, q_load, ks, lane);
  load_slab<HD>(kDoInLds ? qb : dob, (uint32_t)(rs * 2), q0w, L, slab, lane);
  issue(0, stage0);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(S::kTileLoads) : "memory");  // ctx rows and slab have landed
#pragma unroll
  for (int ks = 0; ks < kKS; ++ks) {
    settle(of[ks]);
    if (kDoInLds)
      qf[ks] = rows_frag<HD>(slab, 0, ks, lane);
    else
      dof[ks] = rows_frag<HD>(slab, 0, ks, lane);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // fragments read before the slab is overwritten
  load_slab<HD>(kDoInLds ? dob : qb, (uint32_t)(rs * 2), q0w, L, slab, lane);
  if (kDoInLds) wait_loads();  // delta needs the dctx rows now
  // delta: this lane holds half of its row's d (the lane 32 further on holds the rest)
  float delta = 0.f;
#pragma unroll
  for (int ks = 0; ks < kKS; ++ks) {
    union {
      bf16x8 v;
      uint32_t w[4];
    } o, g;
    o.v = of[ks];
    g.v = kDoInLds ? rows_frag<HD>(slab, 0, ks, lane) : dof[ks];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      delta = fmaf(__uint_as_float(o.w[i] << 16), __uint_as_float(g.w[i] << 16), delta);
      delta = fmaf(__uint_as_float(o.w[i] & 0xffff0000u), __uint_as_float(g.w[i] & 0xffff0000u), delta);
    }
  }
  delta += __shfl_xor(delta, 32);
  if (qr.active && q_lane < L && hf == 0) a.delta_out[stat] = delta;
  const float dls = delta * a.scale;
  const float c2 = a.scale * kLog2e;
  if (!kDoInLds) {
    wait_loads();
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) qf[ks] = rows_frag<HD>(slab, 0, ks, lane);
  }

  f32x16 dq[kBlk];
#pragma unroll
  for (int i = 0; i < kBlk; ++i) dq[i] = zero16();

  auto process = [&](int t, const char* st) {
    const int kv0 = t * kTR;
    const char *kt_ = st, *vt_ = st + kTileBytes;
    constexpr int kKvb = kTR / 32, kT = kTR / 16;
    bf16x8 dsf[kT];
    // Pinning the fragment reads ahead of their MFMAs, as the forward kernel does, costs this
    // kernel more registers than it has at either width (its q fragments end up spilled): the
    // scheduler is left alone.
    constexpr bool kPinned = HD == 256;
    constexpr int kDepth = 1, kRing = kDepth + 1;
    constexpr int kItems1 = kKvb * kKS;  // first products, item n = kvb*kKS + ks
    constexpr int kItems2 = kT * kBlk;   // last product, item n = t*kBlk + blk
    bf16x8 fk[kRing], fv[kRing], fd[kDoInLds ? kRing : 1], ck[kRing];
    auto fetch_rows = [&](int n) {
      fk[n % kRing] = rows_frag<HD>(kt_, (n / kKS) * 32, n % kKS, lane);
      fv[n % kRing] = rows_frag<HD>(vt_, (n / kKS) * 32, n % kKS, lane);
      if (kDoInLds) fd[n % kRing] = rows_frag<HD>(slab, 0, n % kKS, lane);
    };
    auto fetch_cols = [&](int n) { ck[n % kRing] = cols_frag<HD>(kt_, (n % kBlk) * 32, (n / kBlk) * 16, lane); };
    if (kPinned) {
#pragma unroll
      for (int n = 0; n < kDepth; ++n) fetch_rows(n);
    }
#pragma unroll
    for (int kvb = 0; kvb < kKvb; ++kvb) {
      f32x16 s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) {
        if (kPinned) {
          const int n = kvb * kKS + ks;
          if (n + kDepth < kItems1)
            fetch_rows(n + kDepth);
          else
            fetch_cols(n + kDepth - kItems1);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[n % kRing], qf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[n % kRing], kDoInLds ? fd[n % kRing] : dof[ks], dp, 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        } else {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows_frag<HD>(kt_, kvb * 32, ks, lane), qf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows_frag<HD>(vt_, kvb * 32, ks, lane),
                                                       kDoInLds ? rows_frag<HD>(slab, 0, ks, lane) : dof[kDoInLds ? 0 : ks],
                                                       dp, 0, 0, 0);
        }
      }
      float ds[16];
      const bool need_mask = kv0 + kTR > L || (a.causal && kv0 + kTR - 1 > q0w);
#pragma unroll
      for (int jj = 0; jj < 16; ++jj) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[jj], c2, -lse2));
        ds[jj] = p * fmaf(dp[jj], a.scale, -dls);  // p * (dp - delta) * scale
      }
      if (need_mask) {  // one wave-uniform branch; whatever a hidden pair produced is discarded
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
          const int kv = kv0 + kvb * 32 + acc_row(jj, hf);
          const bool vis = kv < L && (!a.causal || kv <= q_lane);
          ds[jj] = vis ? ds[jj] : 0.f;
        }
      }
      dsf[kvb * 2 + 0] = pack8(ds);
      dsf[kvb * 2 + 1] = pack8(ds + 8);
      if (kPinned) __builtin_amdgcn_sched_barrier(0);
    }
    if (kPinned) {
#pragma unroll
      for (int n = 0; n < kItems2; ++n) {
        if (n + kDepth < kItems2) fetch_cols(n + kDepth);
        dq[n % kBlk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ck[n % kRing], dsf[n / kBlk], dq[n % kBlk], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int blk = 0; blk < kBlk; ++blk)
#pragma unroll
        for (int t2 = 0; t2 < kT; ++t2)
          dq[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cols_frag<HD>(kt_, blk * 32, t2 * 16, lane), dsf[t2],
                                                            dq[blk], 0, 0, 0);
    }
  };
  for (int t = 0; t < my_tiles; ++t) {
    char* cur = (t & 1) ? stage1 : stage0;
    char* nxt = (t & 1) ? stage0 : stage1;
    wait_loads_then_barrier();
    if (t + 1 < n_tiles) issue(t + 1, nxt);
    process(t, cur);
  }
  for (int t = my_tiles; t < n_tiles; ++t) {  // tiles only later waves of the workgroup can see
    wait_loads_then_barrier();
    if (t + 1 < n_tiles) issue(t + 1, (t & 1) ? stage0 : stage1);
  }
  if (!S::kOwnSlabs) __syncthreads();  // stage 1 may still be read by a slower wave
  if (!qr.active) return;
  store_rows_bf16<HD>(a.out0 + head0, rs, q0w, L, dq, 1.f, slab, lane);
}

// dk, dv: one workgroup per NWAVES*32 memory rows; loops over query tiles.  DK / DV select which of
// the two gradients a launch produces: both at head width 128; at 256 one launch each (a wave
// cannot hold its K and V fragments and both accumulator sets), each recomputing the
// probabilities it needs.
template <int HD, int NWAVES, bool DK, bool DV>
__global__ void __launch_bounds__(NWAVES * 64, 1) attn_dkv_kernel(AttnArgs a) {
  using G = Geo<HD>;
  constexpr int kTileBytes = G::kTileBytes, kSlabBytes = G::kSlabBytes, kKS = G::kKS, kBlk = G::kBlk;
  static_assert(DK || DV, "something to compute");
  __shared__ __attribute__((aligned(1024))) char stage0[2 * kTileBytes];  // Q tile, dO tile
  __shared__ __attribute__((aligned(1024))) char stage1[2 * kTileBytes];
  __shared__ __attribute__((aligned(16))) float stats0[2 * kTileRows];  // lse * log2(e), delta
  __shared__ __attribute__((aligned(16))) float stats1[2 * kTileRows];
  // Slabs (a wave's K rows and V rows on the way in, its dk and dv rows on the way out): two per
  // wave when both gradients are produced, else one that serves K, V and the result in turn.  The
  // 4-wave kernel at width 128 gives them LDS of their own (registers allow one workgroup per CU
  // anyway); the others borrow stage 1, which the pipeline first writes at the barrier of its
  // first step and last reads before the barrier that precedes the final stores.
  constexpr bool kTwoSlabs = DK && DV;
  constexpr int kSlabsPerWave = kTwoSlabs ? 2 : 1;
  constexpr bool kOwnSlabs = HD == 128 && NWAVES == 4 && kTwoSlabs;
  static_assert(kOwnSlabs || NWAVES * kSlabsPerWave * kSlabBytes <= 2 * kTileBytes, "borrowed slabs fit stage 1");
  __shared__ __attribute__((aligned(1024))) char slabs[kOwnSlabs ? NWAVES * 2 * kSlabBytes : 16];
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* slab_k = (kOwnSlabs ? slabs : stage1) + wave * kSlabsPerWave * kSlabBytes;
  char* slab_v = kTwoSlabs ? slab_k + kSlabBytes : slab_k;
  const int L = a.length, H = a.heads;
  const int b = blockIdx.y, h = blockIdx.x;
  const int kvblk0 = blockIdx.z * (NWAVES * 32);  // causal: early memory rows are seen by more queries
  const int64_t rs = (int64_t)H * HD;
  const int64_t head0 = ((int64_t)b * L) * rs + (int64_t)h * HD;
  const bf16_t *qb = a.q + head0, *kb = a.k + head0, *vb = a.v + head0, *dob = a.dctx + head0;
  const float* lse_row = a.lse_in + ((int64_t)b * H + h) * L;
  const float* delta_row = a.delta_in + ((int64_t)b * H + h) * L;

  const int kv_row0 = kvblk0 + wave * 32;                // this wave's memory rows
  const int kv_lane = kv_row0 + (lane & 31);             // this lane's memory row
  bf16x8 kf[kKS], vf[DK ? kKS : 1];                      // its K (and V) fragments, set before the tile loop
  const float c2 = a.scale * kLog2e;
  f32x16 dk[DK ? kBlk : 1], dv[DV ? kBlk : 1];
#pragma unroll
  for (int i = 0; i < kBlk; ++i) {
    if (DK) dk[i] = zero16();
    if (DV) dv[i] = zero16();
  }

  const int t_begin = a.causal ? kvblk0 / kTileRows : 0;  // earlier queries see none of these rows
  const int t_end = (L + kTileRows - 1) / kTileRows;
  // The per-query statistics of a tile travel through registers of the first 64 threads: loaded
  // with the tile (no wait), written to LDS after the wait that ends the tile's flight.
  float st_lse = 0.f, st_delta = 0.f;
  auto issue = [&](int t, char* st) {
    const int q0 = t * kTileRows;
    load_tile<HD, NWAVES>(qb, (uint32_t)(rs * 2), q0, L, st, wave, lane);
    load_tile<HD, NWAVES>(dob, (uint32_t)(rs * 2), q0, L, st + kTileBytes, wave, lane);
    if (threadIdx.x < kTileRows) {
      const int qi = min(q0 + (int)threadIdx.x, L - 1);
      st_lse = lse_row[qi];
      if (DK) st_delta = delta_row[qi];
    }
  };
  // Called between the wait and the barrier that open a step: every wave is past its reads of
  // the tile that used `stats` two steps ago (it passed the previous barrier after them).
  auto commit_stats = [&](float* stats) {
    if (threadIdx.x < kTileRows) {
      stats[threadIdx.x] = st_lse * kLog2e;
      stats[kTileRows + threadIdx.x] = st_delta * a.scale;
    }
  };
  // One wave per SIMD here, so nothing but this wave's own instruction order hides the LDS
  // latency: every operand fragment is fetched kDepth MFMA pairs ahead of its use, through rings
  // of kDepth+1 register buffers, and a scheduling barrier after each pair keeps that order (left
  // alone, the scheduler sinks each read to just before its MFMA and every pair waits out a full
  // LDS round trip).
  constexpr int kDepth = 3;
  constexpr int kRowItems = 2 * kKS;   // first products: item n = qblk*kKS + ks
  constexpr int kColItems = kBlk * 4;  // second products: item n = blk*4 + t
  auto process = [&](int t, const char* st, const float* stats) {
    const int q0 = t * kTileRows;
    const char *qt_ = st, *dot_ = st + kTileBytes;
    const float *lset_ = stats, *delt_ = stats + kTileRows;
    if (a.causal && q0 + kTileRows - 1 < kvblk0 + wave * 32) return;  // all queries precede this wave's rows
    bf16x8 pf[DV ? 4 : 1], dsf[DK ? 4 : 1];
    // first products: (Q rows, dO rows) fragments of k-step ks
    bf16x8 fq[kDepth + 1], fo[DK ? kDepth + 1 : 1];
    auto fetch_rows = [&](int n) {
      fq[n & kDepth] = rows_frag<HD>(qt_, (n / kKS) * 32, n % kKS, lane);
      if (DK) fo[n & kDepth] = rows_frag<HD>(dot_, (n / kKS) * 32, n % kKS, lane);
    };
    // second products: (dO^T, Q^T) fragments of 32 columns x 16 queries
    bf16x8 co[DV ? kDepth + 1 : 1], cq[DK ? kDepth + 1 : 1];
    auto fetch_cols = [&](int n) {
      if (DV) co[n & kDepth] = cols_frag<HD>(dot_, (n >> 2) * 32, (n & 3) * 16, lane);
      if (DK) cq[n & kDepth] = cols_frag<HD>(qt_, (n >> 2) * 32, (n & 3) * 16, lane);
    };
    static_assert((kDepth & (kDepth + 1)) == 0, "ring index by mask");
#pragma unroll
    for (int n = 0; n < kDepth; ++n) fetch_rows(n);
#pragma unroll
    for (int qblk = 0; qblk < 2; ++qblk) {
      f32x16 s = zero16(), dp = zero16();
      // the statistics of this block's queries: read now, needed after the MFMAs
      f32x4 l4[4], d4[4];  // lse * log2(e), delta * scale of 4 consecutive query rows per group
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int r0 = qblk * 32 + g4 * 8 + hf * 4;
        l4[g4] = *LDS_PTR(const f32x4, reinterpret_cast<const char*>(lset_) + r0 * 4);
        if (DK) d4[g4] = *LDS_PTR(const f32x4, reinterpret_cast<const char*>(delt_) + r0 * 4);
      }
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) {
        const int n = qblk * kKS + ks;
        if (n + kDepth < kRowItems)
          fetch_rows(n + kDepth);
        else
          fetch_cols(n + kDepth - kRowItems);  // the last steps already bring in the second products' operands
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n & kDepth], kf[ks], s, 0, 0, 0);
        if (DK) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[n & kDepth], vf[ks], dp, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      float p[16], ds[16];
      // a hidden (query, memory) pair can only occur on ragged or diagonal tiles (wave-uniform)
      const bool need_mask = q0 + kTileRows > L || kvblk0 + wave * 32 + 32 > L ||
                             (a.causal && kvblk0 + wave * 32 + 31 > q0);
#pragma unroll
      for (int jj = 0; jj < 16; ++jj) {
        p[jj] = __builtin_amdgcn_exp2f(fmaf(s[jj], c2, -l4[jj >> 2][jj & 3]));
        if (DK) ds[jj] = p[jj] * fmaf(dp[jj], a.scale, -d4[jj >> 2][jj & 3]);  // p * (dp - delta) * scale
      }
      if (need_mask) {  // one wave-uniform branch; whatever a hidden pair produced is discarded
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
          const int qi = q0 + qblk * 32 + acc_row(jj, hf);
          const bool vis = qi < L && kv_lane < L && (!a.causal || kv_lane <= qi);
          p[jj] = vis ? p[jj] : 0.f;
          if (DK) ds[jj] = vis ? ds[jj] : 0.f;
        }
      }
      if (DV) {
        pf[qblk * 2 + 0] = pack8(p);
        pf[qblk * 2 + 1] = pack8(p + 8);
      }
      if (DK) {
        dsf[qblk * 2 + 0] = pack8(ds);
        dsf[qblk * 2 + 1] = pack8(ds + 8);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int n = 0; n < kColItems; ++n) {
      const int blk = n >> 2, tq = n & 3;
      if (n + kDepth < kColItems) fetch_cols(n + kDepth);
      if (DV) dv[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(co[n & kDepth], pf[tq], dv[blk], 0, 0, 0);
      if (DK) dk[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cq[n & kDepth], dsf[tq], dk[blk], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // this wave's K (and V) rows and the first Q/dO tile travel together
  constexpr int kTileLoads = 2 * (G::kTileRuns / NWAVES);  // loads per wave of one issue()
  load_slab<HD>(kb, (uint32_t)(rs * 2), kv_row0, L, slab_k, lane);
  if (DK && kTwoSlabs) load_slab<HD>(vb, (uint32_t)(rs * 2), kv_row0, L, slab_v, lane);
  issue(t_begin, stage0);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kTileLoads) : "memory");  // the slabs have landed
#pragma unroll
  for (int ks = 0; ks < kKS; ++ks) {
    kf[ks] = rows_frag<HD>(slab_k, 0, ks, lane);
    if (DK && kTwoSlabs) vf[ks] = rows_frag<HD>(slab_v, 0, ks, lane);
  }
  if (DK && !kTwoSlabs) {  // the one slab takes the V rows next
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // K fragments read before the slab is overwritten
    load_slab<HD>(vb, (uint32_t)(rs * 2), kv_row0, L, slab_v, lane);
    wait_loads();
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) vf[ks] = rows_frag<HD>(slab_v, 0, ks, lane);
  }
  for (int t = t_begin; t < t_end; t += 2) {
    wait_loads();
    commit_stats(stats0);
    __syncthreads();
    if (t + 1 < t_end) issue(t + 1, stage1);
    process(t, stage0, stats0);
    if (t + 1 >= t_end) break;
    wait_loads();
    commit_stats(stats1);
    __syncthreads();
    if (t + 2 < t_end) issue(t + 2, stage0);
    process(t + 1, stage1, stats1);
  }
  if (!kOwnSlabs) __syncthreads();  // stage 1 may still be read by a slower wave
  if (DK) store_rows_bf16<HD>(a.out0 + head0, rs, kv_row0, L, dk, 1.f, slab_k, lane);
  if (DV) store_rows_bf16<HD>(a.out1 + head0, rs, kv_row0, L, dv, 1.f, slab_v, lane);
}

int check_shape(const AttnShape& s) {
  if (s.batch <= 0 || s.length <= 0 || s.heads <= 0)
    return fail(MTF_ERR_SIZE_MISMATCH, "attention shape %d x %d x %d", s.batch, s.length, s.heads);
  if (!attn_fused_width(s.head_dim))
    return fail(MTF_ERR_UNSUPPORTED, "fused attention needs d_k = d_v = 128 or 256, not %d", s.head_dim);
  // grid = (heads, batch, row blocks of >= 64 rows): heads vary fastest so that every XCD
  // (workgroups go to XCDs round-robin) gets row blocks of every weight
  if (s.batch > 65535 || s.length > 65535 * 64) return fail(MTF_ERR_UNSUPPORTED, "batch > 65535 or length > 65535*64");
  if ((int64_t)s.length * s.heads * s.head_dim * 2 >= (int64_t)1 << 32)
    return fail(MTF_ERR_UNSUPPORTED, "length * heads too large for 32-bit tile offsets");
  return MTF_OK;
}

AttnArgs make_args(const AttnShape& s) {
  AttnArgs a{};
  a.batch = s.batch;
  a.length = s.length;
  a.heads = s.heads;
  a.scale = s.scale;
  a.causal = s.causal;
  return a;
}

// Query (or memory) rows per workgroup: as many as still give every CU a workgroup (more rows
// share each K/V tile that is loaded); `max_waves` caps it for the register-hungry kernel.
int waves_per_group(const AttnShape& s, int max_waves) {
  for (int nw = max_waves; nw > 2; nw /= 2)
    if (ceil_div(s.length, nw * 32) * s.heads * s.batch >= 256) return nw;
  return 2;
}

dim3 row_block_grid(const AttnShape& s, int nw) {
  return dim3((unsigned)s.heads, (unsigned)s.batch, (unsigned)ceil_div(s.length, nw * 32));
}

}  // namespace

bool attn_fused_width(int64_t head_dim) { return head_dim == 128 || head_dim == 256; }

int attn_fwd_launch(const AttnShape& s, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                    bf16_t* ctx, float* lse, hipStream_t stream) {
  if (int rc = check_shape(s)) return rc;
  AttnArgs a = make_args(s);
  a.q = q; a.k = k; a.v = v; a.out0 = ctx; a.lse_out = lse;
  // algorithmic work: two contractions over the visible (l, m) pairs
  const double pairs = s.causal ? 0.5 * s.length * (s.length + 1.0) : (double)s.length * s.length;
  const double flops = 2.0 * 2.0 * s.batch * s.heads * pairs * s.head_dim;
  const double bytes = 4.0 * s.batch * s.length * s.heads * s.head_dim * 2;
  if (s.head_dim == 256) {  // one wave per SIMD at this width: two workgroups of 2 waves share a CU
    LaunchTimer timer("attn_fwd_kernel<256, 2>", flops, bytes, stream);
    attn_fwd_kernel<256, 2><<<row_block_grid(s, 2), 128, 0, stream>>>(a);
    return launch_status("attn_fwd_kernel");
  }
  const int nw = waves_per_group(s, 8);
  const dim3 grid = row_block_grid(s, nw);
  if (nw == 8) {
    LaunchTimer timer("attn_fwd_kernel<128, 8>", flops, bytes, stream);
    attn_fwd_kernel<128, 8><<<grid, 512, 0, stream>>>(a);
  } else if (nw == 4) {
    LaunchTimer timer("attn_fwd_kernel<128, 4>", flops, bytes, stream);
    attn_fwd_kernel<128, 4><<<grid, 256, 0, stream>>>(a);
  } else {
    LaunchTimer timer("attn_fwd_kernel<128, 2>", flops, bytes, stream);
    attn_fwd_kernel<128, 2><<<grid, 128, 0, stream>>>(a);
  }
  return launch_status("attn_fwd_kernel");
}

int attn_bwd_launch(const AttnShape& s, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                    const bf16_t* ctx, const float* lse, const bf16_t* dctx, bf16_t* dq, bf16_t* dk,
                    bf16_t* dv, float* delta, hipStream_t stream) {
  if (int rc = check_shape(s)) return rc;
  const double pairs = s.causal ? 0.5 * s.length * (s.length + 1.0) : (double)s.length * s.length;
  const double unit = 2.0 * s.batch * s.heads * pairs * s.head_dim;  // one contraction over visible pairs
  const double act = (double)s.batch * s.length * s.heads * s.head_dim * 2;
  AttnArgs a = make_args(s);
  a.q = q; a.k = k; a.v = v; a.ctx = ctx; a.dctx = dctx; a.lse_in = lse; a.delta_in = delta; a.delta_out = delta;
  a.out0 = dq;
  if (s.head_dim == 256) {
    const dim3 grid = row_block_grid(s, 4);
    {  // dq = einsum(ds, k) (+ delta): 1 of the 4 backward contractions
      LaunchTimer timer("attn_dq_kernel<256, 4>", unit, 6.0 * act, stream);
      attn_dq_kernel<256, 4><<<grid, 256, 0, stream>>>(a);
    }
    if (int rc = launch_status("attn_dq_kernel")) return rc;
    a.out0 = dk;
    a.out1 = dv;
    {  // dk = einsum(ds, q) (dp recomputed with it): 2 of the 4
      LaunchTimer timer("attn_dkv_kernel<256, 4, true, false>", 2.0 * unit, 5.0 * act, stream);
      attn_dkv_kernel<256, 4, true, false><<<grid, 256, 0, stream>>>(a);
    }
    if (int rc = launch_status("attn_dkv_kernel (dk)")) return rc;
    {  // dv = einsum(p, dctx): the last one
      LaunchTimer timer("attn_dkv_kernel<256, 4, false, true>", unit, 4.0 * act, stream);
      attn_dkv_kernel<256, 4, false, true><<<grid, 256, 0, stream>>>(a);
    }
    return launch_status("attn_dkv_kernel (dv)");
  }
  {  // dq = einsum(ds, k): 1 of the 4 backward contractions (the recomputed logits and dp are overhead here)
    const int nw = waves_per_group(s, 8);
    const dim3 grid = row_block_grid(s, nw);
    LaunchTimer timer(nw == 8 ? "attn_dq_kernel<128, 8>" : nw == 4 ? "attn_dq_kernel<128, 4>" : "attn_dq_kernel<128, 2>",
                      unit, 6.0 * act, stream);
    if (nw == 8)
      attn_dq_kernel<128, 8><<<grid, 512, 0, stream>>>(a);
    else if (nw == 4)
      attn_dq_kernel<128, 4><<<grid, 256, 0, stream>>>(a);
    else
      attn_dq_kernel<128, 2><<<grid, 128, 0, stream>>>(a);
  }
  if (int rc = launch_status("attn_dq_kernel")) return rc;
  const int nw = waves_per_group(s, 4);
  const dim3 grid = row_block_grid(s, nw);
  a.out0 = dk;
  a.out1 = dv;
  {  // dp, dv, dk: 3 of the 4 backward contractions
    LaunchTimer timer(nw == 4 ? "attn_dkv_kernel<128, 4, true, true>" : "attn_dkv_kernel<128, 2, true, true>",
                      3.0 * unit, 6.0 * act, stream);
    if (nw == 4)
      attn_dkv_kernel<128, 4, true, true><<<grid, 256, 0, stream>>>(a);
    else
      attn_dkv_kernel<128, 2, true, true><<<grid, 128, 0, stream>>>(a);
  }
  return launch_status("attn_dkv_kernel");
}

}  // namespace mtf
