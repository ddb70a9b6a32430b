// Host side of the bf16 MFMA GEMM family: which problems the kernels take, and which tile shape
// runs a given launch.  The kernel template is in gemm_bf16_kernel.h; each tile shape is compiled
// in its own translation unit (gemm_bf16_<shape>.hip).  Every contraction of the Transformer-layer
// path lowers to this kernel (section "Performance Comparison": the einsums are where the
// computation time goes).
#include "gemm_bf16_kernel.h"


namespace mtf {

// The tile loaders keep per-lane byte offsets relative to the tile origin in 32 bits: up to
// (tile rows - 1) * ld * 2 + 128 for a k-contiguous operand (256-row tile) and 63 * ld * 2 +
// 2 * tile columns for an mn-contiguous one.  Leading dims beyond this would wrap.
namespace {
bool ld_fits_32bit_offsets(int64_t ld, bool kcontig) {
  const int64_t worst = kcontig ? 255 * ld * 2 + 128 : 63 * ld * 2 + 512;
  return ld >= 0 && ld < (INT64_C(1) << 40) && worst <= (int64_t)UINT32_MAX;
}
}  // namespace

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
  if (d.nextra > 0 && ((1 + d.nextra) * d.nseg > kMaxSlots || d.batch0 * d.batch1 != 1 || d.accumulate ||
                       d.epi != MTF_EPI_NONE))
    return false;
  for (int p = 0; p < d.nextra; ++p) {
    const GemmDesc::Extra& e = d.extra[p];
    if (e.M <= 0 || e.N <= 0 || e.M > INT32_MAX || e.N > INT32_MAX) return false;
    if (e.lda % 8 || e.ldb % 8 || e.ldc % 4 || e.N % 8 || (!d.a_kcontig && e.M % 8)) return false;
    for (int s = 0; s < d.nseg; ++s) {
      if (e.K[s] < 0 || e.K[s] > INT32_MAX) return false;
      if ((d.a_kcontig || d.b_kcontig) && e.K[s] % 8) return false;
      if (!e.A[s] || !e.B[s] || !aligned16(e.A[s]) || !aligned16(e.B[s])) return false;
    }
    if (!e.C || !aligned16(e.C)) return false;
  }
  return true;
}

int gemm_bf16_launch(const GemmDesc& d, hipStream_t stream) {
  if (!gemm_bf16_supported(d)) return fail(MTF_ERR_UNSUPPORTED, "GEMM shape/alignment");
  GemmArgs a;
  for (int s = 0; s < kMaxSlots; ++s) {
    a.A[s] = s < d.nseg ? d.A[s] : d.A[0];
    a.B[s] = s < d.nseg ? d.B[s] : d.B[0];
    a.K[s] = s < d.nseg ? (int)d.K[s] : 0;
  }
  for (int s = 0; s < kMaxGroup; ++s) {
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
    for (int s = 0; s < d.nseg; ++s) {
      const int slot = (p + 1) * d.nseg + s;
      a.A[slot] = e.A[s]; a.B[slot] = e.B[s]; a.K[slot] = (int)e.K[s];
    }
    a.C[p + 1] = e.C;
    a.M[p + 1] = (int)e.M; a.N[p + 1] = (int)e.N;
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
  // Tile choice by a cost model in microseconds, fitted to kernel traces of the layer's launches:
  // a 128 x 128 x 1024 block of the iteration space takes a CU about 7.8 us at the large tile's
  // rate; a shape's time is its rounds of tiles over the slots the machine has for it, each round
  // the blocks of a tile at the shape's relative rate plus what the shape exposes of prologue and
  // epilogue (two workgroups per CU cover each other's; one per CU does not).
  auto count = [&](int bm, int bn) {
    int64_t n = ceil_div(d.M, bm) * ceil_div(d.N, bn) * batch;
    for (int p = 0; p < d.nextra; ++p) n += ceil_div(d.extra[p].M, bm) * ceil_div(d.extra[p].N, bn);
    return n;
  };
  double k_total = 0;
  for (int s = 0; s < d.nseg; ++s) k_total += (double)d.K[s];
  for (int p = 0; p < d.nextra; ++p) {
    double k_p = 0;
    for (int s = 0; s < d.nseg; ++s) k_p += (double)d.extra[p].K[s];
    k_total = std::max(k_total, k_p);
  }
  const double block_us = 7.8 * k_total / 1024.0;
  const int64_t large_tiles = count(256, 256), medium_tiles = count(256, 128), small_tiles = count(128, 128);
  const double cost_large = (double)ceil_div(large_tiles, 256) * (4.0 * block_us + 5.0);
  // small tiles: two workgroups share a CU (a round of 512 takes two blocks' time at 0.8 of the
  // rate); with at most one per CU a workgroup of 4 waves runs alone, at about 0.55
  const double cost_small = small_tiles <= 256 ? block_us / 0.55 + 2.0
                                               : (double)ceil_div(small_tiles, 512) * (2.0 * block_us / 0.8 + 2.0);
  // the narrow tile in two k-groups keeps its rate only when A is read along k
  const double cost_split = (double)ceil_div(medium_tiles, 256) * (2.0 * block_us / (d.a_kcontig ? 0.9 : 0.8) + 6.0);
  if (cost_large <= cost_split && cost_large <= cost_small) return launch_large(d, a, batch, stream);
  if (cost_split <= cost_small) return launch_split(d, a, batch, stream);
  return small_tiles <= 256 ? launch_small_deep(d, a, batch, stream) : launch_small(d, a, batch, stream);
}

}  // namespace mtf
