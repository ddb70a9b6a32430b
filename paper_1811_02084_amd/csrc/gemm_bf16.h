// Launcher interface of the bf16 MFMA GEMM family (gfx950).
#pragma once
#include <hip/hip_runtime.h>

#include "device_common.h"

namespace mtf {

constexpr int kMaxSegments = 3;
constexpr int kMaxGroup = 4;
constexpr int kMaxSlots = 8;  // (A, B, K) triples of one launch: problems x segments per problem

// C[z][m][n] (+)= alpha * sum_s sum_k A_s[z][m][k] * B_s[z][k][n], then the epilogue.
//
// Operands are bf16.  An operand is either "k-contiguous" (consecutive k adjacent in memory;
// ld = stride between consecutive m resp. n) or "mn-contiguous" (consecutive m resp. n adjacent;
// ld = stride between consecutive k).  C is row-major with n contiguous.  Up to kMaxSegments
// (A, B, K) triples share M, N, the leading dims and the layout flags and are accumulated into
// one C (a contraction whose reduced dim is spread over several tensors).
struct GemmDesc {
  int nseg = 1;
  const bf16_t* A[kMaxSegments] = {nullptr, nullptr, nullptr};
  const bf16_t* B[kMaxSegments] = {nullptr, nullptr, nullptr};
  int64_t K[kMaxSegments] = {0, 0, 0};
  int64_t M = 0, N = 0;
  bool a_kcontig = true, b_kcontig = false;
  int64_t lda = 0, ldb = 0, ldc = 0;
  void* C = nullptr;
  bool out_bf16 = false;
  int epi = MTF_EPI_NONE;      // mtf_epilogue
  const bf16_t* aux = nullptr; // MTF_EPI_MASK_GT0: same shape / ldc / batch strides as C
  // optional: bias[n] (N values, 8-byte aligned) added to every row after alpha / accumulate and
  // before the epilogue: C = epi(alpha * sum + old C + bias).  Not with grouped launches.
  const bf16_t* bias = nullptr;
  // optional: one fp32 factor per output row, row_scale[z * M + m] (z = batch index), applied to
  // alpha * sum before accumulate / bias / epilogue (softmax normalisation of an attention row)
  const float* row_scale = nullptr;
  float alpha = 1.f;
  bool accumulate = false;
  // batch: z = z0 * batch1 + z1
  int64_t batch0 = 1, batch1 = 1;
  int64_t sA0 = 0, sA1 = 0, sB0 = 0, sB1 = 0, sC0 = 0, sC1 = 0;
  // Grouped launch: up to kMaxGroup - 1 further independent problems with the same operand
  // layouts, epilogue (NONE only), output dtype and alpha run in the same launch, so that several
  // small outputs fill the machine together.  Every problem of the group has `nseg` segments
  // ((1 + nextra) * nseg <= kMaxSlots; a segment may have K = 0).  No batch, no accumulate.
  struct Extra {
    const bf16_t* A[kMaxSegments] = {nullptr, nullptr, nullptr};
    const bf16_t* B[kMaxSegments] = {nullptr, nullptr, nullptr};
    int64_t K[kMaxSegments] = {0, 0, 0};
    void* C = nullptr;
    int64_t M = 0, N = 0, lda = 0, ldb = 0, ldc = 0;
  };
  int nextra = 0;
  Extra extra[kMaxGroup - 1];
};

// True when the MFMA kernel can run this problem (alignment, divisibility of the leading dims by
// 8 elements, leading dims small enough for the kernel's 32-bit per-lane byte offsets); otherwise
// the caller must use the generic kernel.  Looks at sizes and addresses only (no GPU needed).
bool gemm_bf16_supported(const GemmDesc& d);

// Enqueues the GEMM on `stream`.  Returns MTF_OK or an error code (nothing launched on error).
int gemm_bf16_launch(const GemmDesc& d, hipStream_t stream);

}  // namespace mtf
