// Launcher interface of the fused softmax-attention kernels (gfx950, head width 128).
#pragma once
#include <hip/hip_runtime.h>

#include "device_common.h"

namespace mtf {

constexpr int kHeadDim = 128;  // d_k = d_v supported by the fused kernels

// All tensors use the einsum layouts of the layer: q, k, v, ctx, dctx, dq, dk, dv are
// [batch, length, heads, 128] bf16; lse and delta are [batch, heads, length] fp32.
struct AttnShape {
  int batch, length, heads;
  float scale;
  int causal;
};

// ctx = softmax(scale * q k^T [+ causal mask]) v, lse = log-sum-exp of the scaled logits per row.
int attn_fwd_launch(const AttnShape& s, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                    bf16_t* ctx, float* lse, hipStream_t stream);

// Gradients w.r.t. q, k, v given dctx; probabilities are recomputed from q, k and lse.
// delta: caller-provided scratch of batch*heads*length floats.
int attn_bwd_launch(const AttnShape& s, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                    const bf16_t* ctx, const float* lse, const bf16_t* dctx, bf16_t* dq, bf16_t* dk,
                    bf16_t* dv, float* delta, hipStream_t stream);

}  // namespace mtf
