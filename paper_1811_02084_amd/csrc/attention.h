// Launcher interface of the fused softmax-attention kernels (gfx950, head width 128 or 256).
#pragma once
#include <hip/hip_runtime.h>

#include "device_common.h"

namespace mtf {

// d_k = d_v the fused kernels support: 128 (the translation models of the paper's experiments)
// and 256 (its language models).
bool attn_fused_width(int64_t head_dim);

// All tensors use the einsum layouts of the layer: q, k, v, ctx, dctx, dq, dk, dv are
// [batch, length, heads, head_dim] bf16; lse and delta are [batch, heads, length] fp32.
struct AttnShape {
  int batch, length, heads, head_dim;
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
