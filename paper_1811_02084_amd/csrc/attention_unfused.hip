// The attention core as the paper's operations, for head widths the fused kernels do not cover:
// logits = einsum(q[b,l,h,k], k[b,m,h,k] -> [b,h,l,m]) and ctx = einsum(p[b,h,l,m], v[b,m,h,v] ->
// [b,l,h,v]) run on the GEMM kernel with (batch, heads) as batch dims (no operand is moved: the
// head stride is a batch stride), the softmax over memory_length between them is a row kernel
// (reduce_max, exp, reduce_sum: memory_length is not split, so these reductions are local).
// Backward: the same einsums transposed, and the softmax Jacobian as a row kernel.
// Also the dispatcher behind mtf_attention_fwd / mtf_attention_bwd.
#include <algorithm>

#include "attention.h"
#include "device_common.h"
#include "gemm_bf16.h"
#include "timing.h"

namespace mtf {
namespace {

size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }

// One wave per row of the [rows, m] logits (already scaled): e = exp(s - row max) on the visible
// positions (bf16, hidden positions exactly 0), inv = 1 / row sum of the unrounded e (the second
// einsum multiplies its rows by it), lse = log-sum-exp.  Row r belongs to query l = r % length;
// position j is visible iff !causal or j <= l.
__global__ void __launch_bounds__(256) softmax_rows_kernel(const float* __restrict__ s, bf16_t* __restrict__ p,
                                                          float* __restrict__ lse, float* __restrict__ inv_out,
                                                          int64_t rows, int length, int mem, int causal) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int l = (int)(r % length);
  const int vis = causal ? min(mem, l + 1) : mem;
  const float* sr = s + r * mem;
  float mx = -INFINITY;
  for (int j = lane; j < vis; j += 64) mx = fmaxf(mx, sr[j]);
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m));
  float tot = 0.f;
  for (int j = lane; j < vis; j += 64) tot += __expf(sr[j] - mx);
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) tot += __shfl_xor(tot, m);
  bf16_t* pr = p + r * mem;
  for (int j = lane; j < mem; j += 64) pr[j] = j < vis ? f32_to_bf16(__expf(sr[j] - mx)) : (bf16_t)0;
  if (lane == 0) {
    lse[r] = mx + __logf(tot);
    inv_out[r] = 1.f / tot;
  }
}

// delta[b,h,l] = sum_v dctx[b,l,h,v] * ctx[b,l,h,v] (= sum_m p * dp of the softmax Jacobian, taken
// from the stored ctx).  16 lanes per (b, l, h) row, 8 values per lane and pass.
__global__ void __launch_bounds__(256) delta_rows_kernel(const bf16_t* __restrict__ ctx, const bf16_t* __restrict__ dctx,
                                                        float* __restrict__ delta, int64_t rows, int length, int heads,
                                                        int width) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);  // (b, l, h) in memory order
  const int sub = threadIdx.x & 15;
  float acc = 0.f;
  if (row < rows)
    for (int c = sub * 8; c < width; c += 128) {
      const uint4 x = *reinterpret_cast<const uint4*>(ctx + row * width + c);
      const uint4 y = *reinterpret_cast<const uint4*>(dctx + row * width + c);
      const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc = fmaf(__uint_as_float(xs[i] << 16), __uint_as_float(ys[i] << 16), acc);
        acc = fmaf(__uint_as_float(xs[i] & 0xffff0000u), __uint_as_float(ys[i] & 0xffff0000u), acc);
      }
    }
#pragma unroll
  for (int m = 8; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
  if (row < rows && sub == 0) {
    const int64_t h = row % heads, l = (row / heads) % length, b = row / ((int64_t)heads * length);
    delta[(b * heads + h) * length + l] = acc;
  }
}

// Backward row kernel: p = exp(s - lse) on the visible positions (s already scaled),
// ds = p * (dp - delta) * scale.  Writes p and ds as bf16.
__global__ void __launch_bounds__(256) softmax_bwd_rows_kernel(const float* __restrict__ s, const float* __restrict__ dp,
                                                              const float* __restrict__ lse,
                                                              const float* __restrict__ delta_in, bf16_t* __restrict__ p,
                                                              bf16_t* __restrict__ ds, int64_t rows, int length,
                                                              int mem, int causal, float scale) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int l = (int)(r % length);
  const int vis = causal ? min(mem, l + 1) : mem;
  const float* sr = s + r * mem;
  const float* dr = dp + r * mem;
  const float z = lse[r];
  const float delta = delta_in[r];
  for (int j = lane; j < mem; j += 64) {
    const float pj = j < vis ? __expf(sr[j] - z) : 0.f;
    p[r * mem + j] = f32_to_bf16(pj);
    ds[r * mem + j] = f32_to_bf16(pj * (dr[j] - delta) * scale);
  }
}

struct Geometry {
  int64_t B, L, H, K;           // batch, length (= memory length), heads, head width
  int64_t row;                  // H * K: row pitch of q / k / v / ctx
  int64_t act, sq;              // elements of one [b,l,h,k] tensor and of one [b,h,l,m] tensor
};
Geometry geometry(const mtf_mha_dims* d) {
  Geometry g;
  g.B = d->batch; g.L = d->length; g.H = d->heads; g.K = d->d_k;
  g.row = g.H * g.K;
  g.act = g.B * g.L * g.row;
  g.sq = g.B * g.H * g.L * g.L;
  return g;
}

// [b,h,l,m] = alpha * X[b,l,h,:] . Y[b,m,h,:]  (both row operands: "nt"), fp32 out
GemmDesc rows_times_rows(const Geometry& g, const bf16_t* x, const bf16_t* y, float* out, float alpha) {
  GemmDesc d;
  d.A[0] = x; d.B[0] = y; d.K[0] = g.K;
  d.M = g.L; d.N = g.L;
  d.a_kcontig = true; d.b_kcontig = true;
  d.lda = g.row; d.ldb = g.row; d.ldc = g.L;
  d.C = out; d.out_bf16 = false; d.alpha = alpha;
  d.batch0 = g.B; d.batch1 = g.H;
  d.sA0 = g.L * g.row; d.sA1 = g.K;
  d.sB0 = g.L * g.row; d.sB1 = g.K;
  d.sC0 = g.H * g.L * g.L; d.sC1 = g.L * g.L;
  return d;
}
// out[b,l,h,:] = W[b,h,l,m] . Y[b,m,h,:]  (transpose_w: W[b,h,m,l]^T, i.e. contraction over W's rows)
GemmDesc square_times_rows(const Geometry& g, const bf16_t* w, bool transpose_w, const bf16_t* y, bf16_t* out) {
  GemmDesc d;
  d.A[0] = w; d.B[0] = y; d.K[0] = g.L;
  d.M = g.L; d.N = g.K;
  d.a_kcontig = !transpose_w; d.b_kcontig = false;
  d.lda = g.L; d.ldb = g.row; d.ldc = g.row;
  d.C = out; d.out_bf16 = true;
  d.batch0 = g.B; d.batch1 = g.H;
  d.sA0 = g.H * g.L * g.L; d.sA1 = g.L * g.L;
  d.sB0 = g.L * g.row; d.sB1 = g.K;
  d.sC0 = g.L * g.row; d.sC1 = g.K;
  return d;
}

int launch(const GemmDesc& d, hipStream_t s) {
  if (!gemm_bf16_supported(d)) return fail(MTF_ERR_UNSUPPORTED, "attention einsum does not fit the GEMM kernel");
  return gemm_bf16_launch(d, s);
}

int check_dims(const mtf_mha_dims* d) {
  if (!d) return fail(MTF_ERR_NULL, "dims");
  if (d->batch <= 0 || d->length <= 0 || d->heads <= 0 || d->d_k <= 0)
    return fail(MTF_ERR_SIZE_MISMATCH, "non-positive attention dim");
  if (d->d_k % 8) return fail(MTF_ERR_UNSUPPORTED, "attention needs d_k divisible by 8");
  if (!attn_fused_width(d->d_k) && d->length % 8)
    return fail(MTF_ERR_UNSUPPORTED, "attention at head widths other than 128 and 256 needs length divisible by 8");
  if (d->batch > INT32_MAX || d->length > INT32_MAX || d->heads > INT32_MAX)
    return fail(MTF_ERR_UNSUPPORTED, "attention dim too large");
  return MTF_OK;
}

}  // namespace
}  // namespace mtf

using namespace mtf;

extern "C" {

size_t mtf_attention_fwd_workspace_bytes(const mtf_mha_dims* d) {
  if (check_dims(d) || attn_fused_width(d->d_k)) return 0;
  const Geometry g = geometry(d);
  // logits fp32, exponentials bf16, 1 / row sums fp32
  return round256((size_t)g.sq * 4) + round256((size_t)g.sq * 2) + round256((size_t)g.B * g.H * g.L * 4);
}

int mtf_attention_fwd(const mtf_mha_dims* d, const void* q, const void* k, const void* v, float scale,
                      int causal, void* ctx, void* lse, void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_dims(d)) return rc;
  if (!q || !k || !v || !ctx || !lse) return fail(MTF_ERR_NULL, "mtf_attention_fwd buffer");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(ctx) || !aligned16(lse) || !aligned16(workspace))
    return fail(MTF_ERR_ALIGN, "mtf_attention_fwd buffer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (attn_fused_width(d->d_k)) {
    AttnShape as{(int)d->batch, (int)d->length, (int)d->heads, (int)d->d_k, scale, causal};
    return attn_fwd_launch(as, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)ctx, (float*)lse, s);
  }
  const size_t need = mtf_attention_fwd_workspace_bytes(d);
  if (!workspace || workspace_bytes < need) return fail(MTF_ERR_WORKSPACE, "mtf_attention_fwd needs %zu bytes", need);
  const Geometry g = geometry(d);
  float* logits = static_cast<float*>(workspace);
  bf16_t* p = reinterpret_cast<bf16_t*>(static_cast<char*>(workspace) + round256((size_t)g.sq * 4));
  float* inv = reinterpret_cast<float*>(static_cast<char*>(workspace) + round256((size_t)g.sq * 4) +
                                        round256((size_t)g.sq * 2));
  if (int rc = launch(rows_times_rows(g, (const bf16_t*)q, (const bf16_t*)k, logits, scale), s)) return rc;
  const int64_t rows = g.B * g.H * g.L;
  {
    LaunchTimer timer("softmax_rows_kernel", 0, 6.0 * g.sq, s);
    softmax_rows_kernel<<<(unsigned)ceil_div(rows, 4), 256, 0, s>>>(logits, p, (float*)lse, inv, rows, (int)g.L,
                                                                   (int)g.L, causal);
  }
  if (int rc = launch_status("softmax_rows_kernel")) return rc;
  // ctx = einsum(e, v) with every row divided by its sum: inv is indexed [b, h, l] like the
  // batch (b, h) and row l of this einsum
  GemmDesc pv = square_times_rows(g, p, false, (const bf16_t*)v, (bf16_t*)ctx);
  pv.row_scale = inv;
  return launch(pv, s);
}

size_t mtf_attention_bwd_workspace_bytes(const mtf_mha_dims* d) {
  if (check_dims(d)) return 0;
  const Geometry g = geometry(d);
  if (attn_fused_width(d->d_k)) return round256((size_t)g.B * g.H * g.L * 4);  // delta
  // logits, dp fp32; p, ds bf16; delta fp32
  return 2 * round256((size_t)g.sq * 4) + 2 * round256((size_t)g.sq * 2) + round256((size_t)g.B * g.H * g.L * 4);
}

int mtf_attention_bwd(const mtf_mha_dims* d, const void* q, const void* k, const void* v, const void* ctx,
                      const void* lse, const void* dctx, float scale, int causal, void* dq, void* dk, void* dv,
                      void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_dims(d)) return rc;
  if (!q || !k || !v || !ctx || !lse || !dctx || !dq || !dk || !dv) return fail(MTF_ERR_NULL, "mtf_attention_bwd buffer");
  for (const void* ptr : {q, k, v, ctx, lse, dctx, (const void*)dq, (const void*)dk, (const void*)dv,
                          (const void*)workspace})
    if (!aligned16(ptr)) return fail(MTF_ERR_ALIGN, "mtf_attention_bwd buffer");
  const size_t need = mtf_attention_bwd_workspace_bytes(d);
  if (!workspace || workspace_bytes < need) return fail(MTF_ERR_WORKSPACE, "mtf_attention_bwd needs %zu bytes", need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (attn_fused_width(d->d_k)) {
    AttnShape as{(int)d->batch, (int)d->length, (int)d->heads, (int)d->d_k, scale, causal};
    return attn_bwd_launch(as, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (const bf16_t*)ctx,
                           (const float*)lse, (const bf16_t*)dctx, (bf16_t*)dq, (bf16_t*)dk, (bf16_t*)dv,
                           (float*)workspace, s);
  }
  const Geometry g = geometry(d);
  char* w = static_cast<char*>(workspace);
  float* logits = reinterpret_cast<float*>(w);
  float* dp = reinterpret_cast<float*>(w + round256((size_t)g.sq * 4));
  bf16_t* p = reinterpret_cast<bf16_t*>(w + 2 * round256((size_t)g.sq * 4));
  bf16_t* ds = reinterpret_cast<bf16_t*>(w + 2 * round256((size_t)g.sq * 4) + round256((size_t)g.sq * 2));
  float* delta = reinterpret_cast<float*>(w + 2 * round256((size_t)g.sq * 4) + 2 * round256((size_t)g.sq * 2));
  // recomputed logits and dp = einsum(dctx[b,l,h,v], v[b,m,h,v] -> [b,h,l,m])
  if (int rc = launch(rows_times_rows(g, (const bf16_t*)q, (const bf16_t*)k, logits, scale), s)) return rc;
  if (int rc = launch(rows_times_rows(g, (const bf16_t*)dctx, (const bf16_t*)v, dp, 1.f), s)) return rc;
  const int64_t rows = g.B * g.H * g.L;
  {
    LaunchTimer timer("delta_rows_kernel", 0, 4.0 * g.act, s);
    delta_rows_kernel<<<(unsigned)ceil_div(rows, 16), 256, 0, s>>>((const bf16_t*)ctx, (const bf16_t*)dctx, delta, rows,
                                                                  (int)g.L, (int)g.H, (int)g.K);
  }
  if (int rc = launch_status("delta_rows_kernel")) return rc;
  {
    LaunchTimer timer("softmax_bwd_rows_kernel", 0, 12.0 * g.sq, s);
    softmax_bwd_rows_kernel<<<(unsigned)ceil_div(rows, 4), 256, 0, s>>>(logits, dp, (const float*)lse, delta, p, ds,
                                                                       rows, (int)g.L, (int)g.L, causal, scale);
  }
  if (int rc = launch_status("softmax_bwd_rows_kernel")) return rc;
  // dv = einsum(p[b,h,l,m], dctx[b,l,h,v] -> [b,m,h,v]); dq = einsum(ds, k); dk = einsum(ds[b,h,l,m], q -> [b,m,h,k])
  if (int rc = launch(square_times_rows(g, p, true, (const bf16_t*)dctx, (bf16_t*)dv), s)) return rc;
  if (int rc = launch(square_times_rows(g, ds, false, (const bf16_t*)k, (bf16_t*)dq), s)) return rc;
  return launch(square_times_rows(g, ds, true, (const bf16_t*)q, (bf16_t*)dk), s);
}

}  // extern "C"
