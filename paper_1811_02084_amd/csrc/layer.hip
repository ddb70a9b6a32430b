// Fixed per-processor layer steps: sequences of the local einsums of the model-parallel
// Transformer layout (d_ff and heads split; section 'Model-Parallel "Transformer"'), each lowered
// to the bf16 MFMA GEMM, plus the fused attention kernels.  Outputs that contract a split dim
// (y, dx) are PARTIAL sums in fp32, ready for the Allreduce of the einsum lowering.
#include "attention.h"
#include "device_common.h"
#include "gemm_bf16.h"

namespace mtf {
namespace {

inline size_t round256(size_t n) { return (n + 255) & ~size_t(255); }

// C[M,N] = A op B with both operands given as plain row-major matrices:
//   a_kc: A is [M,K] (k contiguous) else [K,M];   b_kc: B is [N,K] (k contiguous) else [K,N].
GemmDesc gemm(const void* A, bool a_kc, const void* B, bool b_kc, void* C, bool c_bf16, int64_t M,
              int64_t N, int64_t K) {
  GemmDesc d;
  d.A[0] = static_cast<const bf16_t*>(A);
  d.B[0] = static_cast<const bf16_t*>(B);
  d.K[0] = K;
  d.M = M;
  d.N = N;
  d.a_kcontig = a_kc;
  d.b_kcontig = b_kc;
  d.lda = a_kc ? K : M;
  d.ldb = b_kc ? K : N;
  d.ldc = N;
  d.C = C;
  d.out_bf16 = c_bf16;
  return d;
}

int check_ptrs(std::initializer_list<const void*> ptrs, const char* what) {
  for (const void* p : ptrs) {
    if (!p) return fail(MTF_ERR_NULL, "%s", what);
    if (!aligned16(p)) return fail(MTF_ERR_ALIGN, "%s", what);
  }
  return MTF_OK;
}

int check_ffn(const mtf_ffn_dims* d) {
  if (!d) return fail(MTF_ERR_NULL, "dims");
  if (d->batch <= 0 || d->length <= 0 || d->d_model <= 0 || d->d_ff <= 0)
    return fail(MTF_ERR_SIZE_MISMATCH, "non-positive FFN dim");
  if (d->d_model % 8 || d->d_ff % 8)
    return fail(MTF_ERR_UNSUPPORTED, "FFN step needs d_model and d_ff divisible by 8");
  return MTF_OK;
}

int check_mha(const mtf_mha_dims* d) {
  if (!d) return fail(MTF_ERR_NULL, "dims");
  if (d->batch <= 0 || d->length <= 0 || d->d_model <= 0 || d->heads <= 0 || d->d_k <= 0)
    return fail(MTF_ERR_SIZE_MISMATCH, "non-positive attention dim");
  if (d->d_k != kHeadDim) return fail(MTF_ERR_UNSUPPORTED, "fused attention needs d_k = d_v = %d", kHeadDim);
  if (d->d_model % 8) return fail(MTF_ERR_UNSUPPORTED, "attention step needs d_model divisible by 8");
  return MTF_OK;
}

struct MhaBwdScratch {
  bf16_t *dctx, *dq, *dk, *dv;
  float* delta;
  size_t bytes;
};

MhaBwdScratch mha_bwd_scratch(const mtf_mha_dims* d, void* base) {
  const size_t act = round256((size_t)d->batch * d->length * d->heads * d->d_k * 2);
  const size_t stat = round256((size_t)d->batch * d->heads * d->length * 4);
  char* p = static_cast<char*>(base);
  MhaBwdScratch s;
  s.dctx = reinterpret_cast<bf16_t*>(p);
  s.dq = reinterpret_cast<bf16_t*>(p + act);
  s.dk = reinterpret_cast<bf16_t*>(p + 2 * act);
  s.dv = reinterpret_cast<bf16_t*>(p + 3 * act);
  s.delta = reinterpret_cast<float*>(p + 4 * act);
  s.bytes = 4 * act + stat;
  return s;
}

int ffn_fwd(const mtf_ffn_dims* d, const void* x, const void* w_in, const void* w_out, void* a,
            void* y_partial, hipStream_t s) {
  const int64_t T = d->batch * d->length, D = d->d_model, F = d->d_ff;
  // a = relu(einsum(x[b,l,D], w_in[D,F] -> [b,l,F]))
  GemmDesc g1 = gemm(x, true, w_in, false, a, true, T, F, D);
  g1.epi = MTF_EPI_RELU;
  if (int rc = gemm_bf16_launch(g1, s)) return rc;
  // y_partial = einsum(a[b,l,F], w_out[F,D] -> [b,l,D]); F is the split, reduced-out dim
  return gemm_bf16_launch(gemm(a, true, w_out, false, y_partial, false, T, D, F), s);
}

int ffn_bwd(const mtf_ffn_dims* d, const void* x, const void* a, const void* w_in, const void* w_out,
            const void* dy, void* dw_in, void* dw_out, void* dx_partial, void* dh, hipStream_t s) {
  const int64_t T = d->batch * d->length, D = d->d_model, F = d->d_ff;
  // dw_out = einsum(a[b,l,F], dy[b,l,D] -> [F,D])
  if (int rc = gemm_bf16_launch(gemm(a, false, dy, false, dw_out, false, F, D, T), s)) return rc;
  // dh = einsum(dy[b,l,D], w_out[F,D] -> [b,l,F]) * [a > 0]
  GemmDesc g = gemm(dy, true, w_out, true, dh, true, T, F, D);
  g.epi = MTF_EPI_MASK_GT0;
  g.aux = static_cast<const bf16_t*>(a);
  if (int rc = gemm_bf16_launch(g, s)) return rc;
  // dw_in = einsum(x[b,l,D], dh[b,l,F] -> [D,F])
  if (int rc = gemm_bf16_launch(gemm(x, false, dh, false, dw_in, false, D, F, T), s)) return rc;
  // dx_partial = einsum(dh[b,l,F], w_in[D,F] -> [b,l,D])
  return gemm_bf16_launch(gemm(dh, true, w_in, true, dx_partial, false, T, D, F), s);
}

int mha_fwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k, const void* w_v,
            const void* w_o, float scale, int causal, void* q, void* k, void* v, void* ctx, void* lse,
            void* y_partial, hipStream_t s) {
  const int64_t T = d->batch * d->length, D = d->d_model, HK = d->heads * d->d_k;
  // q, k, v = einsum(x[b,l,D], w[D,h,k] -> [b,l,h,k]); D is not split: complete local slices
  if (int rc = gemm_bf16_launch(gemm(x, true, w_q, false, q, true, T, HK, D), s)) return rc;
  if (int rc = gemm_bf16_launch(gemm(x, true, w_k, false, k, true, T, HK, D), s)) return rc;
  if (int rc = gemm_bf16_launch(gemm(x, true, w_v, false, v, true, T, HK, D), s)) return rc;
  AttnShape as{(int)d->batch, (int)d->length, (int)d->heads, scale, causal};
  if (int rc = attn_fwd_launch(as, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)ctx,
                               (float*)lse, s))
    return rc;
  // y_partial = einsum(ctx[b,l,h,v], w_o[h,v,D] -> [b,l,D]); heads is the split, reduced-out dim
  return gemm_bf16_launch(gemm(ctx, true, w_o, false, y_partial, false, T, D, HK), s);
}

int mha_bwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k, const void* w_v,
            const void* w_o, const void* q, const void* k, const void* v, const void* ctx,
            const void* lse, const void* dy, float scale, int causal, void* dw_q, void* dw_k,
            void* dw_v, void* dw_o, void* dx_partial, const MhaBwdScratch& w, hipStream_t s) {
  const int64_t T = d->batch * d->length, D = d->d_model, HK = d->heads * d->d_k;
  // dw_o = einsum(ctx[b,l,h,v], dy[b,l,D] -> [h,v,D])
  if (int rc = gemm_bf16_launch(gemm(ctx, false, dy, false, dw_o, false, HK, D, T), s)) return rc;
  // dctx = einsum(dy[b,l,D], w_o[h,v,D] -> [b,l,h,v])
  if (int rc = gemm_bf16_launch(gemm(dy, true, w_o, true, w.dctx, true, T, HK, D), s)) return rc;
  AttnShape as{(int)d->batch, (int)d->length, (int)d->heads, scale, causal};
  if (int rc = attn_bwd_launch(as, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v,
                               (const bf16_t*)ctx, (const float*)lse, w.dctx, w.dq, w.dk, w.dv, w.delta, s))
    return rc;
  // dw_{q,k,v} = einsum(x[b,l,D], d{q,k,v}[b,l,h,k] -> [D,h,k])
  if (int rc = gemm_bf16_launch(gemm(x, false, w.dq, false, dw_q, false, D, HK, T), s)) return rc;
  if (int rc = gemm_bf16_launch(gemm(x, false, w.dk, false, dw_k, false, D, HK, T), s)) return rc;
  if (int rc = gemm_bf16_launch(gemm(x, false, w.dv, false, dw_v, false, D, HK, T), s)) return rc;
  // dx_partial = sum over {q,k,v} of einsum(d*[b,l,h,k], w_*[D,h,k] -> [b,l,D]): one contraction
  // whose reduced dims (h,k) are spread over three tensor pairs
  GemmDesc g = gemm(w.dq, true, w_q, true, dx_partial, false, T, D, HK);
  g.nseg = 3;
  g.A[1] = w.dk; g.B[1] = static_cast<const bf16_t*>(w_k); g.K[1] = HK;
  g.A[2] = w.dv; g.B[2] = static_cast<const bf16_t*>(w_v); g.K[2] = HK;
  return gemm_bf16_launch(g, s);
}

int residual_add(const void* partial, const void* residual_bf16, void* out_bf16, int64_t count,
                 hipStream_t s) {
  const void* parts[1] = {partial};
  return mtf_reduce_partials(parts, 1, residual_bf16, MTF_BF16, out_bf16, MTF_BF16, count, s);
}

}  // namespace
}  // namespace mtf

using namespace mtf;

extern "C" {

int mtf_ffn_fwd(const mtf_ffn_dims* d, const void* x, const void* w_in, const void* w_out, void* a,
                void* y_partial, void* stream) {
  if (int rc = check_ffn(d)) return rc;
  if (int rc = check_ptrs({x, w_in, w_out, a, y_partial}, "mtf_ffn_fwd buffer")) return rc;
  return ffn_fwd(d, x, w_in, w_out, a, y_partial, static_cast<hipStream_t>(stream));
}

size_t mtf_ffn_bwd_workspace_bytes(const mtf_ffn_dims* d) {
  if (!d || d->batch <= 0 || d->length <= 0 || d->d_ff <= 0) return 0;
  return round256((size_t)d->batch * d->length * d->d_ff * 2);  // dh, bf16
}

int mtf_ffn_bwd(const mtf_ffn_dims* d, const void* x, const void* a, const void* w_in,
                const void* w_out, const void* dy, void* dw_in, void* dw_out, void* dx_partial,
                void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_ffn(d)) return rc;
  if (int rc = check_ptrs({x, a, w_in, w_out, dy, dw_in, dw_out, dx_partial}, "mtf_ffn_bwd buffer")) return rc;
  if (!workspace || workspace_bytes < mtf_ffn_bwd_workspace_bytes(d) || !aligned16(workspace))
    return fail(MTF_ERR_WORKSPACE, "mtf_ffn_bwd needs %zu bytes", mtf_ffn_bwd_workspace_bytes(d));
  return ffn_bwd(d, x, a, w_in, w_out, dy, dw_in, dw_out, dx_partial, workspace,
                 static_cast<hipStream_t>(stream));
}

int mtf_mha_fwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k,
                const void* w_v, const void* w_o, float scale, int causal, void* q, void* k,
                void* v, void* ctx, void* lse, void* y_partial, void* stream) {
  if (int rc = check_mha(d)) return rc;
  if (int rc = check_ptrs({x, w_q, w_k, w_v, w_o, q, k, v, ctx, lse, y_partial}, "mtf_mha_fwd buffer")) return rc;
  return mha_fwd(d, x, w_q, w_k, w_v, w_o, scale, causal, q, k, v, ctx, lse, y_partial,
                 static_cast<hipStream_t>(stream));
}

size_t mtf_mha_bwd_workspace_bytes(const mtf_mha_dims* d) {
  if (!d || d->batch <= 0 || d->length <= 0 || d->heads <= 0 || d->d_k <= 0) return 0;
  return mha_bwd_scratch(d, nullptr).bytes;
}

int mtf_mha_bwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k,
                const void* w_v, const void* w_o, const void* q, const void* k, const void* v,
                const void* ctx, const void* lse, const void* dy, float scale, int causal,
                void* dw_q, void* dw_k, void* dw_v, void* dw_o, void* dx_partial, void* workspace,
                size_t workspace_bytes, void* stream) {
  if (int rc = check_mha(d)) return rc;
  if (int rc = check_ptrs({x, w_q, w_k, w_v, w_o, q, k, v, ctx, lse, dy, dw_q, dw_k, dw_v, dw_o, dx_partial},
                          "mtf_mha_bwd buffer"))
    return rc;
  if (!workspace || workspace_bytes < mtf_mha_bwd_workspace_bytes(d) || !aligned16(workspace))
    return fail(MTF_ERR_WORKSPACE, "mtf_mha_bwd needs %zu bytes", mtf_mha_bwd_workspace_bytes(d));
  return mha_bwd(d, x, w_q, w_k, w_v, w_o, q, k, v, ctx, lse, dy, scale, causal, dw_q, dw_k, dw_v, dw_o,
                 dx_partial, mha_bwd_scratch(d, workspace), static_cast<hipStream_t>(stream));
}

static int check_layer(const mtf_layer_dims* d, mtf_ffn_dims* f, mtf_mha_dims* m) {
  if (!d) return fail(MTF_ERR_NULL, "dims");
  *f = mtf_ffn_dims{d->batch, d->length, d->d_model, d->d_ff};
  *m = mtf_mha_dims{d->batch, d->length, d->d_model, d->heads, d->d_k};
  if (int rc = check_ffn(f)) return rc;
  return check_mha(m);
}

size_t mtf_layer_fwd_workspace_bytes(const mtf_layer_dims* d) {
  if (!d || d->batch <= 0 || d->length <= 0 || d->d_model <= 0) return 0;
  return round256((size_t)d->batch * d->length * d->d_model * 4);  // one fp32 partial sum
}

int mtf_layer_fwd(const mtf_layer_dims* d, const void* x, const mtf_layer_weights* w, float scale,
                  int causal, const mtf_layer_saved* sv, void* z, void* workspace,
                  size_t workspace_bytes, void* stream) {
  mtf_ffn_dims f;
  mtf_mha_dims m;
  if (int rc = check_layer(d, &f, &m)) return rc;
  if (!w || !sv) return fail(MTF_ERR_NULL, "weights / saved");
  if (int rc = check_ptrs({x, w->w_q, w->w_k, w->w_v, w->w_o, w->w_in, w->w_out, sv->q, sv->k, sv->v,
                           sv->ctx, sv->lse, sv->u, sv->a, z}, "mtf_layer_fwd buffer"))
    return rc;
  if (!workspace || workspace_bytes < mtf_layer_fwd_workspace_bytes(d) || !aligned16(workspace))
    return fail(MTF_ERR_WORKSPACE, "mtf_layer_fwd needs %zu bytes", mtf_layer_fwd_workspace_bytes(d));
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t count = d->batch * d->length * d->d_model;
  // u = x + R(MHA(x)); R = the Allreduce point, identity for a one-slice group
  if (int rc = mha_fwd(&m, x, w->w_q, w->w_k, w->w_v, w->w_o, scale, causal, sv->q, sv->k, sv->v, sv->ctx,
                       sv->lse, workspace, s))
    return rc;
  if (int rc = residual_add(workspace, x, sv->u, count, s)) return rc;
  // z = u + R(FFN(u))
  if (int rc = ffn_fwd(&f, sv->u, w->w_in, w->w_out, sv->a, workspace, s)) return rc;
  return residual_add(workspace, sv->u, z, count, s);
}

size_t mtf_layer_bwd_workspace_bytes(const mtf_layer_dims* d) {
  mtf_ffn_dims f;
  mtf_mha_dims m;
  if (!d || d->batch <= 0 || d->length <= 0 || d->d_model <= 0 || d->heads <= 0 || d->d_k <= 0 || d->d_ff <= 0)
    return 0;
  f = mtf_ffn_dims{d->batch, d->length, d->d_model, d->d_ff};
  m = mtf_mha_dims{d->batch, d->length, d->d_model, d->heads, d->d_k};
  const size_t partial = round256((size_t)d->batch * d->length * d->d_model * 4);
  const size_t du = round256((size_t)d->batch * d->length * d->d_model * 2);
  return partial + du + std::max(mtf_ffn_bwd_workspace_bytes(&f), mtf_mha_bwd_workspace_bytes(&m));
}

int mtf_layer_bwd(const mtf_layer_dims* d, const void* x, const mtf_layer_weights* w,
                  const mtf_layer_saved* sv, const void* dz, float scale, int causal,
                  const mtf_layer_grads* g, void* dx, void* workspace, size_t workspace_bytes,
                  void* stream) {
  mtf_ffn_dims f;
  mtf_mha_dims m;
  if (int rc = check_layer(d, &f, &m)) return rc;
  if (!w || !sv || !g) return fail(MTF_ERR_NULL, "weights / saved / grads");
  if (int rc = check_ptrs({x, w->w_q, w->w_k, w->w_v, w->w_o, w->w_in, w->w_out, sv->q, sv->k, sv->v,
                           sv->ctx, sv->lse, sv->u, sv->a, dz, g->dw_q, g->dw_k, g->dw_v, g->dw_o, g->dw_in,
                           g->dw_out, dx}, "mtf_layer_bwd buffer"))
    return rc;
  if (!workspace || workspace_bytes < mtf_layer_bwd_workspace_bytes(d) || !aligned16(workspace))
    return fail(MTF_ERR_WORKSPACE, "mtf_layer_bwd needs %zu bytes", mtf_layer_bwd_workspace_bytes(d));
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t count = d->batch * d->length * d->d_model;
  char* p = static_cast<char*>(workspace);
  void* partial = p;
  void* du = p + round256((size_t)count * 4);
  void* rest = p + round256((size_t)count * 4) + round256((size_t)count * 2);
  // FFN sublayer: du = dz + R(dx_ffn_partial)
  if (int rc = ffn_bwd(&f, sv->u, sv->a, w->w_in, w->w_out, dz, g->dw_in, g->dw_out, partial, rest, s)) return rc;
  if (int rc = residual_add(partial, dz, du, count, s)) return rc;
  // attention sublayer: dx = du + R(dx_mha_partial)
  if (int rc = mha_bwd(&m, x, w->w_q, w->w_k, w->w_v, w->w_o, sv->q, sv->k, sv->v, sv->ctx, sv->lse, du, scale,
                       causal, g->dw_q, g->dw_k, g->dw_v, g->dw_o, partial, mha_bwd_scratch(&m, rest), s))
    return rc;
  return residual_add(partial, du, dx, count, s);
}

}  // extern "C"
