// Fixed per-processor layer steps: sequences of the local einsums of the model-parallel
// Transformer layout (d_ff and heads split; section 'Model-Parallel "Transformer"'), each lowered
// to the bf16 MFMA GEMM, plus the fused attention kernels.  Outputs that contract a split dim
// (y, dx) are PARTIAL sums in fp32, ready for the Allreduce of the einsum lowering.
#include "attention.h"
#include "device_common.h"
#include "gemm_bf16.h"
#include "reduce_local.h"

namespace mtf {
namespace {

inline size_t round256(size_t n) { return (n + 255) & ~size_t(255); }

constexpr int kLayerPartials = 2;  // fp32 partial-sum buffers a layer step keeps in its workspace

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

// Appends problem `p` (one segment, same layouts / dtype as the group) to a grouped launch.
void add_to_group(GemmDesc* group, const GemmDesc& p) {
  GemmDesc::Extra& e = group->extra[group->nextra++];
  for (int s = 0; s < kMaxSegments; ++s) {
    e.A[s] = p.A[s]; e.B[s] = p.B[s]; e.K[s] = p.K[s];
  }
  e.C = p.C;
  e.M = p.M; e.N = p.N;
  e.lda = p.lda; e.ldb = p.ldb; e.ldc = p.ldc;
}

// Destination of an einsum whose result is wanted as a sum anyway (a partial sum on its way to
// the Allreduce / residual add): n >= 1 fp32 buffers whose sum is the result.  With n > 1 the
// contracted dim is cut into n ranges that run as one grouped launch - on this one GPU the same
// thing the layout does across processors when it splits a reduced-out dim.
struct Partials {
  void* buf[kMaxGroup];
  int n;
};

// C = A op B with K cut into parts.n equal ranges (K % (8 * n) == 0 required), range i -> buf[i].
int gemm_k_split(const void* A, bool a_kc, const void* B, bool b_kc, const Partials& parts, int64_t M,
                 int64_t N, int64_t K, hipStream_t s) {
  const int n = (parts.n > 1 && K % (8 * parts.n) == 0) ? parts.n : 1;
  const int64_t kr = K / n;
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* b = static_cast<const bf16_t*>(B);
  GemmDesc g = gemm(a, a_kc, b, b_kc, parts.buf[0], false, M, N, kr);
  g.lda = a_kc ? K : M;
  g.ldb = b_kc ? K : N;
  for (int i = 1; i < n; ++i) {
    GemmDesc p = gemm(a + (a_kc ? i * kr : i * kr * M), a_kc, b + (b_kc ? i * kr : i * kr * N), b_kc,
                      parts.buf[i], false, M, N, kr);
    p.lda = g.lda;
    p.ldb = g.ldb;
    add_to_group(&g, p);
  }
  if (int rc = gemm_bf16_launch(g, s)) return rc;
  return n;  // number of buffers actually written (positive)
}

// One contraction whose reduced dim runs through `npairs` operand pairs in turn (A_i [M,K] and
// B_i [N,K], both k-contiguous, K elements each), cut into parts.n equal ranges of that
// concatenated axis: range i -> buf[i], all ranges in one grouped launch.  A range that crosses
// a pair boundary has one segment per pair it touches.  Returns the number of buffers written, or
// 0 when the sizes do not allow the cut (nothing launched), or a negative error.
int gemm_pairs_k_split(const bf16_t* const* A, const bf16_t* const* B, int npairs, int64_t K,
                       const Partials& parts, int64_t M, int64_t N, hipStream_t s) {
  const int n = parts.n;
  const int64_t total = K * npairs;
  if (n < 1 || n > kMaxGroup || total % (8 * n) || K % 8) return 0;
  const int64_t kr = total / n;
  GemmDesc range[kMaxGroup];
  int nseg = 1;
  for (int i = 0; i < n; ++i) {
    GemmDesc& g = range[i];
    g = gemm(nullptr, true, nullptr, true, parts.buf[i], false, M, N, 0);
    g.lda = g.ldb = K;
    int seg = 0;
    for (int64_t k0 = i * kr; k0 < (i + 1) * kr;) {
      const int pair = (int)(k0 / K);
      const int64_t in_pair = k0 % K, len = std::min(K - in_pair, (i + 1) * kr - k0);
      if (seg == kMaxSegments) return 0;
      g.A[seg] = A[pair] + in_pair;
      g.B[seg] = B[pair] + in_pair;
      g.K[seg++] = len;
      k0 += len;
    }
    nseg = std::max(nseg, seg);
  }
  if (n * nseg > kMaxSlots) return 0;
  for (int i = 0; i < n; ++i) {  // unused segments: K = 0, pointers valid
    for (int q = 0; q < nseg; ++q)
      if (!range[i].A[q]) { range[i].A[q] = range[i].A[0]; range[i].B[q] = range[i].B[0]; }
    range[i].nseg = nseg;
    if (i > 0) add_to_group(&range[0], range[i]);
  }
  if (int rc = gemm_bf16_launch(range[0], s)) return rc;
  return n;
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
  if (!attn_fused_width(d->d_k))
    return fail(MTF_ERR_UNSUPPORTED, "the attention step needs d_k = d_v = 128 or 256, not %lld", (long long)d->d_k);
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

// Returns the number of buffers of `y` written (their sum is y_partial), or a negative error.
// `bias` (or nullptr): bias[F] added before the ReLU.
int ffn_fwd(const mtf_ffn_dims* d, const void* x, const void* w_in, const void* bias, const void* w_out,
            void* a, const Partials& y, hipStream_t s) {
  const int64_t T = d->batch * d->length, D = d->d_model, F = d->d_ff;
  // a = relu(einsum(x[b,l,D], w_in[D,F] -> [b,l,F]) [+ bias[F]])
  GemmDesc g1 = gemm(x, true, w_in, false, a, true, T, F, D);
  g1.epi = MTF_EPI_RELU;
  g1.bias = static_cast<const bf16_t*>(bias);
  if (int rc = gemm_bf16_launch(g1, s)) return rc;
  // y_partial = einsum(a[b,l,F], w_out[F,D] -> [b,l,D]); F is the split, reduced-out dim
  return gemm_k_split(a, true, w_out, false, y, T, D, F, s);
}

// `dbias` (or nullptr): dbias[F] = sum of dh over the tokens, using `red_ws`.
int ffn_bwd(const mtf_ffn_dims* d, const void* x, const void* a, const void* w_in, const void* w_out,
            const void* dy, void* dw_in, void* dw_out, const Partials& dx, void* dh, hipStream_t s,
            void* dbias = nullptr, void* red_ws = nullptr, size_t red_ws_bytes = 0) {
  const int64_t T = d->batch * d->length, D = d->d_model, F = d->d_ff;
  // dh = einsum(dy[b,l,D], w_out[F,D] -> [b,l,F]) * [a > 0]
  GemmDesc g = gemm(dy, true, w_out, true, dh, true, T, F, D);
  g.epi = MTF_EPI_MASK_GT0;
  g.aux = static_cast<const bf16_t*>(a);
  if (int rc = gemm_bf16_launch(g, s)) return rc;
  // dbias = reduce_sum(dh[b,l,F] -> [F])
  if (dbias)
    if (int rc = reduce_cols_sum(static_cast<const bf16_t*>(dh), static_cast<float*>(dbias), T, F, red_ws,
                                 red_ws_bytes, s))
      return rc;
  // dw_out = einsum(a[b,l,F], dy[b,l,D] -> [F,D]) and dw_in = einsum(x[b,l,D], dh[b,l,F] -> [D,F]):
  // two outputs of D * F elements that each reduce out the token dims.  Alone, either has too few
  // large tiles for the machine; as one grouped launch they fill it.
  GemmDesc dw = gemm(a, false, dy, false, dw_out, false, F, D, T);
  add_to_group(&dw, gemm(x, false, dh, false, dw_in, false, D, F, T));
  if (int rc = gemm_bf16_launch(dw, s)) return rc;
  // dx_partial = einsum(dh[b,l,F], w_in[D,F] -> [b,l,D])
  return gemm_k_split(dh, true, w_in, true, dx, T, D, F, s);
}

int mha_fwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k, const void* w_v,
            const void* w_o, float scale, int causal, void* q, void* k, void* v, void* ctx, void* lse,
            const Partials& y, hipStream_t s) {
  const int64_t T = d->batch * d->length, D = d->d_model, HK = d->heads * d->d_k;
  // q, k, v = einsum(x[b,l,D], w[D,h,k] -> [b,l,h,k]); D is not split: complete local slices.
  // Three independent einsums with one shared operand: one grouped launch.
  GemmDesc qkv = gemm(x, true, w_q, false, q, true, T, HK, D);
  add_to_group(&qkv, gemm(x, true, w_k, false, k, true, T, HK, D));
  add_to_group(&qkv, gemm(x, true, w_v, false, v, true, T, HK, D));
  if (int rc = gemm_bf16_launch(qkv, s)) return rc;
  AttnShape as{(int)d->batch, (int)d->length, (int)d->heads, (int)d->d_k, scale, causal};
  if (int rc = attn_fwd_launch(as, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)ctx,
                               (float*)lse, s))
    return rc;
  // y_partial = einsum(ctx[b,l,h,v], w_o[h,v,D] -> [b,l,D]); heads is the split, reduced-out dim
  return gemm_k_split(ctx, true, w_o, false, y, T, D, HK, s);
}

int mha_bwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k, const void* w_v,
            const void* w_o, const void* q, const void* k, const void* v, const void* ctx,
            const void* lse, const void* dy, float scale, int causal, void* dw_q, void* dw_k,
            void* dw_v, void* dw_o, const Partials& dx, const MhaBwdScratch& w, hipStream_t s) {
  const int64_t T = d->batch * d->length, D = d->d_model, HK = d->heads * d->d_k;
  // dctx = einsum(dy[b,l,D], w_o[h,v,D] -> [b,l,h,v])
  if (int rc = gemm_bf16_launch(gemm(dy, true, w_o, true, w.dctx, true, T, HK, D), s)) return rc;
  AttnShape as{(int)d->batch, (int)d->length, (int)d->heads, (int)d->d_k, scale, causal};
  if (int rc = attn_bwd_launch(as, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v,
                               (const bf16_t*)ctx, (const float*)lse, w.dctx, w.dq, w.dk, w.dv, w.delta, s))
    return rc;
  // dw_o = einsum(ctx[b,l,h,v], dy[b,l,D] -> [h,v,D]) and
  // dw_{q,k,v} = einsum(x[b,l,D], d{q,k,v}[b,l,h,k] -> [D,h,k]): four small outputs that each
  // reduce out the (long) token dims; launched as one group so that together they fill the CUs
  GemmDesc dw = gemm(ctx, false, dy, false, dw_o, false, HK, D, T);
  add_to_group(&dw, gemm(x, false, w.dq, false, dw_q, false, D, HK, T));
  add_to_group(&dw, gemm(x, false, w.dk, false, dw_k, false, D, HK, T));
  add_to_group(&dw, gemm(x, false, w.dv, false, dw_v, false, D, HK, T));
  if (int rc = gemm_bf16_launch(dw, s)) return rc;
  // dx_partial = sum over {q,k,v} of einsum(d*[b,l,h,k], w_*[D,h,k] -> [b,l,D]): one contraction
  // whose reduced dims (h,k) are spread over three tensor pairs
  if (dx.n > 1) {  // the (h,k) axis of all three pairs, end to end, cut into dx.n equal ranges
    const bf16_t* as[3] = {w.dq, w.dk, w.dv};
    const bf16_t* bs[3] = {static_cast<const bf16_t*>(w_q), static_cast<const bf16_t*>(w_k),
                           static_cast<const bf16_t*>(w_v)};
    if (int n = gemm_pairs_k_split(as, bs, 3, HK, dx, T, D, s)) return n;
  }
  GemmDesc g = gemm(w.dq, true, w_q, true, dx.buf[0], false, T, D, HK);
  g.nseg = 3;  // one output: the three (A, B) pairs are consecutive ranges of one reduction
  g.A[1] = w.dk; g.B[1] = static_cast<const bf16_t*>(w_k); g.K[1] = HK;
  g.A[2] = w.dv; g.B[2] = static_cast<const bf16_t*>(w_v); g.K[2] = HK;
  if (int rc = gemm_bf16_launch(g, s)) return rc;
  return 1;
}

// out = residual + sum of the first n buffers of `parts` (bf16 out): the Allreduce point of a
// one-slice group followed by the residual add.
int residual_add(const Partials& parts, int n, const void* residual_bf16, void* out_bf16, int64_t count,
                 hipStream_t s) {
  return mtf_reduce_partials(parts.buf, n, residual_bf16, MTF_BF16, out_bf16, MTF_BF16, count, s);
}

Partials single(void* buf) {
  Partials p{};
  p.buf[0] = buf;
  p.n = 1;
  return p;
}

// n fp32 buffers of `count` elements carved from a workspace.
Partials carve(void* base, int n, int64_t count) {
  Partials p{};
  p.n = n;
  for (int i = 0; i < n; ++i) p.buf[i] = static_cast<char*>(base) + (size_t)i * round256((size_t)count * 4);
  return p;
}

}  // namespace
}  // namespace mtf

using namespace mtf;

extern "C" {

int mtf_ffn_fwd(const mtf_ffn_dims* d, const void* x, const void* w_in, const void* w_out, void* a,
                void* y_partial, void* stream) {
  if (int rc = check_ffn(d)) return rc;
  if (int rc = check_ptrs({x, w_in, w_out, a, y_partial}, "mtf_ffn_fwd buffer")) return rc;
  const int rc = ffn_fwd(d, x, w_in, nullptr, w_out, a, single(y_partial), static_cast<hipStream_t>(stream));
  return rc < 0 ? rc : MTF_OK;
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
  const int rc = ffn_bwd(d, x, a, w_in, w_out, dy, dw_in, dw_out, single(dx_partial), workspace,
                         static_cast<hipStream_t>(stream));
  return rc < 0 ? rc : MTF_OK;
}

int mtf_ffn_bias_fwd(const mtf_ffn_dims* d, const void* x, const void* w_in, const void* bias,
                     const void* w_out, void* a, void* y_partial, void* stream) {
  if (int rc = check_ffn(d)) return rc;
  if (int rc = check_ptrs({x, w_in, bias, w_out, a, y_partial}, "mtf_ffn_bias_fwd buffer")) return rc;
  const int rc = ffn_fwd(d, x, w_in, bias, w_out, a, single(y_partial), static_cast<hipStream_t>(stream));
  return rc < 0 ? rc : MTF_OK;
}

size_t mtf_ffn_bias_bwd_workspace_bytes(const mtf_ffn_dims* d) {
  if (!d || d->batch <= 0 || d->length <= 0 || d->d_ff <= 0) return 0;
  return mtf_ffn_bwd_workspace_bytes(d) + round256(reduce_cols_workspace_bytes(d->batch * d->length, d->d_ff));
}

int mtf_ffn_bias_bwd(const mtf_ffn_dims* d, const void* x, const void* a, const void* w_in,
                     const void* w_out, const void* dy, void* dw_in, void* dbias, void* dw_out,
                     void* dx_partial, void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_ffn(d)) return rc;
  if (int rc = check_ptrs({x, a, w_in, w_out, dy, dw_in, dbias, dw_out, dx_partial}, "mtf_ffn_bias_bwd buffer"))
    return rc;
  if (!workspace || workspace_bytes < mtf_ffn_bias_bwd_workspace_bytes(d) || !aligned16(workspace))
    return fail(MTF_ERR_WORKSPACE, "mtf_ffn_bias_bwd needs %zu bytes", mtf_ffn_bias_bwd_workspace_bytes(d));
  const size_t dh_bytes = mtf_ffn_bwd_workspace_bytes(d);
  const int rc = ffn_bwd(d, x, a, w_in, w_out, dy, dw_in, dw_out, single(dx_partial), workspace,
                         static_cast<hipStream_t>(stream), dbias, static_cast<char*>(workspace) + dh_bytes,
                         workspace_bytes - dh_bytes);
  return rc < 0 ? rc : MTF_OK;
}

int mtf_mha_fwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k,
                const void* w_v, const void* w_o, float scale, int causal, void* q, void* k,
                void* v, void* ctx, void* lse, void* y_partial, void* stream) {
  if (int rc = check_mha(d)) return rc;
  if (int rc = check_ptrs({x, w_q, w_k, w_v, w_o, q, k, v, ctx, lse, y_partial}, "mtf_mha_fwd buffer")) return rc;
  const int rc = mha_fwd(d, x, w_q, w_k, w_v, w_o, scale, causal, q, k, v, ctx, lse, single(y_partial),
                         static_cast<hipStream_t>(stream));
  return rc < 0 ? rc : MTF_OK;
}

// Ranges the attention sublayer's dx is cut into when it is called on its own (the whole-layer
// step has its own partial-sum buffers): 4 give a 2048-token shard 512 small tiles.
constexpr int kMhaDxRanges = 4;

size_t mtf_mha_bwd_workspace_bytes(const mtf_mha_dims* d) {
  if (!d || d->batch <= 0 || d->length <= 0 || d->heads <= 0 || d->d_k <= 0 || d->d_model <= 0) return 0;
  return mha_bwd_scratch(d, nullptr).bytes +
         kMhaDxRanges * round256((size_t)d->batch * d->length * d->d_model * 4);
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
  // dx as kMhaDxRanges ranges of its contracted axis (so that a small shard still fills the CUs),
  // summed into dx_partial by the reduce; shapes that cannot be cut write dx_partial directly
  const MhaBwdScratch scratch = mha_bwd_scratch(d, workspace);
  const int64_t count = d->batch * d->length * d->d_model;
  Partials parts = carve(static_cast<char*>(workspace) + scratch.bytes, kMhaDxRanges, count);
  const bool cut = (3 * d->heads * d->d_k) % (8 * kMhaDxRanges) == 0;
  if (!cut) parts = single(dx_partial);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n = mha_bwd(d, x, w_q, w_k, w_v, w_o, q, k, v, ctx, lse, dy, scale, causal, dw_q, dw_k, dw_v, dw_o,
                        parts, scratch, s);
  if (n < 0) return n;
  if (!cut) return MTF_OK;
  return mtf_reduce_partials(parts.buf, n, nullptr, MTF_F32, dx_partial, MTF_F32, count, s);
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
  return kLayerPartials * round256((size_t)d->batch * d->length * d->d_model * 4);  // fp32 partial sums
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
  // u = x + R(MHA(x)); R = the Allreduce point.  For this one-slice group it degenerates to the
  // sum of the k-range partial sums the einsum was cut into.
  const Partials parts = carve(workspace, 2, count);
  int n = mha_fwd(&m, x, w->w_q, w->w_k, w->w_v, w->w_o, scale, causal, sv->q, sv->k, sv->v, sv->ctx, sv->lse,
                  parts, s);
  if (n < 0) return n;
  if (int rc = residual_add(parts, n, x, sv->u, count, s)) return rc;
  // z = u + R(FFN(u))
  n = ffn_fwd(&f, sv->u, w->w_in, nullptr, w->w_out, sv->a, parts, s);
  if (n < 0) return n;
  return residual_add(parts, n, sv->u, z, count, s);
}

size_t mtf_layer_bwd_workspace_bytes(const mtf_layer_dims* d) {
  mtf_ffn_dims f;
  mtf_mha_dims m;
  if (!d || d->batch <= 0 || d->length <= 0 || d->d_model <= 0 || d->heads <= 0 || d->d_k <= 0 || d->d_ff <= 0)
    return 0;
  f = mtf_ffn_dims{d->batch, d->length, d->d_model, d->d_ff};
  m = mtf_mha_dims{d->batch, d->length, d->d_model, d->heads, d->d_k};
  const size_t partial = kLayerPartials * round256((size_t)d->batch * d->length * d->d_model * 4);
  const size_t du = round256((size_t)d->batch * d->length * d->d_model * 2);
  return partial + du + std::max(mtf_ffn_bwd_workspace_bytes(&f), mha_bwd_scratch(&m, nullptr).bytes);
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
  const size_t part_bytes = kLayerPartials * round256((size_t)count * 4);
  void* du = p + part_bytes;
  void* rest = p + part_bytes + round256((size_t)count * 2);
  // FFN sublayer: du = dz + R(dx_ffn_partial)
  int n = ffn_bwd(&f, sv->u, sv->a, w->w_in, w->w_out, dz, g->dw_in, g->dw_out, carve(p, 2, count), rest, s);
  if (n < 0) return n;
  if (int rc = residual_add(carve(p, 2, count), n, dz, du, count, s)) return rc;
  // attention sublayer: dx = du + R(dx_mha_partial)
  n = mha_bwd(&m, x, w->w_q, w->w_k, w->w_v, w->w_o, sv->q, sv->k, sv->v, sv->ctx, sv->lse, du, scale, causal,
              g->dw_q, g->dw_k, g->dw_v, g->dw_o, carve(p, 2, count), mha_bwd_scratch(&m, rest), s);
  if (n < 0) return n;
  return residual_add(carve(p, 2, count), n, du, dx, count, s);
}

}  // extern "C"
