// mtf_einsum_local: one processor's local einsum on its slices (section "Operation
// Implementation", einsum paragraph).  The named dims are canonicalised on the host into loop
// roles; bf16 contractions that fold to a (batched) matrix product go to the MFMA GEMM, every
// other legal request runs on a generic fp32-FMA kernel (one thread per output element).
#include "device_common.h"
#include "gemm_bf16.h"
#include "timing.h"

namespace mtf {

namespace {

constexpr int kMaxLoops = 2 * MTF_MAX_RANK;

struct GenericArgs {
  int n_out, n_red;
  int64_t out_extent[kMaxLoops], out_sa[kMaxLoops], out_sb[kMaxLoops];  // OUT's dims, row-major
  int64_t red_extent[kMaxLoops], red_sa[kMaxLoops], red_sb[kMaxLoops];  // summed-out dims
  int64_t out_elems, red_points;
  int64_t bias_extent;  // > 0: aux is a bias over OUT's innermost dim (that many values)
  float alpha;
  int accumulate, epi, has_b;
};

template <typename InT>
__device__ __forceinline__ float load_in(const InT* p, int64_t i);
template <>
__device__ __forceinline__ float load_in<float>(const float* p, int64_t i) { return p[i]; }
template <>
__device__ __forceinline__ float load_in<bf16_t>(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }

// out[o] = epilogue(alpha * sum_r a[..] * b[..] (+ out[o])): the definition, one thread per o,
// reduced dims visited in a fixed (row-major) order.
template <typename InT, typename OutT>
__global__ void __launch_bounds__(256) einsum_generic_kernel(const InT* __restrict__ a,
                                                            const InT* __restrict__ b,
                                                            OutT* __restrict__ out,
                                                            const InT* __restrict__ aux,
                                                            GenericArgs g) {
  for (int64_t o = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; o < g.out_elems;
       o += (int64_t)gridDim.x * blockDim.x) {
    int64_t rem = o, base_a = 0, base_b = 0;
    for (int d = g.n_out - 1; d >= 0; --d) {
      const int64_t i = rem % g.out_extent[d];
      rem /= g.out_extent[d];
      base_a += i * g.out_sa[d];
      base_b += i * g.out_sb[d];
    }
    float acc = 0.f;
    int64_t idx[kMaxLoops];
    for (int d = 0; d < g.n_red; ++d) idx[d] = 0;
    int64_t oa = base_a, ob = base_b;
    for (int64_t r = 0; r < g.red_points; ++r) {
      const float av = load_in<InT>(a, oa);
      const float bv = g.has_b ? load_in<InT>(b, ob) : 1.f;
      acc = fmaf(av, bv, acc);
      for (int d = g.n_red - 1; d >= 0; --d) {  // odometer over the reduced dims
        oa += g.red_sa[d];
        ob += g.red_sb[d];
        if (++idx[d] < g.red_extent[d]) break;
        oa -= idx[d] * g.red_sa[d];
        ob -= idx[d] * g.red_sb[d];
        idx[d] = 0;
      }
    }
    float v = g.alpha * acc;
    if (g.accumulate) v += sizeof(OutT) == 2 ? bf16_to_f32((bf16_t)out[o]) : (float)out[o];
    if (g.bias_extent > 0) v += load_in<InT>(aux, o % g.bias_extent);
    if (g.epi == MTF_EPI_RELU) v = fmaxf(v, 0.f);
    if (g.epi == MTF_EPI_MASK_GT0) v = load_in<InT>(aux, o) > 0.f ? v : 0.f;
    if (sizeof(OutT) == 2)
      out[o] = (OutT)f32_to_bf16(v);
    else
      out[o] = (OutT)v;
  }
}

// Component-wise operation on one tensor (section "Operation Implementation", component-wise
// paragraph: same dims in and out, purely local): out = epilogue(alpha * a (+ out)).  8 elements
// per thread, 16-byte accesses; HBM-bound.
template <typename InT, typename OutT>
__global__ void __launch_bounds__(256) componentwise_kernel(const InT* __restrict__ a, OutT* __restrict__ out,
                                                           const InT* __restrict__ aux, int64_t count, float alpha,
                                                           int accumulate, int epi) {
  auto load8 = [](const void* p, int64_t i, bool bf16, float* v) {
    if (bf16) {
      const uint4 w = *reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(p) + i);
      const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[2 * e] = __uint_as_float(u[e] << 16);
        v[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
      }
    } else {
      const float4 lo = *reinterpret_cast<const float4*>(static_cast<const float*>(p) + i);
      const float4 hi = *reinterpret_cast<const float4*>(static_cast<const float*>(p) + i + 4);
      v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
      v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    }
  };
  for (int64_t i = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) * 8; i < count;
       i += (int64_t)gridDim.x * blockDim.x * 8) {
    float v[8], m[8], o[8];
    load8(a, i, sizeof(InT) == 2, v);
    if (epi == MTF_EPI_MASK_GT0) load8(aux, i, sizeof(InT) == 2, m);
    if (accumulate) load8(out, i, sizeof(OutT) == 2, o);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float r = alpha * v[e];
      if (accumulate) r += o[e];
      if (epi == MTF_EPI_RELU) r = fmaxf(r, 0.f);
      if (epi == MTF_EPI_MASK_GT0) r = m[e] > 0.f ? r : 0.f;
      v[e] = r;
    }
    if (sizeof(OutT) == 2) {
      *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(out) + i) =
          make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
    } else {
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + i) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + i + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
  }
}

// True when the one-operand einsum keeps every dim in place: a component-wise operation.
bool is_componentwise(const Dims& da, const Dims& dout, int epi, int64_t* count) {
  if (da.rank != dout.rank) return false;
  int64_t n = 1;
  for (int i = 0; i < da.rank; ++i) {
    if (!same(da.name[i], dout.name[i])) return false;
    n *= da.size[i];
  }
  *count = n;
  return n % 8 == 0 && (epi == MTF_EPI_NONE || epi == MTF_EPI_RELU || epi == MTF_EPI_MASK_GT0);
}

int launch_componentwise(const void* a, void* out, int64_t count, mtf_dtype in_dt, mtf_dtype out_dt, int epi,
                         const void* aux, float alpha, int accumulate, hipStream_t stream) {
  const int blocks = (int)std::min<int64_t>(ceil_div(count / 8, 256), 256 * 16);
  const double bytes = (double)count * ((in_dt == MTF_BF16 ? 2 : 4) * (epi == MTF_EPI_MASK_GT0 ? 2 : 1) +
                                        (out_dt == MTF_BF16 ? 2 : 4) * (accumulate ? 2 : 1));
  LaunchTimer timer("componentwise_kernel", 0, bytes, stream);
  if (in_dt == MTF_F32 && out_dt == MTF_F32)
    componentwise_kernel<float, float><<<blocks, 256, 0, stream>>>((const float*)a, (float*)out, (const float*)aux,
                                                                 count, alpha, accumulate, epi);
  else if (in_dt == MTF_F32)
    componentwise_kernel<float, bf16_t><<<blocks, 256, 0, stream>>>((const float*)a, (bf16_t*)out, (const float*)aux,
                                                                  count, alpha, accumulate, epi);
  else if (out_dt == MTF_F32)
    componentwise_kernel<bf16_t, float><<<blocks, 256, 0, stream>>>((const bf16_t*)a, (float*)out, (const bf16_t*)aux,
                                                                  count, alpha, accumulate, epi);
  else
    componentwise_kernel<bf16_t, bf16_t><<<blocks, 256, 0, stream>>>((const bf16_t*)a, (bf16_t*)out,
                                                                   (const bf16_t*)aux, count, alpha, accumulate, epi);
  return launch_status("componentwise_kernel");
}

int launch_generic(const void* a, const Dims& da, const void* b, const Dims* db, void* out,
                   const Dims& dout, mtf_dtype in_dt, mtf_dtype out_dt, int epi, const void* aux,
                   float alpha, int accumulate, hipStream_t stream) {
  GenericArgs g;
  Dims empty;
  const Dims& dbb = db ? *db : empty;
  auto strides = [](const Dims& d, int64_t* s) {
    int64_t acc = 1;
    for (int i = d.rank - 1; i >= 0; --i) {
      s[i] = acc;
      acc *= d.size[i];
    }
  };
  int64_t sa[MTF_MAX_RANK], sb[MTF_MAX_RANK];
  strides(da, sa);
  strides(dbb, sb);
  g.n_out = dout.rank;
  g.out_elems = 1;
  for (int i = 0; i < dout.rank; ++i) {
    int ia = find(da, dout.name[i]), ib = find(dbb, dout.name[i]);
    g.out_extent[i] = dout.size[i];
    g.out_sa[i] = ia >= 0 ? sa[ia] : 0;
    g.out_sb[i] = ib >= 0 ? sb[ib] : 0;
    g.out_elems *= dout.size[i];
  }
  g.n_red = 0;
  g.red_points = 1;
  auto add_red = [&](const char* nm, int64_t extent) {
    int ia = find(da, nm), ib = find(dbb, nm);
    g.red_extent[g.n_red] = extent;
    g.red_sa[g.n_red] = ia >= 0 ? sa[ia] : 0;
    g.red_sb[g.n_red] = ib >= 0 ? sb[ib] : 0;
    g.red_points *= extent;
    ++g.n_red;
  };
  for (int i = 0; i < da.rank; ++i)
    if (find(dout, da.name[i]) < 0) add_red(da.name[i], da.size[i]);
  for (int i = 0; i < dbb.rank; ++i)
    if (find(dout, dbb.name[i]) < 0 && find(da, dbb.name[i]) < 0) add_red(dbb.name[i], dbb.size[i]);
  g.alpha = alpha;
  g.accumulate = accumulate;
  g.bias_extent = 0;
  if (epi == MTF_EPI_BIAS || epi == MTF_EPI_BIAS_RELU) {
    g.bias_extent = dout.rank ? dout.size[dout.rank - 1] : 1;
    epi = epi == MTF_EPI_BIAS_RELU ? MTF_EPI_RELU : MTF_EPI_NONE;
  }
  g.epi = epi;
  g.has_b = db ? 1 : 0;
  const int blocks = (int)std::min<int64_t>(ceil_div(g.out_elems, 256), 256 * 32);
  LaunchTimer timer("einsum_generic_kernel", 2.0 * g.out_elems * g.red_points, 0, stream);
  if (in_dt == MTF_F32 && out_dt == MTF_F32)
    einsum_generic_kernel<float, float><<<blocks, 256, 0, stream>>>(
        (const float*)a, (const float*)b, (float*)out, (const float*)aux, g);
  else if (in_dt == MTF_F32)
    einsum_generic_kernel<float, bf16_t><<<blocks, 256, 0, stream>>>(
        (const float*)a, (const float*)b, (bf16_t*)out, (const float*)aux, g);
  else if (out_dt == MTF_F32)
    einsum_generic_kernel<bf16_t, float><<<blocks, 256, 0, stream>>>(
        (const bf16_t*)a, (const bf16_t*)b, (float*)out, (const bf16_t*)aux, g);
  else
    einsum_generic_kernel<bf16_t, bf16_t><<<blocks, 256, 0, stream>>>(
        (const bf16_t*)a, (const bf16_t*)b, (bf16_t*)out, (const bf16_t*)aux, g);
  return launch_status("einsum_generic_kernel");
}

// Tries to express the canonical einsum as the batched GEMM of gemm_bf16.h.  Returns false when
// the loop structure does not fold (then the generic kernel runs).
bool as_gemm(const Canon& c, GemmDesc* d, bool* swapped) {
  if (c.n[R_RA] || c.n[R_RB]) return false;                       // one-sided reductions
  if (c.n[R_M] > 1 || c.n[R_N] > 1 || c.n[R_K] > 1) return false;  // non-foldable groups
  if (c.n[R_BATCH] > 2 || c.n[R_K] == 0) return false;
  Loop m = c.n[R_M] ? c.loop[R_M][0] : Loop{1, 0, 0, 0};
  Loop n = c.n[R_N] ? c.loop[R_N][0] : Loop{1, 0, 0, 0};
  const Loop k = c.loop[R_K][0];
  bool swap = false;
  if (c.n[R_N] && n.so == 1) {
    swap = false;
  } else if (c.n[R_M] && m.so == 1) {
    swap = true;  // OUT has m innermost: compute OUT^T = B^T A^T, i.e. exchange the operands
  } else {
    return false;  // neither an m nor an n dim is innermost in OUT
  }
  *swapped = swap;
  // after the (possible) exchange: "row" operand carries m, "col" operand carries n
  Loop row = swap ? n : m, col = swap ? m : n;
  const int64_t row_s = swap ? row.sb : row.sa;   // stride of the row index in its operand
  const int64_t col_s = swap ? col.sa : col.sb;
  const int64_t rk_s = swap ? k.sb : k.sa;        // k stride in the row operand
  const int64_t ck_s = swap ? k.sa : k.sb;
  if (col.so != 1 && col.extent != 1) return false;
  d->M = row.extent;
  d->N = col.extent;
  d->nseg = 1;
  d->K[0] = k.extent;
  if (rk_s == 1) {
    d->a_kcontig = true;
    d->lda = row.extent == 1 ? k.extent : row_s;
  } else if (row_s == 1 || row.extent == 1) {
    d->a_kcontig = false;
    d->lda = rk_s;
  } else {
    return false;
  }
  if (ck_s == 1) {
    d->b_kcontig = true;
    d->ldb = col.extent == 1 ? k.extent : col_s;
  } else if (col_s == 1 || col.extent == 1) {
    d->b_kcontig = false;
    d->ldb = ck_s;
  } else {
    return false;
  }
  d->ldc = row.extent == 1 ? col.extent : row.so;
  d->batch0 = d->batch1 = 1;
  for (int i = 0; i < c.n[R_BATCH]; ++i) {
    const Loop& bl = c.loop[R_BATCH][i];
    int64_t sa = swap ? bl.sb : bl.sa, sb = swap ? bl.sa : bl.sb;
    if (c.n[R_BATCH] == 2 && i == 0) {
      d->batch0 = bl.extent; d->sA0 = sa; d->sB0 = sb; d->sC0 = bl.so;
    } else {
      d->batch1 = bl.extent; d->sA1 = sa; d->sB1 = sb; d->sC1 = bl.so;
    }
  }
  d->A[0] = nullptr;  // filled by the caller (depends on swap)
  return true;
}

}  // namespace

}  // namespace mtf

using namespace mtf;

namespace {

// Validation and kernel choice shared by mtf_einsum_local and mtf_einsum_local_path.
struct EinsumRoute {
  Dims da, db, dout;
  bool has_b = false;
  bool use_gemm = false;
  GemmDesc gemm;
};

int route_einsum(const void* a, const mtf_shape* a_local, const void* b, const mtf_shape* b_local, void* out,
                 const mtf_shape* out_local, mtf_dtype in_dt, mtf_dtype out_dt, mtf_epilogue epi, const void* aux,
                 float alpha, int accumulate, EinsumRoute* r) {
  if (int rc = load_shape(a_local, "a", &r->da)) return rc;
  r->has_b = b != nullptr || b_local != nullptr;
  if (r->has_b) {
    if (!b || !b_local) return fail(MTF_ERR_NULL, "b given without its shape (or the reverse)");
    if (int rc = load_shape(b_local, "b", &r->db)) return rc;
  }
  if (int rc = load_shape(out_local, "output", &r->dout)) return rc;
  if (!a || !out) return fail(MTF_ERR_NULL, "a / out");
  if ((in_dt != MTF_F32 && in_dt != MTF_BF16) || (out_dt != MTF_F32 && out_dt != MTF_BF16))
    return fail(MTF_ERR_UNSUPPORTED, "dtype");
  const bool with_bias = epi == MTF_EPI_BIAS || epi == MTF_EPI_BIAS_RELU;
  if (epi != MTF_EPI_NONE && epi != MTF_EPI_RELU && epi != MTF_EPI_MASK_GT0 && !with_bias)
    return fail(MTF_ERR_UNSUPPORTED, "epilogue %d", (int)epi);
  if ((epi == MTF_EPI_MASK_GT0 || with_bias) && !aux) return fail(MTF_ERR_NULL, "aux for this epilogue");
  if (!aligned16(a) || !aligned16(b) || !aligned16(out) || !aligned16(aux))
    return fail(MTF_ERR_ALIGN, "a / b / out / aux");
  Canon c;
  if (int rc = canonicalize(r->da, r->has_b ? &r->db : nullptr, r->dout, &c)) return rc;
  if (in_dt == MTF_BF16 && r->has_b) {
    GemmDesc& d = r->gemm;
    bool swapped = false;
    if (as_gemm(c, &d, &swapped)) {  // exchanges the operands when OUT has A's dims innermost
      d.A[0] = static_cast<const bf16_t*>(swapped ? b : a);
      d.B[0] = static_cast<const bf16_t*>(swapped ? a : b);
      d.C = out;
      d.out_bf16 = out_dt == MTF_BF16;
      d.epi = with_bias ? (epi == MTF_EPI_BIAS_RELU ? MTF_EPI_RELU : MTF_EPI_NONE) : epi;
      d.aux = with_bias ? nullptr : static_cast<const bf16_t*>(aux);
      // the bias runs over OUT's innermost dim: a plain n-vector unless that dim was merged
      // with the one before it
      d.bias = with_bias ? static_cast<const bf16_t*>(aux) : nullptr;
      const bool bias_ok = !with_bias || (r->dout.rank > 0 && d.N == r->dout.size[r->dout.rank - 1]);
      d.alpha = alpha;
      d.accumulate = accumulate != 0;
      r->use_gemm = bias_ok && gemm_bf16_supported(d);
    }
  }
  return MTF_OK;
}

}  // namespace

extern "C" int mtf_einsum_local(const void* a, const mtf_shape* a_local, const void* b,
                                const mtf_shape* b_local, void* out, const mtf_shape* out_local,
                                mtf_dtype in_dt, mtf_dtype out_dt, mtf_epilogue epi,
                                const void* aux, float alpha, int accumulate, void* stream) {
  EinsumRoute r;
  if (int rc = route_einsum(a, a_local, b, b_local, out, out_local, in_dt, out_dt, epi, aux, alpha, accumulate, &r))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (r.use_gemm) return gemm_bf16_launch(r.gemm, s);
  int64_t count = 0;
  if (!r.has_b && is_componentwise(r.da, r.dout, epi, &count))
    return launch_componentwise(a, out, count, in_dt, out_dt, epi, aux, alpha, accumulate, s);
  return launch_generic(a, r.da, r.has_b ? b : nullptr, r.has_b ? &r.db : nullptr, out, r.dout, in_dt, out_dt,
                        epi, aux, alpha, accumulate, s);
}

extern "C" int mtf_einsum_local_kranges(const void* a, const mtf_shape* a_local, const void* b,
                                        const mtf_shape* b_local, void* const* outs, int32_t n,
                                        const mtf_shape* out_local, void* stream) {
  if (!outs) return fail(MTF_ERR_NULL, "outs");
  if (n < 1 || n > kMaxGroup) return fail(MTF_ERR_UNSUPPORTED, "%d ranges (1..%d)", n, kMaxGroup);
  for (int i = 0; i < n; ++i) {
    if (!outs[i]) return fail(MTF_ERR_NULL, "out %d", i);
    if (!aligned16(outs[i])) return fail(MTF_ERR_ALIGN, "out %d", i);
  }
  EinsumRoute r;
  if (int rc = route_einsum(a, a_local, b, b_local, outs[0], out_local, MTF_BF16, MTF_F32, MTF_EPI_NONE, nullptr,
                            1.f, 0, &r))
    return rc;
  GemmDesc& d = r.gemm;
  if (!r.use_gemm || d.batch0 * d.batch1 != 1)
    return fail(MTF_ERR_UNSUPPORTED, "not a plain matrix product of bf16 operands");
  const int64_t K = d.K[0];
  if (K % (8 * (int64_t)n)) return fail(MTF_ERR_UNSUPPORTED, "contracted size %lld not divisible by 8 x %d", (long long)K, n);
  const int64_t kr = K / n;
  const bf16_t *a0 = d.A[0], *b0 = d.B[0];
  d.K[0] = kr;
  for (int i = 1; i < n; ++i) {
    GemmDesc::Extra& e = d.extra[d.nextra++];
    e.A[0] = a0 + (d.a_kcontig ? i * kr : i * kr * d.lda);
    e.B[0] = b0 + (d.b_kcontig ? i * kr : i * kr * d.ldb);
    e.K[0] = kr;
    e.C = outs[i];
    e.M = d.M; e.N = d.N;
    e.lda = d.lda; e.ldb = d.ldb; e.ldc = d.ldc;
  }
  return gemm_bf16_launch(d, static_cast<hipStream_t>(stream));
}

extern "C" int mtf_einsum_local_path(const void* a, const mtf_shape* a_local, const void* b,
                                     const mtf_shape* b_local, void* out, const mtf_shape* out_local,
                                     mtf_dtype in_dt, mtf_dtype out_dt, mtf_epilogue epi,
                                     const void* aux, float alpha, int accumulate) {
  EinsumRoute r;
  if (int rc = route_einsum(a, a_local, b, b_local, out, out_local, in_dt, out_dt, epi, aux, alpha, accumulate, &r))
    return rc;
  int64_t count = 0;
  if (r.use_gemm) return MTF_PATH_MFMA;
  return !r.has_b && is_componentwise(r.da, r.dout, epi, &count) ? MTF_PATH_COMPONENTWISE : MTF_PATH_GENERIC;
}
