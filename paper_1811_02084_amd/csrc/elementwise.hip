// HBM-bound helpers: slice gather/scatter, partial-sum reduce, dtype cast.
#include <type_traits>

#include "device_common.h"
#include "timing.h"

namespace mtf {

// ------------------------------------------------------------------------------ slice copy
// The slice is a dense box inside a dense row-major tensor ("Tensor Representations": every
// split dim keeps one contiguous stripe).  After merging dims the box has <= MTF_MAX_RANK dims;
// the innermost is copied in vectors of VEC elements.
struct BoxArgs {
  int rank;
  int64_t extent[MTF_MAX_RANK];  // box extents, innermost counted in vectors
  int64_t stride[MTF_MAX_RANK];  // element strides of the full tensor
  int64_t base;                  // element offset of the box origin in the full tensor
  int64_t vectors;               // total vectors in the box
};

template <typename VecT, int VEC_ELEMS, typename ElemT>
__global__ void __launch_bounds__(256) slice_copy_kernel(const ElemT* __restrict__ full_c,
                                                        ElemT* __restrict__ full_m,
                                                        ElemT* __restrict__ slice, BoxArgs box,
                                                        int scatter) {
  for (int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; v < box.vectors;
       v += (int64_t)gridDim.x * blockDim.x) {
    int64_t rem = v, off = box.base;
    for (int d = box.rank - 1; d >= 0; --d) {
      int64_t i = rem % box.extent[d];
      rem /= box.extent[d];
      off += i * box.stride[d] * (d == box.rank - 1 ? VEC_ELEMS : 1);
    }
    VecT* s = reinterpret_cast<VecT*>(slice + v * VEC_ELEMS);
    if (scatter)
      *reinterpret_cast<VecT*>(full_m + off) = *s;
    else
      *s = *reinterpret_cast<const VecT*>(full_c + off);
  }
}

template <typename ElemT>
static int slice_copy_typed(const void* full, void* slice, const Dims& t, const int64_t* offset,
                            const int64_t* size, int scatter, hipStream_t stream) {
  // full-tensor strides
  int64_t stride[MTF_MAX_RANK], acc = 1;
  for (int i = t.rank - 1; i >= 0; --i) {
    stride[i] = acc;
    acc *= t.size[i];
  }
  BoxArgs box;
  box.rank = 0;
  box.base = 0;
  int64_t elems = 1;
  for (int i = 0; i < t.rank; ++i) {
    box.base += offset[i] * stride[i];
    elems *= size[i];
    // merge with the previous box dim when that keeps addressing linear: the current dim must be
    // whole (not split) for its outer neighbour's stride to continue it
    if (box.rank > 0 && size[i] == t.size[i]) {
      box.extent[box.rank - 1] *= size[i];
      box.stride[box.rank - 1] = stride[i];
    } else {
      box.extent[box.rank] = size[i];
      box.stride[box.rank] = stride[i];
      ++box.rank;
    }
  }
  if (box.rank == 0) {  // rank-0 tensor: one element
    box.rank = 1;
    box.extent[0] = 1;
    box.stride[0] = 1;
  }
  if (elems == 0) return MTF_OK;
  const int kVec = 16 / (int)sizeof(ElemT);
  int64_t inner = box.extent[box.rank - 1];
  bool vec_ok = inner % kVec == 0 && box.base % kVec == 0 && aligned16(full) && aligned16(slice);
  for (int d = 0; d + 1 < box.rank; ++d) vec_ok = vec_ok && box.stride[d] % kVec == 0;
  const ElemT* fc = static_cast<const ElemT*>(full);
  ElemT* fm = scatter ? const_cast<ElemT*>(fc) : nullptr;
  LaunchTimer timer("slice_copy_kernel", 0, 2.0 * elems * sizeof(ElemT), stream);
  if (vec_ok) {
    box.extent[box.rank - 1] = inner / kVec;
    box.vectors = elems / kVec;
    int blocks = (int)std::min<int64_t>(ceil_div(box.vectors, 256), 256 * 16);
    slice_copy_kernel<uint4, kVec, ElemT><<<blocks, 256, 0, stream>>>(fc, fm, static_cast<ElemT*>(slice), box, scatter);
  } else {
    box.vectors = elems;
    int blocks = (int)std::min<int64_t>(ceil_div(box.vectors, 256), 256 * 16);
    slice_copy_kernel<ElemT, 1, ElemT><<<blocks, 256, 0, stream>>>(fc, fm, static_cast<ElemT*>(slice), box, scatter);
  }
  return launch_status("slice_copy_kernel");
}

// ------------------------------------------------------------------------------ partial-sum reduce
struct PartialPtrs {
  const float* p[64];
};

// NFIX > 0: exactly NFIX partials, their loads unrolled so that all of a thread's requests are in
// flight before the first addition; NFIX == 0: any n, one partial at a time.  A thread handles 8
// consecutive elements: two 16-byte loads per fp32 operand, one 16-byte access per bf16 operand.
template <bool RES_BF16, bool OUT_BF16, int NFIX>
__global__ void __launch_bounds__(256) reduce_partials_kernel(PartialPtrs parts, int n,
                                                             const void* __restrict__ residual,
                                                             void* __restrict__ out, int64_t count, int epi,
                                                             const bf16_t* __restrict__ aux) {
  const int64_t vecs = count / 8;
  for (int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; v < vecs;
       v += (int64_t)gridDim.x * blockDim.x) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float4 x[NFIX > 0 ? NFIX : 1][2];
    if (NFIX > 0) {
#pragma unroll
      for (int i = 0; i < NFIX; ++i) {
        x[i][0] = reinterpret_cast<const float4*>(parts.p[i])[2 * v];
        x[i][1] = reinterpret_cast<const float4*>(parts.p[i])[2 * v + 1];
      }
    }
    uint4 m = make_uint4(0u, 0u, 0u, 0u);  // the mask operand travels with the partials
    if (epi == MTF_EPI_MASK_GT0) m = reinterpret_cast<const uint4*>(aux)[v];
    if (residual) {
      if (RES_BF16) {
        const uint4 r = reinterpret_cast<const uint4*>(residual)[v];
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[2 * e] = __uint_as_float(w[e] << 16);
          acc[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
        }
      } else {
        const float4 lo = reinterpret_cast<const float4*>(residual)[2 * v];
        const float4 hi = reinterpret_cast<const float4*>(residual)[2 * v + 1];
        acc[0] = lo.x; acc[1] = lo.y; acc[2] = lo.z; acc[3] = lo.w;
        acc[4] = hi.x; acc[5] = hi.y; acc[6] = hi.z; acc[7] = hi.w;
      }
    }
    // fixed order: residual, then partial 0, 1, ...
    auto add = [&](const float4& lo, const float4& hi) {
      acc[0] += lo.x; acc[1] += lo.y; acc[2] += lo.z; acc[3] += lo.w;
      acc[4] += hi.x; acc[5] += hi.y; acc[6] += hi.z; acc[7] += hi.w;
    };
    if (NFIX > 0) {
#pragma unroll
      for (int i = 0; i < NFIX; ++i) add(x[i][0], x[i][1]);
    } else {
      for (int i = 0; i < n; ++i)
        add(reinterpret_cast<const float4*>(parts.p[i])[2 * v], reinterpret_cast<const float4*>(parts.p[i])[2 * v + 1]);
    }
    // component-wise epilogue on the complete sum (one branch, uniform over the launch)
    if (epi == MTF_EPI_RELU) {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaxf(acc[e], 0.f);
    } else if (epi == MTF_EPI_MASK_GT0) {
      const uint32_t w[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] = __uint_as_float(w[e] << 16) > 0.f ? acc[2 * e] : 0.f;
        acc[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u) > 0.f ? acc[2 * e + 1] : 0.f;
      }
    }
    if (OUT_BF16) {
      reinterpret_cast<uint4*>(out)[v] = make_uint4(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                                                   pack_bf16x2(acc[4], acc[5]), pack_bf16x2(acc[6], acc[7]));
    } else {
      reinterpret_cast<float4*>(out)[2 * v] = make_float4(acc[0], acc[1], acc[2], acc[3]);
      reinterpret_cast<float4*>(out)[2 * v + 1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
  }
  // ragged tail (count not a multiple of 8): one thread each
  int64_t t = vecs * 8 + blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (t < count) {
    float acc = 0.f;
    if (residual)
      acc = RES_BF16 ? bf16_to_f32(static_cast<const bf16_t*>(residual)[t])
                     : static_cast<const float*>(residual)[t];
    for (int i = 0; i < n; ++i) acc += parts.p[i][t];
    if (epi == MTF_EPI_RELU) acc = fmaxf(acc, 0.f);
    if (epi == MTF_EPI_MASK_GT0) acc = bf16_to_f32(aux[t]) > 0.f ? acc : 0.f;
    if (OUT_BF16)
      static_cast<bf16_t*>(out)[t] = f32_to_bf16(acc);
    else
      static_cast<float*>(out)[t] = acc;
  }
}

// W <- W - lr * (g_0 + g_1 + ...) on the fp32 master copy, summed in that fixed order; the bf16
// copy the einsums read is written alongside.  8 elements per thread, 16-byte accesses.
template <int NFIX>
__global__ void __launch_bounds__(256) sgd_step_kernel(PartialPtrs grads, int n, float lr, float* __restrict__ master,
                                                      bf16_t* __restrict__ weights, int64_t count) {
  const int64_t vecs = count / 8;
  for (int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; v < vecs;
       v += (int64_t)gridDim.x * blockDim.x) {
    float4 x[NFIX > 0 ? NFIX : 1][2];
    if (NFIX > 0) {
#pragma unroll
      for (int i = 0; i < NFIX; ++i) {
        x[i][0] = reinterpret_cast<const float4*>(grads.p[i])[2 * v];
        x[i][1] = reinterpret_cast<const float4*>(grads.p[i])[2 * v + 1];
      }
    }
    const float4 m0 = reinterpret_cast<const float4*>(master)[2 * v];
    const float4 m1 = reinterpret_cast<const float4*>(master)[2 * v + 1];
    float sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto add = [&](const float4& lo, const float4& hi) {
      sum[0] += lo.x; sum[1] += lo.y; sum[2] += lo.z; sum[3] += lo.w;
      sum[4] += hi.x; sum[5] += hi.y; sum[6] += hi.z; sum[7] += hi.w;
    };
    if (NFIX > 0) {
#pragma unroll
      for (int i = 0; i < NFIX; ++i) add(x[i][0], x[i][1]);
    } else {
      for (int i = 0; i < n; ++i)
        add(reinterpret_cast<const float4*>(grads.p[i])[2 * v], reinterpret_cast<const float4*>(grads.p[i])[2 * v + 1]);
    }
    const float w[8] = {m0.x - lr * sum[0], m0.y - lr * sum[1], m0.z - lr * sum[2], m0.w - lr * sum[3],
                        m1.x - lr * sum[4], m1.y - lr * sum[5], m1.z - lr * sum[6], m1.w - lr * sum[7]};
    reinterpret_cast<float4*>(master)[2 * v] = make_float4(w[0], w[1], w[2], w[3]);
    reinterpret_cast<float4*>(master)[2 * v + 1] = make_float4(w[4], w[5], w[6], w[7]);
    if (weights)
      reinterpret_cast<uint4*>(weights)[v] = make_uint4(pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3]),
                                                       pack_bf16x2(w[4], w[5]), pack_bf16x2(w[6], w[7]));
  }
  int64_t t = vecs * 8 + blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (t < count) {
    float sum = 0.f;
    for (int i = 0; i < n; ++i) sum += grads.p[i][t];
    const float w = master[t] - lr * sum;
    master[t] = w;
    if (weights) weights[t] = f32_to_bf16(w);
  }
}

template <bool IN_BF16, bool OUT_BF16>
__global__ void __launch_bounds__(256) cast_kernel(const void* __restrict__ in, void* __restrict__ out,
                                                  int64_t count) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < count;
       i += (int64_t)gridDim.x * blockDim.x) {
    float v = IN_BF16 ? bf16_to_f32(static_cast<const bf16_t*>(in)[i]) : static_cast<const float*>(in)[i];
    if (OUT_BF16)
      static_cast<bf16_t*>(out)[i] = f32_to_bf16(v);
    else
      static_cast<float*>(out)[i] = v;
  }
}

}  // namespace mtf

using namespace mtf;

extern "C" {

int mtf_slice_copy(void* full, void* slice, const mtf_shape* t, const mtf_place* p,
                   mtf_dtype dt, int scatter, void* stream) {
  Dims d;
  if (int rc = load_shape(t, "tensor", &d)) return rc;
  if (!full || !slice) return fail(MTF_ERR_NULL, "full / slice");
  if (dt != MTF_F32 && dt != MTF_BF16) return fail(MTF_ERR_UNSUPPORTED, "dtype %d", (int)dt);
  int64_t off[MTF_MAX_RANK], sz[MTF_MAX_RANK];
  if (int rc = slice_of(d, p, off, sz)) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  return dt == MTF_F32 ? slice_copy_typed<float>(full, slice, d, off, sz, scatter, s)
                       : slice_copy_typed<bf16_t>(full, slice, d, off, sz, scatter, s);
}

int mtf_reduce_partials(const void* const* partials, int32_t n, const void* residual,
                        mtf_dtype residual_dt, void* out, mtf_dtype out_dt, int64_t count,
                        void* stream) {
  return mtf_reduce_partials_epi(partials, n, residual, residual_dt, out, out_dt, count, MTF_EPI_NONE, nullptr,
                                 stream);
}

int mtf_reduce_partials_epi(const void* const* partials, int32_t n, const void* residual,
                            mtf_dtype residual_dt, void* out, mtf_dtype out_dt, int64_t count,
                            mtf_epilogue epi, const void* aux, void* stream) {
  if (!partials) return fail(MTF_ERR_NULL, "partials");
  if (epi != MTF_EPI_NONE && epi != MTF_EPI_RELU && epi != MTF_EPI_MASK_GT0)
    return fail(MTF_ERR_UNSUPPORTED, "epilogue %d of a partial-sum reduce", (int)epi);
  if (epi == MTF_EPI_MASK_GT0 && count > 0 && !aux) return fail(MTF_ERR_NULL, "aux");
  if (epi == MTF_EPI_MASK_GT0 && !aligned16(aux)) return fail(MTF_ERR_ALIGN, "aux");
  if (n < 1 || n > 64) return fail(MTF_ERR_UNSUPPORTED, "%d partials (1..64)", n);
  if (count < 0) return fail(MTF_ERR_SIZE_MISMATCH, "count %lld", (long long)count);
  if (count == 0) return MTF_OK;  // nothing to sum: buffers may legitimately be empty (NULL)
  if (!out) return fail(MTF_ERR_NULL, "out");
  PartialPtrs pp;
  for (int i = 0; i < n; ++i) {
    if (!partials[i]) return fail(MTF_ERR_NULL, "partial %d", i);
    if (!aligned16(partials[i])) return fail(MTF_ERR_ALIGN, "partial %d", i);
    pp.p[i] = static_cast<const float*>(partials[i]);
  }
  if (!aligned16(out) || !aligned16(residual)) return fail(MTF_ERR_ALIGN, "out / residual");
  hipStream_t s = static_cast<hipStream_t>(stream);
  int blocks = (int)std::min<int64_t>(ceil_div(ceil_div(count, 8), 256), 256 * 8);
  bool rb = residual && residual_dt == MTF_BF16, ob = out_dt == MTF_BF16;
  LaunchTimer timer("reduce_partials_kernel", 0,
                    (double)count * (4.0 * n + (residual ? (rb ? 2 : 4) : 0) + (ob ? 2 : 4) +
                                     (epi == MTF_EPI_MASK_GT0 ? 2 : 0)), s);
  const int e = (int)epi;
  const bf16_t* ax = static_cast<const bf16_t*>(aux);
  // one vector per thread (count / 8 threads) up to 8 workgroups per CU, grid-stride beyond
  auto launch = [&](auto res_bf16, auto out_bf16) {
    constexpr bool RB = decltype(res_bf16)::value, OB = decltype(out_bf16)::value;
    switch (n) {
      case 1: reduce_partials_kernel<RB, OB, 1><<<blocks, 256, 0, s>>>(pp, n, residual, out, count, e, ax); break;
      case 2: reduce_partials_kernel<RB, OB, 2><<<blocks, 256, 0, s>>>(pp, n, residual, out, count, e, ax); break;
      case 3: reduce_partials_kernel<RB, OB, 3><<<blocks, 256, 0, s>>>(pp, n, residual, out, count, e, ax); break;
      case 4: reduce_partials_kernel<RB, OB, 4><<<blocks, 256, 0, s>>>(pp, n, residual, out, count, e, ax); break;
      default: reduce_partials_kernel<RB, OB, 0><<<blocks, 256, 0, s>>>(pp, n, residual, out, count, e, ax); break;
    }
  };
  if (rb && ob)
    launch(std::true_type{}, std::true_type{});
  else if (rb)
    launch(std::true_type{}, std::false_type{});
  else if (ob)
    launch(std::false_type{}, std::true_type{});
  else
    launch(std::false_type{}, std::false_type{});
  return launch_status("reduce_partials_kernel");
}

int mtf_sgd_step(const void* const* grads, int32_t n, float lr, void* master, void* weights,
                 int64_t count, void* stream) {
  if (!grads) return fail(MTF_ERR_NULL, "grads");
  if (n < 1 || n > 64) return fail(MTF_ERR_UNSUPPORTED, "%d gradient buffers (1..64)", n);
  if (count < 0) return fail(MTF_ERR_SIZE_MISMATCH, "count %lld", (long long)count);
  if (count == 0) return MTF_OK;
  if (!master) return fail(MTF_ERR_NULL, "master");
  PartialPtrs pp;
  for (int i = 0; i < n; ++i) {
    if (!grads[i]) return fail(MTF_ERR_NULL, "gradient %d", i);
    if (!aligned16(grads[i])) return fail(MTF_ERR_ALIGN, "gradient %d", i);
    pp.p[i] = static_cast<const float*>(grads[i]);
  }
  if (!aligned16(master) || !aligned16(weights)) return fail(MTF_ERR_ALIGN, "master / weights");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int blocks = (int)std::min<int64_t>(ceil_div(ceil_div(count, 8), 256), 256 * 8);
  LaunchTimer timer("sgd_step_kernel", 0, (double)count * (4.0 * n + 8.0 + (weights ? 2.0 : 0.0)), s);
  float* m = static_cast<float*>(master);
  bf16_t* w = static_cast<bf16_t*>(weights);
  switch (n) {
    case 1: sgd_step_kernel<1><<<blocks, 256, 0, s>>>(pp, n, lr, m, w, count); break;
    case 2: sgd_step_kernel<2><<<blocks, 256, 0, s>>>(pp, n, lr, m, w, count); break;
    case 4: sgd_step_kernel<4><<<blocks, 256, 0, s>>>(pp, n, lr, m, w, count); break;
    default: sgd_step_kernel<0><<<blocks, 256, 0, s>>>(pp, n, lr, m, w, count); break;
  }
  return launch_status("sgd_step_kernel");
}

int mtf_cast(const void* in, mtf_dtype in_dt, void* out, mtf_dtype out_dt, int64_t count,
             void* stream) {
  if (count < 0) return fail(MTF_ERR_SIZE_MISMATCH, "count %lld", (long long)count);
  if (count == 0) return MTF_OK;
  if (!in || !out) return fail(MTF_ERR_NULL, "in / out");
  hipStream_t s = static_cast<hipStream_t>(stream);
  int blocks = (int)std::min<int64_t>(ceil_div(count, 256), 256 * 8);
  bool ib = in_dt == MTF_BF16, ob = out_dt == MTF_BF16;
  LaunchTimer timer("cast_kernel", 0, (double)count * ((ib ? 2 : 4) + (ob ? 2 : 4)), s);
  if (ib && ob)
    cast_kernel<true, true><<<blocks, 256, 0, s>>>(in, out, count);
  else if (ib)
    cast_kernel<true, false><<<blocks, 256, 0, s>>>(in, out, count);
  else if (ob)
    cast_kernel<false, true><<<blocks, 256, 0, s>>>(in, out, count);
  else
    cast_kernel<false, false><<<blocks, 256, 0, s>>>(in, out, count);
  return launch_status("cast_kernel");
}

}  // extern "C"
