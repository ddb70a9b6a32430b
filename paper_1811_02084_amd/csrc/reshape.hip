// Reshape on a virtual mesh (subsection "Reshape"): one processor's output slice gathered from
// the input slices of all processors held on this GPU.  A copy: HBM-bound, bit-exact.
#include <algorithm>

#include "device_common.h"
#include "timing.h"

namespace mtf {
namespace {

constexpr int kMaxProcessors = 64;

struct ReshapeArgs {
  const void* src[kMaxProcessors];  // input slice of every processor, by rank
  int rank, mesh_rank;
  int64_t out_local[MTF_MAX_RANK], out_offset[MTF_MAX_RANK];  // this processor's output slice
  int64_t in_local[MTF_MAX_RANK], in_stride[MTF_MAX_RANK];     // any processor's input slice
  int in_axis[MTF_MAX_RANK];                                   // mesh axis splitting position i in the input
  int64_t rank_stride[MTF_MAX_RANK];                           // row-major processor numbering
  int64_t own_rank_part;  // rank contribution of this processor's coordinates on axes the input does not use
  int64_t runs;           // output slice elements / vec
};

// One wave per row (all positions but the innermost) at a time, its lanes over runs of VEC
// consecutive elements of the innermost position (the host picks VEC so that a run never crosses
// a stripe of the input or the end of a row).  The row's part of the source processor and offset
// is computed once per row; a run adds one division by the input's stripe length.
template <typename T, int VEC>
__global__ void __launch_bounds__(256) reshape_kernel(ReshapeArgs g, T* __restrict__ out) {
  const int last = g.rank - 1;
  const int64_t rows = g.runs;  // here: number of rows
  const uint32_t row_runs = (uint32_t)(g.out_local[last] / VEC);
  const uint32_t in_len = (uint32_t)g.in_local[last], out_off = (uint32_t)g.out_offset[last];
  const bool last_split = g.in_axis[last] >= 0;
  const int64_t last_proc_stride = last_split ? g.rank_stride[g.in_axis[last]] : 0;
  const int lane = threadIdx.x & 63;
  for (int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); row < rows; row += (int64_t)gridDim.x * 4) {
    int64_t rem = row, proc = g.own_rank_part, off = 0;
    for (int i = last - 1; i >= 0; --i) {
      const int64_t global = g.out_offset[i] + rem % g.out_local[i];
      rem /= g.out_local[i];
      int64_t local = global;
      if (g.in_axis[i] >= 0) {  // the stripe of the input that holds it, and the index inside
        proc += (global / g.in_local[i]) * g.rank_stride[g.in_axis[i]];
        local = global % g.in_local[i];
      }
      off += local * g.in_stride[i];
    }
    T* dst_row = out + row * (int64_t)row_runs * VEC;
    for (uint32_t j = lane; j < row_runs; j += 64) {
      const uint32_t global = out_off + j * VEC;
      const uint32_t stripe = last_split ? global / in_len : 0u;
      const uint32_t local = last_split ? global - stripe * in_len : global;
      const T* src = static_cast<const T*>(g.src[proc + stripe * last_proc_stride]) + off + local;
      T* dst = dst_row + j * VEC;
      if (VEC * sizeof(T) == 16) {
        *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) dst[e] = src[e];
      }
    }
  }
}

struct GeneralArgs {
  const void* src[kMaxProcessors];  // input slice of every processor, by rank
  int in_rank, out_rank;
  int64_t out_size[MTF_MAX_RANK], out_local[MTF_MAX_RANK], out_offset[MTF_MAX_RANK];
  int64_t in_size[MTF_MAX_RANK], in_local[MTF_MAX_RANK], in_stride[MTF_MAX_RANK];
  int in_axis[MTF_MAX_RANK];
  int64_t rank_stride[MTF_MAX_RANK];
  int64_t own_rank_part;
  int64_t runs;  // output slice elements / VEC
};

// Reshape that changes rank / sizes: one thread per run of VEC consecutive elements of the output
// slice's innermost dim.  The run's first element has a position in the full output, hence a
// row-major rank among all elements, hence a position in the full input; from that, the processor
// whose input slice holds it and the offset inside that slice.  (The host picks VEC so that a run
// stays inside one stripe of the input's innermost dim.)  Index arithmetic per run, not per byte:
// with VEC = 16 bytes the copy is still bound by memory.
template <typename T, int VEC>
__global__ void __launch_bounds__(256) reshape_general_kernel(GeneralArgs g, T* __restrict__ out) {
  const int olast = g.out_rank - 1;
  const int64_t row_runs = g.out_local[olast] / VEC;
  for (int64_t run = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; run < g.runs;
       run += (int64_t)gridDim.x * blockDim.x) {
    // position in the output slice -> row-major rank in the full tensor (Horner over the dims)
    int64_t rem = run / row_runs;
    int64_t idx[MTF_MAX_RANK];
    idx[olast] = g.out_offset[olast] + (run % row_runs) * VEC;
    for (int i = olast - 1; i >= 0; --i) {
      idx[i] = g.out_offset[i] + rem % g.out_local[i];
      rem /= g.out_local[i];
    }
    int64_t lin = 0;
    for (int i = 0; i <= olast; ++i) lin = lin * g.out_size[i] + idx[i];
    // -> position in the full input -> owner and offset
    int64_t proc = g.own_rank_part, off = 0;
    for (int i = g.in_rank - 1; i >= 0; --i) {
      int64_t pos = lin % g.in_size[i];
      lin /= g.in_size[i];
      if (g.in_axis[i] >= 0) {
        proc += (pos / g.in_local[i]) * g.rank_stride[g.in_axis[i]];
        pos %= g.in_local[i];
      }
      off += pos * g.in_stride[i];
    }
    const T* src = static_cast<const T*>(g.src[proc]) + off;
    T* dst = out + run * VEC;
    if (VEC * sizeof(T) == 16) {
      *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) dst[e] = src[e];
    }
  }
}

template <typename T>
int launch_general(const GeneralArgs& g, void* out, int vec, int64_t elems, hipStream_t s) {
  const int blocks = (int)std::min<int64_t>(ceil_div(g.runs, 256), 256 * 32);
  LaunchTimer timer("reshape_general_kernel", 0, 2.0 * elems * sizeof(T), s);
  constexpr int kFull = 16 / sizeof(T);
  if (vec == kFull)
    reshape_general_kernel<T, kFull><<<blocks, 256, 0, s>>>(g, static_cast<T*>(out));
  else
    reshape_general_kernel<T, 1><<<blocks, 256, 0, s>>>(g, static_cast<T*>(out));
  return launch_status("reshape_general_kernel");
}

template <typename T>
int launch(const ReshapeArgs& g, void* out, int vec, int64_t elems, hipStream_t s) {
  const int blocks = (int)std::min<int64_t>(ceil_div(g.runs, 4), 256 * 32);
  LaunchTimer timer("reshape_kernel", 0, 2.0 * elems * sizeof(T), s);
  constexpr int kFull = 16 / sizeof(T);  // elements per 16-byte access
  if (vec == kFull)
    reshape_kernel<T, kFull><<<blocks, 256, 0, s>>>(g, static_cast<T*>(out));
  else
    reshape_kernel<T, 1><<<blocks, 256, 0, s>>>(g, static_cast<T*>(out));
  return launch_status("reshape_kernel");
}

}  // namespace
}  // namespace mtf

using namespace mtf;

extern "C" int mtf_reshape_virtual(const void* const* in_slices, const mtf_shape* in, const mtf_shape* out,
                                   const mtf_place* p, void* out_slice, mtf_dtype dt, void* stream) {
  Dims din, dout;
  if (int rc = load_shape(in, "input", &din)) return rc;
  if (int rc = load_shape(out, "output", &dout)) return rc;
  if (!in_slices || !out_slice) return fail(MTF_ERR_NULL, "in_slices / out_slice");
  if (dt != MTF_F32 && dt != MTF_BF16) return fail(MTF_ERR_UNSUPPORTED, "dtype %d", (int)dt);
  ReshapeInfo r;
  if (int rc = reshape_info(din, dout, p, true, &r)) return rc;
  int64_t processors = 1;
  for (int m = 0; m < r.mesh_rank; ++m) processors *= r.mesh_size[m];
  if (processors > kMaxProcessors)
    return fail(MTF_ERR_UNSUPPORTED, "virtual reshape over %lld processors (at most %d)", (long long)processors,
                kMaxProcessors);
  // a rank-0 tensor has no dim to rename or split (and no innermost position for the copy kernel)
  if (r.rank == 0) return fail(MTF_ERR_RANK, "reshape of a rank-0 tensor");
  ReshapeArgs g{};
  for (int64_t q = 0; q < processors; ++q) {
    if (!in_slices[q]) return fail(MTF_ERR_NULL, "in_slices[%lld]", (long long)q);
    g.src[q] = in_slices[q];
  }
  g.rank = r.rank;
  g.mesh_rank = r.mesh_rank;
  int64_t acc = 1;
  for (int m = r.mesh_rank - 1; m >= 0; --m) {
    g.rank_stride[m] = acc;
    acc *= r.mesh_size[m];
  }
  bool used[MTF_MAX_RANK] = {};
  int64_t elems = 1, stride = 1;
  for (int i = r.rank - 1; i >= 0; --i) {
    g.out_local[i] = r.out_local[i];
    g.out_offset[i] = r.out_offset[i];
    g.in_local[i] = r.in_local[i];
    g.in_axis[i] = r.in_axis[i];
    g.in_stride[i] = stride;
    stride *= r.in_local[i];
    elems *= r.out_local[i];
    if (r.in_axis[i] >= 0) used[r.in_axis[i]] = true;
  }
  g.own_rank_part = 0;
  for (int m = 0; m < r.mesh_rank; ++m)
    if (!used[m]) g.own_rank_part += r.coord[m] * g.rank_stride[m];
  if (elems == 0) return MTF_OK;
  // 16-byte runs along the innermost position must stay inside one input stripe and one output
  // row, and start 16-byte aligned in both slices
  const int last = r.rank - 1;
  const int full = dt == MTF_F32 ? 4 : 8;
  if (r.out_local[last] >= ((int64_t)1 << 31) || r.in_local[last] >= ((int64_t)1 << 31))
    return fail(MTF_ERR_UNSUPPORTED, "innermost position too long");
  bool aligned = aligned16(out_slice) && r.out_local[last] % full == 0 && r.out_offset[last] % full == 0 &&
                 r.in_local[last] % full == 0;
  for (int64_t q = 0; q < processors; ++q) aligned = aligned && aligned16(in_slices[q]);
  const int vec = aligned ? full : 1;
  g.runs = elems / r.out_local[last];  // rows
  hipStream_t s = static_cast<hipStream_t>(stream);
  return dt == MTF_F32 ? launch<float>(g, out_slice, vec, elems, s) : launch<bf16_t>(g, out_slice, vec, elems, s);
}

extern "C" int mtf_reshape_general_virtual(const void* const* in_slices, const mtf_shape* in, const mtf_shape* out,
                                           const mtf_place* p, void* out_slice, mtf_dtype dt, void* stream) {
  Dims din, dout;
  if (int rc = load_shape(in, "input", &din)) return rc;
  if (int rc = load_shape(out, "output", &dout)) return rc;
  if (!in_slices || !out_slice) return fail(MTF_ERR_NULL, "in_slices / out_slice");
  if (dt != MTF_F32 && dt != MTF_BF16) return fail(MTF_ERR_UNSUPPORTED, "dtype %d", (int)dt);
  if (din.rank == 0 || dout.rank == 0) return fail(MTF_ERR_RANK, "reshape of a rank-0 tensor");
  GeneralReshapeInfo r;
  if (int rc = reshape_general_info(din, dout, p, &r)) return rc;
  int64_t processors = 1;
  for (int m = 0; m < r.mesh_rank; ++m) processors *= r.mesh_size[m];
  if (processors > kMaxProcessors)
    return fail(MTF_ERR_UNSUPPORTED, "virtual reshape over %lld processors (at most %d)", (long long)processors,
                kMaxProcessors);
  GeneralArgs g{};
  for (int64_t q = 0; q < processors; ++q) {
    if (!in_slices[q]) return fail(MTF_ERR_NULL, "in_slices[%lld]", (long long)q);
    g.src[q] = in_slices[q];
  }
  g.in_rank = r.in_rank;
  g.out_rank = r.out_rank;
  int64_t acc = 1;
  for (int m = r.mesh_rank - 1; m >= 0; --m) {
    g.rank_stride[m] = acc;
    acc *= r.mesh_size[m];
  }
  bool used[MTF_MAX_RANK] = {};
  int64_t stride = 1;
  for (int i = r.in_rank - 1; i >= 0; --i) {
    g.in_size[i] = r.in_size[i];
    g.in_local[i] = r.in_local[i];
    g.in_axis[i] = r.in_axis[i];
    g.in_stride[i] = stride;
    stride *= r.in_local[i];
    if (r.in_axis[i] >= 0) used[r.in_axis[i]] = true;
  }
  int64_t elems = 1;
  for (int i = 0; i < r.out_rank; ++i) {
    g.out_size[i] = r.out_size[i];
    g.out_local[i] = r.out_local[i];
    g.out_offset[i] = r.out_offset[i];
    elems *= r.out_local[i];
  }
  for (int m = 0; m < r.mesh_rank; ++m)
    if (!used[m]) g.own_rank_part += r.coord[m] * g.rank_stride[m];
  if (elems == 0) return MTF_OK;
  // a 16-byte run along the output's innermost dim starts at a multiple of its length in the
  // element order; it stays inside one stripe of the input's innermost dim if that stripe's length
  // is a multiple of the run length too
  const int full = dt == MTF_F32 ? 4 : 8;
  bool aligned = aligned16(out_slice) && r.out_local[r.out_rank - 1] % full == 0 && r.in_local[r.in_rank - 1] % full == 0;
  for (int64_t q = 0; q < processors; ++q) aligned = aligned && aligned16(in_slices[q]);
  const int vec = aligned ? full : 1;
  g.runs = elems / vec;
  hipStream_t s = static_cast<hipStream_t>(stream);
  return dt == MTF_F32 ? launch_general<float>(g, out_slice, vec, elems, s)
                       : launch_general<bf16_t>(g, out_slice, vec, elems, s);
}
