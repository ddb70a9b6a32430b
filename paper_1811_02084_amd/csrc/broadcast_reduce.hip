// Component-wise addition with implicit broadcasting (section "Mesh-TensorFlow syntax") and local
// reductions (section "Operation Implementation", paragraph "Reduction"), on one processor's
// slices.  Both are HBM-bound: every element is read once.
#include <algorithm>
#include <mutex>

#include "device_common.h"
#include "reduce_local.h"
#include "timing.h"

namespace mtf {
namespace {

template <typename T>
__device__ __forceinline__ float ld(const T* p, int64_t i);
template <>
__device__ __forceinline__ float ld<float>(const float* p, int64_t i) { return p[i]; }
template <>
__device__ __forceinline__ float ld<bf16_t>(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }
template <typename T>
__device__ __forceinline__ void st(T* p, int64_t i, float v);
template <>
__device__ __forceinline__ void st<float>(float* p, int64_t i, float v) { p[i] = v; }
template <>
__device__ __forceinline__ void st<bf16_t>(bf16_t* p, int64_t i, float v) { p[i] = f32_to_bf16(v); }

// ------------------------------------------------------------------------------- a + b
struct AddArgs {
  int rank;
  int64_t extent[MTF_MAX_RANK];    // a's dims, row-major
  int64_t b_stride[MTF_MAX_RANK];  // element stride of that dim in b, 0 where b lacks it
  int64_t count;
};

// One thread per run of 4 consecutive elements of a's innermost dim (a run never crosses a row:
// the host only picks this kernel when that dim is a multiple of 4).
template <typename InT, typename OutT>
__global__ void __launch_bounds__(256) add_broadcast_kernel(const InT* __restrict__ a, const InT* __restrict__ b,
                                                           OutT* __restrict__ out, AddArgs g, int vec) {
  const int64_t runs = g.count / vec;
  for (int64_t r = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; r < runs; r += (int64_t)gridDim.x * blockDim.x) {
    const int64_t first = r * vec;
    int64_t rem = first, ib = 0;
    for (int d = g.rank - 1; d >= 0; --d) {
      ib += (rem % g.extent[d]) * g.b_stride[d];
      rem /= g.extent[d];
    }
    const int64_t step = g.rank > 0 ? g.b_stride[g.rank - 1] : 0;  // rank 0: one element
    for (int e = 0; e < vec; ++e) st<OutT>(out, first + e, ld<InT>(a, first + e) + ld<InT>(b, ib + e * step));
  }
}

// ------------------------------------------------------------------------------- reductions
template <int OP>
__device__ __forceinline__ float combine(float x, float y) {
  return OP == MTF_REDUCE_SUM ? x + y : fmaxf(x, y);
}
template <int OP>
__device__ __forceinline__ float identity() {
  return OP == MTF_REDUCE_SUM ? 0.f : -INFINITY;
}

// Column reduction, first pass: in[rows, cols] -> part[chunks, cols].  A workgroup covers
// kColsPerGroup columns (threadIdx.x % 64 picks 8 of them, threadIdx.x / 64 one of 4 row lanes)
// and the rows [chunk * rows_per_chunk, ...).  Row lanes are combined through LDS in lane order.
constexpr int kColsPerGroup = 512;
template <typename InT, int OP>
__global__ void __launch_bounds__(256) reduce_cols_kernel(const InT* __restrict__ in, float* __restrict__ part,
                                                         int64_t rows, int64_t cols, int64_t rows_per_chunk) {
  __shared__ float lds[4][kColsPerGroup];
  const int cl = (threadIdx.x & 63) * 8, rl = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * kColsPerGroup + cl;
  const int64_t r_begin = (int64_t)blockIdx.y * rows_per_chunk;
  const int64_t r_end = min(rows, r_begin + rows_per_chunk);
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = identity<OP>();
  if (c0 < cols) {  // cols is a multiple of 8
    for (int64_t r = r_begin + rl; r < r_end; r += 4) {
      const InT* p = in + r * cols + c0;
      if (sizeof(InT) == 2) {
        const uint4 w = *reinterpret_cast<const uint4*>(p);
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[2 * e] = combine<OP>(acc[2 * e], __uint_as_float(u[e] << 16));
          acc[2 * e + 1] = combine<OP>(acc[2 * e + 1], __uint_as_float(u[e] & 0xffff0000u));
        }
      } else {
        const float4 lo = *reinterpret_cast<const float4*>(p), hi = *reinterpret_cast<const float4*>(p + 4);
        const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = combine<OP>(acc[e], v[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) lds[rl][cl + e] = acc[e];
  __syncthreads();
  for (int c = threadIdx.x; c < kColsPerGroup; c += 256) {
    const int64_t col = (int64_t)blockIdx.x * kColsPerGroup + c;
    if (col < cols)
      part[(int64_t)blockIdx.y * cols + col] =
          combine<OP>(combine<OP>(lds[0][c], lds[1][c]), combine<OP>(lds[2][c], lds[3][c]));
  }
}

// Second pass: out[c] = combine over the chunks.  64 columns per workgroup; row lane j of 4
// combines the chunks k = j, j+4, ... in that order, then the 4 lanes are combined in lane order
// (a fixed association, so the result is reproducible).
template <typename OutT, int OP>
__global__ void __launch_bounds__(256) reduce_chunks_kernel(const float* __restrict__ part, OutT* __restrict__ out,
                                                           int64_t chunks, int64_t cols) {
  __shared__ float lds[4][64];
  const int cl = threadIdx.x & 63, j = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * 64 + cl;
  float acc = identity<OP>();
  if (c < cols) {
#pragma unroll 4
    for (int64_t k = j; k < chunks; k += 4) acc = combine<OP>(acc, part[k * cols + c]);
  }
  lds[j][cl] = acc;
  __syncthreads();
  if (j == 0 && c < cols)
    st<OutT>(out, c, combine<OP>(combine<OP>(lds[0][cl], lds[1][cl]), combine<OP>(lds[2][cl], lds[3][cl])));
}

// Row reduction: in[rows, cols] -> out[rows]; one wave per row, lanes stride the row, then a
// butterfly over the wave (fixed order).
template <typename InT, typename OutT, int OP>
__global__ void __launch_bounds__(256) reduce_rows_kernel(const InT* __restrict__ in, OutT* __restrict__ out,
                                                         int64_t rows, int64_t cols) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  float acc = identity<OP>();
  if (sizeof(InT) == 4 && cols % 4 == 0) {  // fp32 rows, 16-byte aligned: 16 bytes per lane
    const float* p = reinterpret_cast<const float*>(in) + row * cols;
    for (int64_t c = lane * 4; c < cols; c += 256) {
      const float4 q = *reinterpret_cast<const float4*>(p + c);
      acc = combine<OP>(acc, combine<OP>(combine<OP>(q.x, q.y), combine<OP>(q.z, q.w)));
    }
  } else {
    for (int64_t c = lane; c < cols; c += 64) acc = combine<OP>(acc, ld<InT>(in, row * cols + c));
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) acc = combine<OP>(acc, __shfl_xor(acc, m));
  if (lane == 0) st<OutT>(out, row, acc);
}

// Anything else: one thread per output element, reduced dims visited in row-major order.
struct GenericReduce {
  int n_out, n_red;
  int64_t out_extent[MTF_MAX_RANK], out_stride[MTF_MAX_RANK];
  int64_t red_extent[MTF_MAX_RANK], red_stride[MTF_MAX_RANK];
  int64_t out_elems, red_points;
};
template <typename InT, typename OutT, int OP>
__global__ void __launch_bounds__(256) reduce_generic_kernel(const InT* __restrict__ in, OutT* __restrict__ out,
                                                            GenericReduce g) {
  for (int64_t o = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; o < g.out_elems;
       o += (int64_t)gridDim.x * blockDim.x) {
    int64_t rem = o, base = 0;
    for (int d = g.n_out - 1; d >= 0; --d) {
      base += (rem % g.out_extent[d]) * g.out_stride[d];
      rem /= g.out_extent[d];
    }
    float acc = identity<OP>();
    int64_t idx[MTF_MAX_RANK];
    for (int d = 0; d < g.n_red; ++d) idx[d] = 0;
    int64_t off = base;
    for (int64_t r = 0; r < g.red_points; ++r) {
      acc = combine<OP>(acc, ld<InT>(in, off));
      for (int d = g.n_red - 1; d >= 0; --d) {
        off += g.red_stride[d];
        if (++idx[d] < g.red_extent[d]) break;
        off -= idx[d] * g.red_stride[d];
        idx[d] = 0;
      }
    }
    st<OutT>(out, o, acc);
  }
}

// How a reduction maps onto the kernels above.
enum Pattern { P_COLS, P_ROWS, P_GENERIC };
struct ReducePlan {
  Pattern pattern;
  int64_t rows, cols;  // P_COLS: reduce rows, keep cols; P_ROWS: keep rows, reduce cols
  int64_t chunks, rows_per_chunk;
  size_t workspace;
};

// The kept dims form OUT in the same relative order as in IN and are either all trailing
// (P_COLS) or all leading (P_ROWS); otherwise the generic kernel runs.
ReducePlan plan_reduce(const Dims& in, const Dims& out) {
  ReducePlan p{};
  p.pattern = P_GENERIC;
  int64_t total = 1, kept = 1;
  for (int i = 0; i < in.rank; ++i) total *= in.size[i];
  for (int i = 0; i < out.rank; ++i) kept *= out.size[i];
  const int n_red = in.rank - out.rank;
  if (out.rank == 0 || n_red == 0) return p;
  bool trailing = true, leading = true;
  for (int i = 0; i < out.rank; ++i) {
    if (!same(out.name[i], in.name[n_red + i])) trailing = false;
    if (!same(out.name[i], in.name[i])) leading = false;
  }
  if (trailing && kept % 8 == 0) {
    p.pattern = P_COLS;
    p.cols = kept;
    p.rows = total / kept;
    const int64_t col_groups = ceil_div(p.cols, kColsPerGroup);
    // enough workgroups to fill the chip (>= 16 rows each), few enough chunks that the second
    // pass (one thread per column, chunks summed in order) stays short
    p.chunks = std::max<int64_t>(
        1, std::min<int64_t>(std::min<int64_t>(ceil_div(p.rows, 16), ceil_div(1024, col_groups)), 64));
    p.rows_per_chunk = ceil_div(p.rows, p.chunks);
    p.chunks = ceil_div(p.rows, p.rows_per_chunk);
    p.workspace = (size_t)p.chunks * p.cols * sizeof(float);
  } else if (leading) {
    p.pattern = P_ROWS;
    p.rows = kept;
    p.cols = total / kept;
  }
  return p;
}

template <typename InT, typename OutT, int OP>
int run_reduce(const void* in, const Dims& din, void* out, const Dims& dout, const ReducePlan& p, void* workspace,
               hipStream_t s) {
  int64_t total = 1, kept = 1;
  for (int i = 0; i < din.rank; ++i) total *= din.size[i];
  for (int i = 0; i < dout.rank; ++i) kept *= dout.size[i];
  const double bytes = (double)total * sizeof(InT) + (double)kept * sizeof(OutT);
  if (p.pattern == P_COLS) {
    float* part = static_cast<float*>(workspace);
    {
      LaunchTimer timer("reduce_cols_kernel", 0, (double)total * sizeof(InT) + (double)p.workspace, s);
      dim3 grid((unsigned)ceil_div(p.cols, kColsPerGroup), (unsigned)p.chunks);
      reduce_cols_kernel<InT, OP><<<grid, 256, 0, s>>>(static_cast<const InT*>(in), part, p.rows, p.cols,
                                                     p.rows_per_chunk);
    }
    if (int rc = launch_status("reduce_cols_kernel")) return rc;
    {
      LaunchTimer timer("reduce_chunks_kernel", 0, (double)p.workspace + (double)kept * sizeof(OutT), s);
      reduce_chunks_kernel<OutT, OP><<<(unsigned)ceil_div(p.cols, 64), 256, 0, s>>>(part, static_cast<OutT*>(out),
                                                                                 p.chunks, p.cols);
    }
    return launch_status("reduce_chunks_kernel");
  }
  if (p.pattern == P_ROWS) {
    LaunchTimer timer("reduce_rows_kernel", 0, bytes, s);
    reduce_rows_kernel<InT, OutT, OP><<<(unsigned)ceil_div(p.rows, 4), 256, 0, s>>>(
        static_cast<const InT*>(in), static_cast<OutT*>(out), p.rows, p.cols);
    return launch_status("reduce_rows_kernel");
  }
  GenericReduce g{};
  int64_t stride[MTF_MAX_RANK], acc = 1;
  for (int i = din.rank - 1; i >= 0; --i) {
    stride[i] = acc;
    acc *= din.size[i];
  }
  g.n_out = dout.rank;
  g.out_elems = kept;
  for (int i = 0; i < dout.rank; ++i) {
    g.out_extent[i] = dout.size[i];
    g.out_stride[i] = stride[find(din, dout.name[i])];
  }
  g.red_points = 1;
  for (int i = 0; i < din.rank; ++i)
    if (find(dout, din.name[i]) < 0) {
      g.red_extent[g.n_red] = din.size[i];
      g.red_stride[g.n_red] = stride[i];
      g.red_points *= din.size[i];
      ++g.n_red;
    }
  LaunchTimer timer("reduce_generic_kernel", 0, bytes, s);
  const int blocks = (int)std::min<int64_t>(ceil_div(g.out_elems, 256), 256 * 32);
  reduce_generic_kernel<InT, OutT, OP><<<blocks, 256, 0, s>>>(static_cast<const InT*>(in), static_cast<OutT*>(out), g);
  return launch_status("reduce_generic_kernel");
}

template <typename InT, typename OutT>
int run_reduce_op(int op, const void* in, const Dims& din, void* out, const Dims& dout, const ReducePlan& p,
                  void* workspace, hipStream_t s) {
  return op == MTF_REDUCE_SUM ? run_reduce<InT, OutT, MTF_REDUCE_SUM>(in, din, out, dout, p, workspace, s)
                              : run_reduce<InT, OutT, MTF_REDUCE_MAX>(in, din, out, dout, p, workspace, s);
}

int check_reduce_shapes(const mtf_shape* in_local, const mtf_shape* out_local, Dims* din, Dims* dout) {
  if (int rc = load_shape(in_local, "input", din)) return rc;
  if (int rc = load_shape(out_local, "output", dout)) return rc;
  for (int i = 0; i < dout->rank; ++i) {
    const int j = find(*din, dout->name[i]);
    if (j < 0) return fail(MTF_ERR_OUT_NOT_SUBSET, "output dim '%s' is not a dim of the input", dout->name[i]);
    if (din->size[j] != dout->size[i])
      return fail(MTF_ERR_SIZE_MISMATCH, "dim '%s': %lld vs %lld", dout->name[i], (long long)din->size[j],
                  (long long)dout->size[i]);
  }
  return MTF_OK;
}

}  // namespace

size_t reduce_cols_workspace_bytes(int64_t rows, int64_t cols) {
  Dims din, dout;
  din.rank = 2;
  din.name[0] = "r";
  din.name[1] = "c";
  din.size[0] = rows;
  din.size[1] = cols;
  dout.rank = 1;
  dout.name[0] = "c";
  dout.size[0] = cols;
  return plan_reduce(din, dout).workspace;
}

int reduce_cols_sum(const bf16_t* in, float* out, int64_t rows, int64_t cols, void* workspace, size_t workspace_bytes,
                    hipStream_t s) {
  Dims din, dout;
  din.rank = 2;
  din.name[0] = "r";
  din.name[1] = "c";
  din.size[0] = rows;
  din.size[1] = cols;
  dout.rank = 1;
  dout.name[0] = "c";
  dout.size[0] = cols;
  const ReducePlan p = plan_reduce(din, dout);
  if (p.pattern == P_COLS && (!workspace || workspace_bytes < p.workspace))
    return fail(MTF_ERR_WORKSPACE, "column reduction needs %zu bytes", p.workspace);
  return run_reduce<bf16_t, float, MTF_REDUCE_SUM>(in, din, out, dout, p, workspace, s);
}

}  // namespace mtf

using namespace mtf;

// ------------------------------------------------------------------------------- static scratch
// Scratch of the entry point that allocates nothing (mtf_reduce_local_static): the chunk partials
// of the column reduction live in a file-scope device array instead of a caller workspace.  Every
// device the library runs on holds its own copy of the array at its own address; in host code the
// array's NAME is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[MTF_REDUCE_STATIC_MAX_SCRATCH];

static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};  // per device: address of `scratch` there (nullptr: not asked yet)

// *out = device address of `scratch` on the current device (looked up once per device, with that
// device current).  Returns MTF_OK or the error.
static int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices)
    return fail(MTF_ERR_UNSUPPORTED, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!ptr) return fail(MTF_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return MTF_OK;
}


extern "C" {

int mtf_add_broadcast(const void* a, const mtf_shape* a_local, const void* b, const mtf_shape* b_local, void* out,
                      mtf_dtype in_dt, mtf_dtype out_dt, void* stream) {
  Dims da, db;
  if (int rc = load_shape(a_local, "a", &da)) return rc;
  if (int rc = load_shape(b_local, "b", &db)) return rc;
  if (!a || !b || !out) return fail(MTF_ERR_NULL, "a / b / out");
  if ((in_dt != MTF_F32 && in_dt != MTF_BF16) || (out_dt != MTF_F32 && out_dt != MTF_BF16))
    return fail(MTF_ERR_UNSUPPORTED, "dtype");
  if (!aligned16(a) || !aligned16(b) || !aligned16(out)) return fail(MTF_ERR_ALIGN, "a / b / out");
  AddArgs g{};
  int64_t sb[MTF_MAX_RANK], acc = 1;
  for (int i = db.rank - 1; i >= 0; --i) {
    sb[i] = acc;
    acc *= db.size[i];
  }
  for (int i = 0; i < db.rank; ++i) {
    const int j = find(da, db.name[i]);
    if (j < 0) return fail(MTF_ERR_OUT_NOT_SUBSET, "dim '%s' of b is not a dim of a", db.name[i]);
    if (da.size[j] != db.size[i])
      return fail(MTF_ERR_SIZE_MISMATCH, "dim '%s': %lld vs %lld", db.name[i], (long long)da.size[j],
                  (long long)db.size[i]);
  }
  g.rank = da.rank;
  g.count = 1;
  for (int i = 0; i < da.rank; ++i) {
    const int j = find(db, da.name[i]);
    g.extent[i] = da.size[i];
    g.b_stride[i] = j >= 0 ? sb[j] : 0;
    g.count *= da.size[i];
  }
  const int vec = da.rank > 0 && da.size[da.rank - 1] % 4 == 0 ? 4 : 1;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t runs = g.count / vec;
  const int blocks = (int)std::min<int64_t>(ceil_div(runs, 256), 256 * 32);
  const double bytes = (double)g.count * ((in_dt == MTF_BF16 ? 2 : 4) + (out_dt == MTF_BF16 ? 2 : 4)) +
                       (double)acc * (in_dt == MTF_BF16 ? 2 : 4);
  LaunchTimer timer("add_broadcast_kernel", 0, bytes, s);
  if (in_dt == MTF_F32 && out_dt == MTF_F32)
    add_broadcast_kernel<float, float><<<blocks, 256, 0, s>>>((const float*)a, (const float*)b, (float*)out, g, vec);
  else if (in_dt == MTF_F32)
    add_broadcast_kernel<float, bf16_t><<<blocks, 256, 0, s>>>((const float*)a, (const float*)b, (bf16_t*)out, g, vec);
  else if (out_dt == MTF_F32)
    add_broadcast_kernel<bf16_t, float><<<blocks, 256, 0, s>>>((const bf16_t*)a, (const bf16_t*)b, (float*)out, g, vec);
  else
    add_broadcast_kernel<bf16_t, bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)a, (const bf16_t*)b, (bf16_t*)out, g,
                                                              vec);
  return launch_status("add_broadcast_kernel");
}

size_t mtf_reduce_local_workspace_bytes(const mtf_shape* in_local, const mtf_shape* out_local) {
  Dims din, dout;
  if (check_reduce_shapes(in_local, out_local, &din, &dout)) return 0;
  return plan_reduce(din, dout).workspace;
}

// Shared body of mtf_reduce_local and mtf_reduce_local_static.  use_static: the chunk partials go
// to the library's static device array instead of `workspace`.
static int reduce_local_impl(const void* in, const mtf_shape* in_local, void* out, const mtf_shape* out_local,
                             mtf_dtype in_dt, mtf_dtype out_dt, mtf_reduce_op op, bool use_static, void* workspace,
                             size_t workspace_bytes, void* stream) {
  Dims din, dout;
  if (int rc = check_reduce_shapes(in_local, out_local, &din, &dout)) return rc;
  if (!in || !out) return fail(MTF_ERR_NULL, "in / out");
  if ((in_dt != MTF_F32 && in_dt != MTF_BF16) || (out_dt != MTF_F32 && out_dt != MTF_BF16))
    return fail(MTF_ERR_UNSUPPORTED, "dtype");
  if (op != MTF_REDUCE_SUM && op != MTF_REDUCE_MAX) return fail(MTF_ERR_UNSUPPORTED, "reduction %d", (int)op);
  if (!aligned16(in) || !aligned16(out) || (!use_static && !aligned16(workspace)))
    return fail(MTF_ERR_ALIGN, "in / out / workspace");
  const ReducePlan p = plan_reduce(din, dout);
  if (use_static) {
    if (p.workspace > (size_t)MTF_REDUCE_STATIC_MAX_SCRATCH)
      return fail(MTF_ERR_WORKSPACE,
                  "mtf_reduce_local_static: this reduction needs %zu bytes of scratch, the static buffer holds %zu; "
                  "use mtf_reduce_local with a workspace",
                  p.workspace, (size_t)MTF_REDUCE_STATIC_MAX_SCRATCH);
    workspace = nullptr;
    if (p.workspace > 0)
      if (int rc = static_scratch(&workspace)) return rc;
  } else if (p.workspace > 0 && (!workspace || workspace_bytes < p.workspace)) {
    return fail(MTF_ERR_WORKSPACE, "mtf_reduce_local needs %zu bytes", p.workspace);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (in_dt == MTF_F32 && out_dt == MTF_F32) return run_reduce_op<float, float>(op, in, din, out, dout, p, workspace, s);
  if (in_dt == MTF_F32) return run_reduce_op<float, bf16_t>(op, in, din, out, dout, p, workspace, s);
  if (out_dt == MTF_F32) return run_reduce_op<bf16_t, float>(op, in, din, out, dout, p, workspace, s);
  return run_reduce_op<bf16_t, bf16_t>(op, in, din, out, dout, p, workspace, s);
}

int mtf_reduce_local(const void* in, const mtf_shape* in_local, void* out, const mtf_shape* out_local,
                     mtf_dtype in_dt, mtf_dtype out_dt, mtf_reduce_op op, void* workspace, size_t workspace_bytes,
                     void* stream) {
  return reduce_local_impl(in, in_local, out, out_local, in_dt, out_dt, op, false, workspace, workspace_bytes, stream);
}

int mtf_reduce_local_static(const void* in, const mtf_shape* in_local, void* out, const mtf_shape* out_local,
                            mtf_dtype in_dt, mtf_dtype out_dt, mtf_reduce_op op, void* stream) {
  return reduce_local_impl(in, in_local, out, out_local, in_dt, out_dt, op, true, nullptr, 0, stream);
}

}  // extern "C"
