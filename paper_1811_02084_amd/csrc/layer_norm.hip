// Layer normalisation over d_model (gfx950): y = gain * (x - mean) / sqrt(var + eps) + bias, forward
// and backward, alone or as the tail of the pass that adds a sublayer's partial sums to the
// residual.  In the paper's terms (section "Operation Implementation") two reductions over d_model
// and component-wise operations with implicit broadcasting; d_model is unsplit, so both reductions
// are local.  HBM-bound: one wavefront per row, the row kept in registers between the passes
// (sum, squared deviations, output), every access 16 bytes per lane.
#include <algorithm>
#include <type_traits>

#include "device_common.h"
#include "timing.h"

namespace mtf {
namespace {

constexpr int kMaxParts = 4;
constexpr int kWaves = 4;             // waves (= rows in flight) per workgroup
constexpr int kChunk = 512;           // elements a wave covers per step: 64 lanes x 8

struct NormParts {
  const float* p[kMaxParts];
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);  // fixed order: the same bits in every lane
  return v;
}

__device__ __forceinline__ void unpack8(const uint4& r, float* v) {
  v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
  v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
  v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xffff0000u);
  v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xffff0000u);
}

__device__ __forceinline__ uint4 pack8(const float* v) {
  return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                    pack_bf16x2(v[6], v[7]));
}

// A wave's share of a [d] parameter vector: chunk c, lane l -> elements (c * 64 + l) * 8 .. + 8.
template <int NC>
__device__ __forceinline__ void load_param(const bf16_t* p, int d, int lane, float (*v)[8]) {
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int e = (c * 64 + lane) * 8;
    if (e < d) {
      unpack8(*reinterpret_cast<const uint4*>(p + e), v[c]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[c][i] = 0.f;
    }
  }
}

// One wave per row.  NC = chunks of 512 elements a row needs (d <= NC * 512, d % 8 == 0); NP =
// partial sums added to the residual first (0: `residual` is the tensor to normalise).
template <int NC, int NP>
__global__ void __launch_bounds__(kWaves * 64) layer_norm_fwd_kernel(
    NormParts parts, const bf16_t* __restrict__ residual, const bf16_t* __restrict__ gain,
    const bf16_t* __restrict__ bias, float eps, int64_t rows, int d, bf16_t* __restrict__ u,
    bf16_t* __restrict__ y, float* __restrict__ mean_out, float* __restrict__ rstd_out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float g[NC][8], b[NC][8];
  load_param<NC>(gain, d, lane, g);
  load_param<NC>(bias, d, lane, b);
  const float inv_d = 1.f / (float)d;
  for (int64_t row = (int64_t)blockIdx.x * kWaves + wave; row < rows; row += (int64_t)gridDim.x * kWaves) {
    const int64_t base = row * d;
    float v[NC][8];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int e = (c * 64 + lane) * 8;
      if (e < d) {
        unpack8(*reinterpret_cast<const uint4*>(residual + base + e), v[c]);
        if (NP > 0) {
          // fixed order: residual, then partial 0, 1, ...; the sum is stored in bf16 and it is the
          // stored value that gets normalised
#pragma unroll
          for (int p = 0; p < NP; ++p) {
            const float4 lo = *reinterpret_cast<const float4*>(parts.p[p] + base + e);
            const float4 hi = *reinterpret_cast<const float4*>(parts.p[p] + base + e + 4);
            v[c][0] += lo.x; v[c][1] += lo.y; v[c][2] += lo.z; v[c][3] += lo.w;
            v[c][4] += hi.x; v[c][5] += hi.y; v[c][6] += hi.z; v[c][7] += hi.w;
          }
          const uint4 stored = pack8(v[c]);
          if (u) *reinterpret_cast<uint4*>(u + base + e) = stored;
          unpack8(stored, v[c]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) sum += v[c][i];
      }
    }
    const float mean = wave_sum(sum) * inv_d;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int e = (c * 64 + lane) * 8;
      if (e < d) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          v[c][i] -= mean;
          sq += v[c][i] * v[c][i];
        }
      }
    }
    const float rstd = 1.f / sqrtf(wave_sum(sq) * inv_d + eps);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int e = (c * 64 + lane) * 8;
      if (e < d) {
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = fmaf(v[c][i] * rstd, g[c][i], b[c][i]);
        *reinterpret_cast<uint4*>(y + base + e) = pack8(o);
      }
    }
    if (lane == 0) {
      mean_out[row] = mean;
      rstd_out[row] = rstd;
    }
  }
}

// Backward: dx per row; per-workgroup column partials of dgain = sum_rows dy * xhat and
// dbias = sum_rows dy go to ws[workgroup][2][d] (waves combined through LDS in wave order).
template <int NC>
__global__ void __launch_bounds__(kWaves * 64) layer_norm_bwd_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ gain, const float* __restrict__ mean_in,
    const float* __restrict__ rstd_in, const bf16_t* __restrict__ dy, int64_t rows, int d,
    bf16_t* __restrict__ dx, float* __restrict__ ws) {
  __shared__ float comb[2][NC * kChunk];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float g[NC][8], dg[NC][8], db[NC][8];
  load_param<NC>(gain, d, lane, g);
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) dg[c][i] = db[c][i] = 0.f;
  const float inv_d = 1.f / (float)d;
  for (int64_t row = (int64_t)blockIdx.x * kWaves + wave; row < rows; row += (int64_t)gridDim.x * kWaves) {
    const int64_t base = row * d;
    const float mean = mean_in[row], rstd = rstd_in[row];
    float xh[NC][8], gy[NC][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int e = (c * 64 + lane) * 8;
      if (e < d) {
        float t[8];
        unpack8(*reinterpret_cast<const uint4*>(x + base + e), xh[c]);
        unpack8(*reinterpret_cast<const uint4*>(dy + base + e), t);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          xh[c][i] = (xh[c][i] - mean) * rstd;
          dg[c][i] = fmaf(t[i], xh[c][i], dg[c][i]);
          db[c][i] += t[i];
          gy[c][i] = t[i] * g[c][i];
          s1 += gy[c][i];
          s2 = fmaf(gy[c][i], xh[c][i], s2);
        }
      }
    }
    const float c1 = wave_sum(s1) * inv_d, c2 = wave_sum(s2) * inv_d;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int e = (c * 64 + lane) * 8;
      if (e < d) {
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = rstd * (gy[c][i] - c1 - xh[c][i] * c2);
        *reinterpret_cast<uint4*>(dx + base + e) = pack8(o);
      }
    }
  }
  // waves add their column partials in wave order
  for (int w = 0; w < kWaves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int e = (c * 64 + lane) * 8 + i;
          comb[0][e] = (w == 0 ? 0.f : comb[0][e]) + dg[c][i];
          comb[1][e] = (w == 0 ? 0.f : comb[1][e]) + db[c][i];
        }
    }
    __syncthreads();
  }
  float* out = ws + (int64_t)blockIdx.x * 2 * d;
  for (int e = threadIdx.x; e < d; e += kWaves * 64) {
    out[e] = comb[0][e];
    out[d + e] = comb[1][e];
  }
}

// dgain[c], dbias[c] = sum over the workgroup partials in a fixed association: 16 threads per
// column each add every 16th partial (their loads independent of one another: the pass is all
// latency), then the 16 sums are added in order.  One workgroup per 16 columns of [dgain | dbias].
__global__ void __launch_bounds__(256) layer_norm_bwd_combine_kernel(const float* __restrict__ ws, int groups, int d,
                                                                    float* __restrict__ dgain, float* __restrict__ dbias) {
  __shared__ float part[16][17];
  const int col = threadIdx.x & 15, slice = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + col;  // 2 * d is a multiple of 16
  float acc = 0.f;
#pragma unroll 8
  for (int gidx = slice; gidx < groups; gidx += 16) acc += ws[(int64_t)gidx * 2 * d + c];
  part[slice][col] = acc;
  __syncthreads();
  if (slice == 0) {
    float total = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) total += part[i][col];
    if (c < d)
      dgain[c] = total;
    else
      dbias[c - d] = total;
  }
}

int chunks_for(int64_t d) {
  for (int nc = 1; nc <= 8; nc *= 2)
    if (d <= (int64_t)nc * kChunk) return nc;
  return 0;
}

int check_norm_dims(int64_t rows, int64_t d) {
  if (rows < 0 || d <= 0) return fail(MTF_ERR_SIZE_MISMATCH, "layer norm over [%lld, %lld]", (long long)rows, (long long)d);
  if (d % 8 || chunks_for(d) == 0)
    return fail(MTF_ERR_UNSUPPORTED, "layer norm needs d_model %% 8 == 0 and d_model <= 4096, not %lld", (long long)d);
  return MTF_OK;
}

int bwd_groups(int64_t rows) { return (int)std::min<int64_t>(ceil_div(std::max<int64_t>(rows, 1), kWaves), 512); }

template <int NC>
void launch_fwd(int np, int blocks, hipStream_t s, const NormParts& pp, const bf16_t* res, const bf16_t* gain,
                const bf16_t* bias, float eps, int64_t rows, int d, bf16_t* u, bf16_t* y, float* mean, float* rstd) {
  switch (np) {
    case 0: layer_norm_fwd_kernel<NC, 0><<<blocks, kWaves * 64, 0, s>>>(pp, res, gain, bias, eps, rows, d, u, y, mean, rstd); break;
    case 1: layer_norm_fwd_kernel<NC, 1><<<blocks, kWaves * 64, 0, s>>>(pp, res, gain, bias, eps, rows, d, u, y, mean, rstd); break;
    case 2: layer_norm_fwd_kernel<NC, 2><<<blocks, kWaves * 64, 0, s>>>(pp, res, gain, bias, eps, rows, d, u, y, mean, rstd); break;
    case 3: layer_norm_fwd_kernel<NC, 3><<<blocks, kWaves * 64, 0, s>>>(pp, res, gain, bias, eps, rows, d, u, y, mean, rstd); break;
    default: layer_norm_fwd_kernel<NC, 4><<<blocks, kWaves * 64, 0, s>>>(pp, res, gain, bias, eps, rows, d, u, y, mean, rstd); break;
  }
}

int norm_fwd(const void* const* partials, int n, const void* residual, const void* gain, const void* bias, float eps,
             int64_t rows, int64_t d, void* u, void* y, void* mean, void* rstd, void* stream) {
  if (int rc = check_norm_dims(rows, d)) return rc;
  if (n < 0 || n > kMaxParts) return fail(MTF_ERR_UNSUPPORTED, "%d partial sums (0..%d)", n, kMaxParts);
  if (!(eps >= 0.f)) return fail(MTF_ERR_UNSUPPORTED, "eps %g", (double)eps);
  if (rows == 0) return MTF_OK;
  if (!residual || !gain || !bias || !y || !mean || !rstd || (n > 0 && (!partials || !u)))
    return fail(MTF_ERR_NULL, "layer norm buffer");
  NormParts pp{};
  for (int i = 0; i < n; ++i) {
    if (!partials[i]) return fail(MTF_ERR_NULL, "partial %d", i);
    if (!aligned16(partials[i])) return fail(MTF_ERR_ALIGN, "partial %d", i);
    pp.p[i] = static_cast<const float*>(partials[i]);
  }
  for (const void* p : {residual, gain, bias, (const void*)u, (const void*)y, (const void*)mean, (const void*)rstd})
    if (!aligned16(p)) return fail(MTF_ERR_ALIGN, "layer norm buffer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int blocks = (int)std::min<int64_t>(ceil_div(rows, kWaves), 256 * 8);
  const double bytes = (double)rows * d * (2.0 + 4.0 * n + (n > 0 ? 2.0 : 0.0) + 2.0) + 8.0 * rows;
  LaunchTimer timer("layer_norm_fwd_kernel", 0, bytes, s);
  auto go = [&](auto nc) {
    launch_fwd<decltype(nc)::value>(n, blocks, s, pp, static_cast<const bf16_t*>(residual),
                                    static_cast<const bf16_t*>(gain), static_cast<const bf16_t*>(bias), eps, rows,
                                    (int)d, static_cast<bf16_t*>(u), static_cast<bf16_t*>(y),
                                    static_cast<float*>(mean), static_cast<float*>(rstd));
  };
  switch (chunks_for(d)) {
    case 1: go(std::integral_constant<int, 1>{}); break;
    case 2: go(std::integral_constant<int, 2>{}); break;
    case 4: go(std::integral_constant<int, 4>{}); break;
    default: go(std::integral_constant<int, 8>{}); break;
  }
  return launch_status("layer_norm_fwd_kernel");
}

}  // namespace
}  // namespace mtf

using namespace mtf;

extern "C" {

int mtf_layer_norm_fwd(const void* x, const void* gain, const void* bias, float eps, int64_t rows,
                       int64_t d_model, void* y, void* mean, void* rstd, void* stream) {
  return norm_fwd(nullptr, 0, x, gain, bias, eps, rows, d_model, nullptr, y, mean, rstd, stream);
}

int mtf_residual_layer_norm_fwd(const void* const* partials, int32_t n, const void* residual,
                                const void* gain, const void* bias, float eps, int64_t rows,
                                int64_t d_model, void* u, void* y, void* mean, void* rstd, void* stream) {
  if (n < 1) return fail(MTF_ERR_UNSUPPORTED, "%d partial sums (1..%d)", n, kMaxParts);
  return norm_fwd(partials, n, residual, gain, bias, eps, rows, d_model, u, y, mean, rstd, stream);
}

size_t mtf_layer_norm_bwd_workspace_bytes(int64_t rows, int64_t d_model) {
  if (rows < 0 || d_model <= 0) return 0;
  return (size_t)bwd_groups(rows) * 2 * (size_t)d_model * 4;
}

int mtf_layer_norm_bwd(const void* x, const void* gain, const void* mean, const void* rstd,
                       const void* dy, int64_t rows, int64_t d_model, void* dx, void* dgain,
                       void* dbias, void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_norm_dims(rows, d_model)) return rc;
  if (!dgain || !dbias) return fail(MTF_ERR_NULL, "dgain / dbias");
  if (rows > 0 && (!x || !gain || !mean || !rstd || !dy || !dx)) return fail(MTF_ERR_NULL, "layer norm buffer");
  for (const void* p : {x, gain, mean, rstd, dy, (const void*)dx, (const void*)dgain, (const void*)dbias,
                        (const void*)workspace})
    if (!aligned16(p)) return fail(MTF_ERR_ALIGN, "layer norm buffer");
  const size_t need = mtf_layer_norm_bwd_workspace_bytes(rows, d_model);
  if (rows > 0 && (!workspace || workspace_bytes < need))
    return fail(MTF_ERR_WORKSPACE, "mtf_layer_norm_bwd needs %zu bytes", need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int d = (int)d_model;
  const int groups = rows > 0 ? bwd_groups(rows) : 0;
  if (groups > 0) {
    LaunchTimer timer("layer_norm_bwd_kernel", 0, (double)rows * d * 6.0 + 8.0 * rows + (double)groups * 2 * d * 4, s);
    auto go = [&](auto nc) {
      layer_norm_bwd_kernel<decltype(nc)::value><<<groups, kWaves * 64, 0, s>>>(
          static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(gain), static_cast<const float*>(mean),
          static_cast<const float*>(rstd), static_cast<const bf16_t*>(dy), rows, d, static_cast<bf16_t*>(dx),
          static_cast<float*>(workspace));
    };
    switch (chunks_for(d_model)) {
      case 1: go(std::integral_constant<int, 1>{}); break;
      case 2: go(std::integral_constant<int, 2>{}); break;
      case 4: go(std::integral_constant<int, 4>{}); break;
      default: go(std::integral_constant<int, 8>{}); break;
    }
    if (int rc = launch_status("layer_norm_bwd_kernel")) return rc;
  }
  {
    LaunchTimer timer("layer_norm_bwd_combine_kernel", 0, (double)groups * 2 * d * 4 + 8.0 * d, s);
    layer_norm_bwd_combine_kernel<<<2 * d / 16, 256, 0, s>>>(static_cast<const float*>(workspace), groups, d,
                                                                          static_cast<float*>(dgain),
                                                                          static_cast<float*>(dbias));
  }
  return launch_status("layer_norm_bwd_combine_kernel");
}

}  // extern "C"
