// Vocabulary-split operations of the model-parallel Transformer (section 'Model-Parallel
// "Transformer"': vocab is the third dim split across the mesh), one processor's share:
//   embedding           e = einsum(onehot(ids)[b,l,vocab], E[vocab,D]) on the local vocab stripe
//                       (a row gather; ids outside the stripe contribute 0: a partial sum)
//   embedding gradient  dE = einsum(onehot(ids), de) restricted to the stripe's rows
//   softmax cross-entropy over a split vocab, from the paper's reductions: local reduce_max /
//                       reduce_sum(exp) / the target's logit, combined across the vocab group
//                       by max / sum Allreduces (mtf_max_partials, mtf_reduce_partials), and
//                       the component-wise gradient of the logits.
// All HBM-bound: every logit is read once per pass.
#include <algorithm>

#include "device_common.h"
#include "timing.h"

namespace mtf {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// out[t, :] = table[ids[t] - offset, :] if that row is local, else 0.  One wave per token at a
// time (its id is wave-uniform), 16 bytes of the row per lane.
template <typename OutT>
__global__ void __launch_bounds__(256) embedding_kernel(const int32_t* __restrict__ ids, const bf16_t* __restrict__ table,
                                                       OutT* __restrict__ out, int64_t count, int64_t vocab_local,
                                                       int64_t d_model, int64_t offset) {
  const int lane = threadIdx.x & 63;
  const int chunks = (int)(d_model / 8);
  for (int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); t < count; t += (int64_t)gridDim.x * 4) {
    const int64_t row = (int64_t)ids[t] - offset;
    const bool local = row >= 0 && row < vocab_local;
    const bf16_t* src = table + (local ? row : 0) * d_model;
    for (int c = lane; c < chunks; c += 64) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (local) v = *reinterpret_cast<const u32x4*>(src + c * 8);
      if (sizeof(OutT) == 2) {
        *reinterpret_cast<u32x4*>(out + t * d_model + c * 8) = v;
      } else {
        float* o = reinterpret_cast<float*>(out) + t * d_model + c * 8;
        *reinterpret_cast<float4*>(o) = make_float4(__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xffff0000u),
                                                    __uint_as_float(v[1] << 16), __uint_as_float(v[1] & 0xffff0000u));
        *reinterpret_cast<float4*>(o + 4) = make_float4(__uint_as_float(v[2] << 16), __uint_as_float(v[2] & 0xffff0000u),
                                                        __uint_as_float(v[3] << 16), __uint_as_float(v[3] & 0xffff0000u));
      }
    }
  }
}

// dtable[v, :] = sum over the tokens t with ids[t] == offset + v of de[t, :], in token order (no
// atomics: one workgroup of 2 waves per local vocab row scans all ids, 128 at a time; the hits of
// a block are compacted in ascending order with ballots; a thread owns 8 columns per pass).
__global__ void __launch_bounds__(128) embedding_grad_kernel(const int32_t* __restrict__ ids,
                                                            const bf16_t* __restrict__ de, float* __restrict__ dtable,
                                                            int64_t count, int64_t d_model, int64_t offset) {
  __shared__ int hits[128];
  __shared__ int wave_hits[2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = blockIdx.x;
  const int32_t want = (int32_t)(offset + row);
  const int64_t chunks = d_model / 8;
  for (int64_t c0 = 0; c0 < chunks; c0 += blockDim.x) {  // 8 * 128 columns per pass
    const int64_t c = c0 + threadIdx.x;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int64_t t0 = 0; t0 < count; t0 += 128) {
      const int64_t t = t0 + threadIdx.x;
      const bool hit = t < count && ids[t] == want;
      const uint64_t mask = __ballot(hit);
      if (lane == 0) wave_hits[wave] = __popcll(mask);
      __syncthreads();
      const int first = wave == 0 ? 0 : wave_hits[0];
      const int n = wave_hits[0] + wave_hits[1];
      if (hit) hits[first + __popcll(mask & ((1ull << lane) - 1ull))] = threadIdx.x;
      __syncthreads();
      if (c < chunks)
        for (int h = 0; h < n; ++h) {
          const u32x4 v = *reinterpret_cast<const u32x4*>(de + (t0 + hits[h]) * d_model + c * 8);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[2 * e] += __uint_as_float(v[e] << 16);
            acc[2 * e + 1] += __uint_as_float(v[e] & 0xffff0000u);
          }
        }
      __syncthreads();  // hits / wave_hits are rewritten by the next block of tokens
    }
    if (c < chunks) {
      float* o = dtable + row * d_model + c * 8;
      *reinterpret_cast<float4*>(o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
      *reinterpret_cast<float4*>(o + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
  }
}

struct MaxPtrs {
  const float* p[64];
};
__global__ void __launch_bounds__(256) max_partials_kernel(MaxPtrs in, int n, float* __restrict__ out, int64_t count) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) {
    float m = in.p[0][i];
    for (int k = 1; k < n; ++k) m = fmaxf(m, in.p[k][i]);
    out[i] = m;
  }
}

// One wave per row: sumexp[r] = sum_v exp(z[r,v] - row_max[r]) (lanes stride the row, butterfly in
// a fixed order); picked[r] = z[r, target - offset] if the target is local, else 0.
__global__ void __launch_bounds__(256) xent_stats_kernel(const float* __restrict__ z, const float* __restrict__ row_max,
                                                        const int32_t* __restrict__ targets,
                                                        float* __restrict__ sumexp, float* __restrict__ picked,
                                                        int64_t rows, int64_t vocab_local, int64_t offset) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const float m = row_max[r];
  const float* zr = z + r * vocab_local;
  float acc = 0.f;
  if (vocab_local % 4 == 0) {  // rows are 16-byte aligned then
    for (int64_t v = lane * 4; v < vocab_local; v += 256) {
      const float4 q = *reinterpret_cast<const float4*>(zr + v);
      acc += (__expf(q.x - m) + __expf(q.y - m)) + (__expf(q.z - m) + __expf(q.w - m));
    }
  } else {
    for (int64_t v = lane; v < vocab_local; v += 64) acc += __expf(zr[v] - m);
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) acc += __shfl_xor(acc, s);
  if (lane == 0) {
    sumexp[r] = acc;
    const int64_t t = (int64_t)targets[r] - offset;
    picked[r] = (t >= 0 && t < vocab_local) ? zr[t] : 0.f;
  }
}

__global__ void __launch_bounds__(256) xent_loss_kernel(const float* __restrict__ row_max, const float* __restrict__ sumexp,
                                                       const float* __restrict__ picked, float* __restrict__ loss,
                                                       int64_t rows) {
  const int64_t r = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (r < rows) loss[r] = row_max[r] + __logf(sumexp[r]) - picked[r];
}

// dz[r,v] = (exp(z[r,v] - row_max[r]) / sumexp[r] - [offset + v == targets[r]]) * dloss[r], bf16.
// 4 logits per thread.
__global__ void __launch_bounds__(256) xent_grad_kernel(const float* __restrict__ z, const float* __restrict__ row_max,
                                                       const float* __restrict__ sumexp,
                                                       const int32_t* __restrict__ targets,
                                                       const float* __restrict__ dloss, bf16_t* __restrict__ dz,
                                                       int64_t rows, int64_t vocab_local, int64_t offset) {
  const int64_t quads = vocab_local / 4;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < rows * quads;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / quads, v0 = (i % quads) * 4;
    const float m = row_max[r], inv = 1.f / sumexp[r], g = dloss[r];
    const int64_t t = (int64_t)targets[r] - offset;
    const float4 zz = *reinterpret_cast<const float4*>(z + r * vocab_local + v0);
    const float x[4] = {zz.x, zz.y, zz.z, zz.w};
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (__expf(x[e] - m) * inv - (v0 + e == t ? 1.f : 0.f)) * g;
    *reinterpret_cast<uint2*>(dz + r * vocab_local + v0) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
  }
}

int grid_for(int64_t items) { return (int)std::min<int64_t>(ceil_div(items, 256), 256 * 32); }

}  // namespace
}  // namespace mtf

using namespace mtf;

extern "C" {

int mtf_embedding_local(const void* ids, int64_t count, const void* table_local, int64_t vocab_local,
                        int64_t d_model, int64_t vocab_offset, void* out_partial, mtf_dtype out_dt, void* stream) {
  if (count < 0 || vocab_local <= 0 || d_model <= 0 || vocab_offset < 0)
    return fail(MTF_ERR_SIZE_MISMATCH, "embedding sizes");
  if (d_model % 8) return fail(MTF_ERR_UNSUPPORTED, "embedding needs d_model divisible by 8");
  if (out_dt != MTF_F32 && out_dt != MTF_BF16) return fail(MTF_ERR_UNSUPPORTED, "dtype");
  if (count == 0) return MTF_OK;
  if (!ids || !table_local || !out_partial) return fail(MTF_ERR_NULL, "ids / table / out");
  if (!aligned16(table_local) || !aligned16(out_partial) || ((uintptr_t)ids & 3)) return fail(MTF_ERR_ALIGN, "embedding buffers");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const double bytes = (double)count * d_model * (2 + (out_dt == MTF_BF16 ? 2 : 4)) + 4.0 * count;
  LaunchTimer timer("embedding_kernel", 0, bytes, s);
  const int blocks = (int)std::min<int64_t>(ceil_div(count, 4), 256 * 16);
  if (out_dt == MTF_BF16)
    embedding_kernel<bf16_t><<<blocks, 256, 0, s>>>((const int32_t*)ids, (const bf16_t*)table_local, (bf16_t*)out_partial,
                                                  count, vocab_local, d_model, vocab_offset);
  else
    embedding_kernel<float><<<blocks, 256, 0, s>>>((const int32_t*)ids, (const bf16_t*)table_local, (float*)out_partial,
                                                 count, vocab_local, d_model, vocab_offset);
  return launch_status("embedding_kernel");
}

int mtf_embedding_grad_local(const void* ids, int64_t count, const void* de, int64_t vocab_local, int64_t d_model,
                             int64_t vocab_offset, void* dtable_local, void* stream) {
  if (count < 0 || vocab_local <= 0 || d_model <= 0 || vocab_offset < 0)
    return fail(MTF_ERR_SIZE_MISMATCH, "embedding sizes");
  if (d_model % 8) return fail(MTF_ERR_UNSUPPORTED, "embedding needs d_model divisible by 8");
  if (vocab_local > INT32_MAX) return fail(MTF_ERR_UNSUPPORTED, "vocab_local too large");
  if (!dtable_local || (count > 0 && (!ids || !de))) return fail(MTF_ERR_NULL, "ids / de / dtable");
  if (!aligned16(de) || !aligned16(dtable_local) || ((uintptr_t)ids & 3)) return fail(MTF_ERR_ALIGN, "embedding buffers");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const double bytes = (double)vocab_local * d_model * 4 + (double)count * d_model * 2;
  LaunchTimer timer("embedding_grad_kernel", 0, bytes, s);
  embedding_grad_kernel<<<(unsigned)vocab_local, 128, 0, s>>>((const int32_t*)ids, (const bf16_t*)de, (float*)dtable_local,
                                                             count, d_model, vocab_offset);
  return launch_status("embedding_grad_kernel");
}

int mtf_max_partials(const void* const* partials, int32_t n, void* out, int64_t count, void* stream) {
  if (!partials || n < 1 || n > 64) return fail(MTF_ERR_NULL, "partials (1..64 buffers)");
  if (count < 0) return fail(MTF_ERR_SIZE_MISMATCH, "count %lld", (long long)count);
  if (count == 0) return MTF_OK;
  if (!out) return fail(MTF_ERR_NULL, "out");
  MaxPtrs p{};
  for (int i = 0; i < n; ++i) {
    if (!partials[i]) return fail(MTF_ERR_NULL, "partials[%d]", i);
    p.p[i] = static_cast<const float*>(partials[i]);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  LaunchTimer timer("max_partials_kernel", 0, 4.0 * (n + 1) * count, s);
  max_partials_kernel<<<grid_for(count), 256, 0, s>>>(p, n, static_cast<float*>(out), count);
  return launch_status("max_partials_kernel");
}

int mtf_xent_stats_local(const void* logits_local, int64_t rows, int64_t vocab_local, const void* row_max,
                         const void* targets, int64_t vocab_offset, void* sumexp, void* picked, void* stream) {
  if (rows < 0 || vocab_local <= 0 || vocab_offset < 0) return fail(MTF_ERR_SIZE_MISMATCH, "loss sizes");
  if (rows == 0) return MTF_OK;
  if (!logits_local || !row_max || !targets || !sumexp || !picked) return fail(MTF_ERR_NULL, "loss buffers");
  if (!aligned16(logits_local)) return fail(MTF_ERR_ALIGN, "logits_local");  // 16-byte row loads
  hipStream_t s = static_cast<hipStream_t>(stream);
  LaunchTimer timer("xent_stats_kernel", 0, 4.0 * rows * vocab_local + 16.0 * rows, s);
  xent_stats_kernel<<<(unsigned)ceil_div(rows, 4), 256, 0, s>>>((const float*)logits_local, (const float*)row_max,
                                                               (const int32_t*)targets, (float*)sumexp, (float*)picked,
                                                               rows, vocab_local, vocab_offset);
  return launch_status("xent_stats_kernel");
}

int mtf_xent_loss(const void* row_max, const void* sumexp, const void* picked, void* loss, int64_t rows, void* stream) {
  if (rows < 0) return fail(MTF_ERR_SIZE_MISMATCH, "rows");
  if (rows == 0) return MTF_OK;
  if (!row_max || !sumexp || !picked || !loss) return fail(MTF_ERR_NULL, "loss buffers");
  hipStream_t s = static_cast<hipStream_t>(stream);
  xent_loss_kernel<<<(unsigned)ceil_div(rows, 256), 256, 0, s>>>((const float*)row_max, (const float*)sumexp,
                                                                (const float*)picked, (float*)loss, rows);
  return launch_status("xent_loss_kernel");
}

int mtf_xent_grad_local(const void* logits_local, int64_t rows, int64_t vocab_local, const void* row_max,
                        const void* sumexp, const void* targets, int64_t vocab_offset, const void* dloss,
                        void* dlogits_local, void* stream) {
  if (rows < 0 || vocab_local <= 0 || vocab_offset < 0) return fail(MTF_ERR_SIZE_MISMATCH, "loss sizes");
  if (vocab_local % 4) return fail(MTF_ERR_UNSUPPORTED, "loss gradient needs vocab_local divisible by 4");
  if (rows == 0) return MTF_OK;
  if (!logits_local || !row_max || !sumexp || !targets || !dloss || !dlogits_local)
    return fail(MTF_ERR_NULL, "loss buffers");
  if (!aligned16(logits_local) || !aligned16(dlogits_local)) return fail(MTF_ERR_ALIGN, "logits / dlogits");
  hipStream_t s = static_cast<hipStream_t>(stream);
  LaunchTimer timer("xent_grad_kernel", 0, 6.0 * rows * vocab_local + 16.0 * rows, s);
  xent_grad_kernel<<<grid_for(rows * (vocab_local / 4)), 256, 0, s>>>(
      (const float*)logits_local, (const float*)row_max, (const float*)sumexp, (const int32_t*)targets,
      (const float*)dloss, (bf16_t*)dlogits_local, rows, vocab_local, vocab_offset);
  return launch_status("xent_grad_kernel");
}

}  // extern "C"
