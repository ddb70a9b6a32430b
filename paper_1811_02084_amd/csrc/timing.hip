// Per-launch kernel timing: every launch made while timing is enabled is bracketed by a pair of
// HIP events recorded on the launch's own stream; mtf_timing_collect() turns them into per-kernel
// totals.  Used by the benchmark to time the dominant kernel inside the timed region.
#include "timing.h"

#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "device_common.h"

namespace mtf {
namespace {

struct Record {
  const char* kind;
  double flops, bytes;
  hipEvent_t start, stop;
};

std::mutex g_mu;
std::atomic<bool> g_enabled{false};  // read without the mutex on every launch
std::vector<Record> g_records;
std::vector<hipEvent_t> g_free_events;

hipEvent_t take_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

}  // namespace

LaunchTimer::LaunchTimer(const char* kind, double flops, double bytes, hipStream_t stream)
    : slot_(-1), stream_(stream) {
  if (!g_enabled.load(std::memory_order_relaxed)) return;  // timing off: no lock, no event
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_enabled.load(std::memory_order_relaxed)) return;
  Record r{kind, flops, bytes, take_event(), take_event()};
  if (!r.start || !r.stop) return;
  (void)hipEventRecord(r.start, stream);
  g_records.push_back(r);
  slot_ = (int)g_records.size() - 1;
}

LaunchTimer::~LaunchTimer() {
  if (slot_ < 0) return;
  std::lock_guard<std::mutex> lock(g_mu);
  if (slot_ < (int)g_records.size()) (void)hipEventRecord(g_records[slot_].stop, stream_);
}

}  // namespace mtf

using namespace mtf;

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

// Nothing but MFMAs: 8 independent accumulators per wave, 4 A and 4 B fragments in rotation so
// that consecutive instructions see different operand bits, as they do in a contraction.
__global__ void __launch_bounds__(256, 2) mfma_ceiling_kernel(const uint16_t* __restrict__ operands, int iters,
                                                             float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8_t a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = *reinterpret_cast<const bf16x8_t*>(operands + (i * 64 + lane) * 8);
    b[i] = *reinterpret_cast<const bf16x8_t*>(operands + 2048 + (i * 64 + lane) * 8);
  }
  f32x16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  const unsigned long long cycles0 = clock64(), ticks0 = wall_clock64();
  for (int it = 0; it < iters; it += 4) {  // 4 rounds per trip keep every register index static
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[(i + r) & 3], acc[i], 0, 0, 0);
  }
  float total = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) total += acc[i][e];
  if (blockIdx.x == 0 && threadIdx.x < 64) sink[threadIdx.x] = total;
  // the loop's span on both clocks (the accumulators above are complete: the sum waited for them)
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    sink[64] = (float)(clock64() - cycles0);
    sink[65] = (float)(wall_clock64() - ticks0);
  }
}

}  // namespace

extern "C" {

int mtf_mfma_ceiling(const void* operands, int32_t iters, void* sink, double* flops, void* stream) {
  if (!operands || !sink || !flops) return fail(MTF_ERR_NULL, "operands / sink / flops");
  if (iters <= 0) return fail(MTF_ERR_SIZE_MISMATCH, "iters %d", iters);
  if (!aligned16(operands)) return fail(MTF_ERR_ALIGN, "operands");
  hipDeviceProp_t prop;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
    return fail(MTF_ERR_HIP, "device properties");
  const int groups = prop.multiProcessorCount * 2;  // 2 workgroups of 4 waves per CU
  const int rounds = (iters + 3) / 4 * 4;  // the kernel runs whole trips of 4
  *flops = 2.0 * 32 * 32 * 16 * 8.0 * rounds * 4.0 * groups;
  hipStream_t s = static_cast<hipStream_t>(stream);
  {
    LaunchTimer timer("mfma_ceiling_kernel", *flops, 0, s);
    mfma_ceiling_kernel<<<groups, 256, 0, s>>>(static_cast<const uint16_t*>(operands), iters,
                                              static_cast<float*>(sink));
  }
  return launch_status("mfma_ceiling_kernel");
}

int mtf_timing_enable(int on) {
  std::lock_guard<std::mutex> lock(g_mu);
  g_enabled.store(on != 0, std::memory_order_relaxed);
  return MTF_OK;
}

int mtf_timing_collect(mtf_kernel_time* out, int32_t max_kinds, int32_t* n_kinds) {
  if (!n_kinds || (max_kinds > 0 && !out)) return fail(MTF_ERR_NULL, "out / n_kinds");
  std::lock_guard<std::mutex> lock(g_mu);
  int n = 0;
  int rc = MTF_OK;
  for (Record& r : g_records) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
    if (e != hipSuccess) rc = hip_fail(e, "timing event");
    g_free_events.push_back(r.start);
    g_free_events.push_back(r.stop);
    if (e != hipSuccess) continue;
    int k = 0;
    while (k < n && std::strcmp(out[k].kernel, r.kind) != 0) ++k;
    if (k == n) {
      if (n >= max_kinds) continue;
      std::memset(&out[n], 0, sizeof out[n]);
      std::strncpy(out[n].kernel, r.kind, sizeof out[n].kernel - 1);
      ++n;
    }
    out[k].launches += 1;
    out[k].total_ms += ms;
    out[k].flops += r.flops;
    out[k].bytes += r.bytes;
  }
  g_records.clear();
  *n_kinds = n;
  return rc;
}

}  // extern "C"
