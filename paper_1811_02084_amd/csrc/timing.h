// Optional per-launch timing with HIP events (measurement aid behind mtf_timing_*).
#pragma once
#include <hip/hip_runtime.h>

namespace mtf {

// Brackets one kernel launch with two events on `stream` when timing is enabled; otherwise free.
// `kind` must be a string with static storage duration (kernel name as a profiler prints it).
class LaunchTimer {
 public:
  LaunchTimer(const char* kind, double flops, double bytes, hipStream_t stream);
  ~LaunchTimer();
  LaunchTimer(const LaunchTimer&) = delete;
  LaunchTimer& operator=(const LaunchTimer&) = delete;

 private:
  int slot_;
  hipStream_t stream_;
};

}  // namespace mtf
