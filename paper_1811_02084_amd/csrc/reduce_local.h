// Column reduction used by the fixed layer steps (the local part of reduce_sum over the token
// dims: gradient of a broadcast bias).
#pragma once
#include <hip/hip_runtime.h>

#include "device_common.h"

namespace mtf {

// Scratch the column reduction of an [rows, cols] matrix needs (bytes).
size_t reduce_cols_workspace_bytes(int64_t rows, int64_t cols);

// out[c] = sum_r in[r, c], fp32 accumulation in a fixed order.  cols % 8 == 0.
int reduce_cols_sum(const bf16_t* in, float* out, int64_t rows, int64_t cols, void* workspace,
                    size_t workspace_bytes, hipStream_t stream);

}  // namespace mtf
