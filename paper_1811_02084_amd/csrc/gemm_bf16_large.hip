// Instantiations of the bf16 MFMA GEMM kernel for one tile shape (LargeTile, see gemm_bf16_kernel.h).
#include "gemm_bf16_kernel.h"

namespace mtf {

int launch_large(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s) {
  return launch_cfg<LargeTile>(d, a, batch, s);
}

}  // namespace mtf
