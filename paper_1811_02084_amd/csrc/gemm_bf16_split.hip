// Instantiations of the bf16 MFMA GEMM kernel for one tile shape (SplitTile, see gemm_bf16_kernel.h).
#include "gemm_bf16_kernel.h"

namespace mtf {

int launch_split(const GemmDesc& d, const GemmArgs& a, int batch, hipStream_t s) {
  return launch_cfg<SplitTile>(d, a, batch, s);
}

}  // namespace mtf
