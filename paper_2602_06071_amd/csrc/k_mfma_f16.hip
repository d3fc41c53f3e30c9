// Matrix-core BlockPerm apply: the instantiations for f16 inputs (kernels in k_mfma_kernel.h).
#include "k_mfma_kernel.h"

namespace fs {

hipError_t launch_mfma_f16(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st) {
  return pl.in_stat ? launch_shape<f16, true>(pl, a, grid, st) : launch_shape<f16, false>(pl, a, grid, st);
}

}  // namespace fs
