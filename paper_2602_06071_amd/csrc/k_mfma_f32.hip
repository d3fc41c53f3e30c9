// Matrix-core BlockPerm apply: the instantiations for f32 inputs (kernels in k_mfma_kernel.h).
#include "k_mfma_kernel.h"

namespace fs {

hipError_t launch_mfma_f32(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st) {
  return pl.in_stat ? launch_shape<float, true>(pl, a, grid, st) : launch_shape<float, false>(pl, a, grid, st);
}

}  // namespace fs
