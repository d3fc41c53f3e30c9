// Matrix-core BlockPerm apply: the instantiations for bf16 inputs (kernels in k_mfma_kernel.h).
#include "k_mfma_kernel.h"

namespace fs {

hipError_t launch_mfma_bf16(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st) {
  return pl.in_stat ? launch_shape<uint16_t, true>(pl, a, grid, st) : launch_shape<uint16_t, false>(pl, a, grid, st);
}

}  // namespace fs
