// Matrix-core BlockPerm apply: the element-wise-load instantiations for bf16 inputs whose rows
// are not aligned to 4 columns (kernels in k_mfma_kernel.h).
#include "k_mfma_kernel.h"

namespace fs {

hipError_t launch_mfma_bf16_unal(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st) {
  return pl.in_stat ? launch_shape_unal<uint16_t, true>(pl, a, grid, st) : launch_shape_unal<uint16_t, false>(pl, a, grid, st);
}

}  // namespace fs
