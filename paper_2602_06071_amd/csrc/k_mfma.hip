// placeholder until the matrix-core path lands
#include "handle.h"
namespace fs {
bool mfma_supported(const SketchParams&, const void*, int64_t, int64_t, const void*, int64_t, fs_dtype) { return false; }
size_t mfma_workspace_bytes(const SketchParams&, int64_t, fs_dtype) { return 0; }
hipError_t launch_mfma(const SketchParams&, const void*, int64_t, int64_t, void*, int64_t, fs_dtype, void*, hipStream_t) { return hipErrorNotSupported; }
}
