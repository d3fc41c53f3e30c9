// fs_sketch_apply_static: the column-layout apply for callers that cannot allocate device
// memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// The device memory the kernels of one apply use beyond A and out -- the fp32 partial planes of
// the input-stationary decomposition (or the fp32 accumulator of the scatter baseline), and
// behind them the orbit table of the handle's wiring -- lives in a file-scope device array
// instead of an allocation.  Every device that loads the library holds its own copy of the
// array until the process ends.  In host code `scratch` is only the host-side name of that
// symbol, not a device address: the address on the current device comes from
// hipGetSymbolAddress, once per device, and only that address is handed to kernels.
#include "handle.h"

namespace {

constexpr size_t kPlaneBytes = (size_t)FS_STATIC_SCRATCH_BYTES;
constexpr size_t kOrbitBytes = (size_t)1 << 20;  // room for orbit tables up to M = 2^17
constexpr int kMaxDevices = 64;

unsigned char* g_scratch_ptr[kMaxDevices];  // device address of `scratch`, per device

}  // namespace

static __device__ __align__(256) unsigned char scratch[kPlaneBytes + kOrbitBytes];

namespace {

// Device address of the array on the current device (looked up on the first call there).
fs_status scratch_ptr(fs_sketch_t h, unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fs::hip_fail(h, e);
  if (dev < 0 || dev >= kMaxDevices) return FS_ERR_UNSUPPORTED;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fs::hip_fail(h, e);
    if (!ptr) return fs::hip_fail(h, hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return FS_OK;
}

}  // namespace

extern "C" fs_status fs_sketch_apply_static(fs_sketch_t h, const void* A, int64_t lda, int64_t n,
                                            void* out, int64_t ldo, fs_dtype dt, void* stream) {
  if (!h) return FS_ERR_INVALID_ARG;
  if (n == 0) return FS_OK;  // (as fs_sketch_apply_ld: nothing to do, no HIP call)
  unsigned char* base = nullptr;
  const fs_status rc = scratch_ptr(h, &base);
  if (rc != FS_OK) return rc;
  fs::ScratchSource src;
  src.external = true;
  src.planes = base;
  src.plane_bytes = kPlaneBytes;
  src.orbit = reinterpret_cast<uint32_t*>(base + kPlaneBytes);
  src.orbit_bytes = kOrbitBytes;
  // Everything the kernels read from the array is written earlier in the same call (every plane
  // tile the reduction adds, the scatter accumulator's zero-fill, the orbit table), so nothing
  // has to be cleared between calls.
  return fs::apply_cols(h, A, lda, n, out, ldo, dt, stream, src);
}
