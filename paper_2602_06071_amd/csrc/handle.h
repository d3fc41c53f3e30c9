// Host-side handle and the launchers each kernel file provides.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/flashsketch.h"

// Plain-old-data view of a sketch that kernels take by value.
struct SketchParams {
  int64_t d, k;
  uint32_t Bc, Br, kappa, s, M;
  uint32_t a, b, a_inv;
  uint32_t key1;
  uint32_t br_pow2;  // 1 when Br is a power of two
  float scale;
};

struct fs_sketch_s {
  SketchParams p;
  uint32_t key0;
  int kind;
  int variant;
  int last_variant;
  int last_mode;
  int last_hip_error;
  char last_kernel[64];  // which kernel instantiation the most recent apply launched
  int device;  // device that owns ws / dense (-1: none yet)
  // internal or caller-owned workspace
  void* ws;
  size_t ws_bytes;
  bool ws_owned;
  // optional events of each apply: begin / end around everything it enqueues, start / stop
  // around its dominant kernel
  bool profiling;
  int prof_used;
  int prof_scope;  // FS_PROFILE_KERNEL | FS_PROFILE_APPLY
  std::vector<hipEvent_t> prof_begin, prof_start, prof_stop, prof_end;
  // orbit order of the blocks under the wiring map (2*M words, device), built on first use
  uint32_t* orbit;
  // GAUSS_DENSE: the k x d matrix in its fp32 and bf16 forms (one allocation)
  void* dense;
};

namespace fs {

// Optional event pair recorded immediately before / after the dominant kernel.
struct EventPair {
  hipEvent_t start = nullptr, stop = nullptr;
};

// Where the kernels of one column-layout apply find their scratch memory (partial planes or the
// scatter accumulator, and the orbit table of the wiring).  Default: the handle's own or attached
// workspace and its own table.  external: memory supplied for this call only -- `planes`
// (256-byte aligned, plane_bytes long) and room for an orbit table that is rebuilt on every call
// (orbit_bytes; a longer wiring runs without a table); nothing is then allocated.
struct ScratchSource {
  bool external = false;
  void* planes = nullptr;
  size_t plane_bytes = 0;
  uint32_t* orbit = nullptr;
  size_t orbit_bytes = 0;
};
// Argument checks, variant choice and launches of fs_sketch_apply_ld, on `src`'s memory.
fs_status apply_cols(fs_sketch_t h, const void* A, int64_t lda, int64_t n, void* out, int64_t ldo,
                     fs_dtype dt, void* stream, const ScratchSource& src);
// Records a failed HIP call in the handle, clears the sticky error, returns FS_ERR_HIP.
fs_status hip_fail(fs_sketch_t h, hipError_t e);

// Each launcher validates nothing: api.hip has already checked every argument
// and that the shape fits the kernel.  They return the launch's hipError_t.

hipError_t launch_export(const SketchParams& p, int32_t* rows, int8_t* signs, hipStream_t st);
// Fills tab (2*M words, device) with the orbit of the wiring map from block 0 and its inverse.
hipError_t launch_orbit(const SketchParams& p, uint32_t* tab, hipStream_t st);

// One lane per column, LDS-private output tile.
hipError_t launch_generic(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                          int64_t ldo, fs_dtype dt, hipStream_t st, EventPair ev);
hipError_t launch_generic_rows(const SketchParams& p, const void* G, int64_t ldg, int64_t n, void* out,
                               int64_t ldo, fs_dtype dt, hipStream_t st, EventPair ev);

// Matrix-core path.  ws holds the per-slot partial tiles.
bool mfma_supported(const SketchParams& p, const void* A, int64_t lda, int64_t n, const void* out,
                    int64_t ldo, fs_dtype dt);
size_t mfma_workspace_bytes(const SketchParams& p, int64_t n, fs_dtype dt);
// orbit: device array of 2*M words (block at each orbit position of the wiring map
// starting from block 0, then the inverse), or NULL.
bool mfma_wants_orbit(const SketchParams& p);
// What launch_mfma would do, without launching (pure host work): mode 1 output-stationary, 2
// input-stationary, 3 the same with orbit runs; flags as in fs_plan_flags.  False: unsupported.
bool mfma_describe(const SketchParams& p, const void* A, int64_t lda, int64_t n, fs_dtype dt,
                   bool have_orbit, int* mode, int* flags, size_t* workspace);
hipError_t launch_mfma(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                       int64_t ldo, fs_dtype dt, void* ws, const uint32_t* orbit, hipStream_t st,
                       EventPair ev, int* mode, char* desc, size_t desc_cap);

// Output-stationary matrix-core kernel with Phi tiles shared by a work-group (16-bit types, blocks
// exactly 32, 64 or 128 rows high): whether it takes the call with a given row split, and its
// launch.  Without a row split it stores the result itself; with one, work-group z writes plane z
// of the workspace and the caller runs the plane reduction.
bool outs_supported(const SketchParams& p, const void* A, int64_t lda, int64_t n, fs_dtype dt, int zsplit);
hipError_t launch_outs(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out, int64_t ldo,
                       fs_dtype dt, const uint32_t* orbit, int zsplit, float* ws, int64_t ldw, hipStream_t st,
                       EventPair ev, char* desc, size_t desc_cap);

// Matrix-core kernel that keeps several output blocks, consecutive on the orbit of the wiring, in one
// wave's accumulators (blocks exactly 64 rows high, or 128 for fp32; the slot count divides kappa and
// M; needs the orbit table): whether it takes the call, and its launch.  It stores the result
// itself: no workspace.
bool stacked_supported(const SketchParams& p, const void* A, int64_t lda, int64_t n, fs_dtype dt, bool have_orbit);
hipError_t launch_stacked(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out, int64_t ldo,
                          fs_dtype dt, const uint32_t* orbit, hipStream_t st, EventPair ev, char* desc,
                          size_t desc_cap);

// Matrix-core path for inputs held examples-as-rows: G is n x d (ld = ldg), out is n x k.
bool rows_supported(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt);
bool rows_describe(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt, int* mode,
                   int* flags, size_t* workspace);
size_t rows_workspace_bytes(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt);
hipError_t launch_rows(const SketchParams& p, const void* G, int64_t ldg, int64_t n, void* out,
                       int64_t ldo, fs_dtype dt, void* ws, const uint32_t* orbit, hipStream_t st,
                       EventPair ev);

// Plain SJLT, global float atomics.  ws: k*n floats for bf16 output, unused for fp32.
size_t scatter_workspace_bytes(const SketchParams& p, int64_t n, fs_dtype dt);
hipError_t launch_scatter(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                          int64_t ldo, fs_dtype dt, void* ws, hipStream_t st, EventPair ev);

// FlashBlockRow gather sketch (kind BLOCKROW): no workspace.
hipError_t launch_blockrow(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                           int64_t ldo, fs_dtype dt, hipStream_t st, EventPair ev);
hipError_t launch_blockrow_export(const SketchParams& p, int32_t* cols, int8_t* signs, hipStream_t st);

// Dense Gaussian sketch.  `storage` holds the k x d matrix as fp32, then four bf16
// copies (rounded, and the exact split hi / mid / lo): gauss_bytes(k, d) bytes.
size_t gauss_bytes(int64_t k, int64_t d);
hipError_t gauss_fill(void* storage, int64_t k, int64_t d, uint32_t key1, hipStream_t st);
bool gauss_supported(int64_t k, int64_t d, const void* A, int64_t lda, int64_t n, fs_dtype dt);
hipError_t launch_gauss(const void* storage, int64_t k, int64_t d, const void* A, int64_t lda,
                        int64_t n, void* out, int64_t ldo, fs_dtype dt, hipStream_t st, EventPair ev);

}  // namespace fs
