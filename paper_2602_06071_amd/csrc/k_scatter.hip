// Prior-art baseline: plain SJLT applied as a global scatter-add (paper
// Section 3, "GPU bottlenecks for Sparse Sketching", and Section 5,
// "Comparison to prior GPU SJLT kernels"): every input element issues s signed
// float atomics into the output, Theta(s*d*n) global atomics in total.
// The sketch is the library's S with a single block (M = 1, Bc = d, Br = k).
#include "convert.h"
#include "handle.h"
#include "spec.h"

namespace fs {

constexpr int kScatterRows = 128;  // input rows per work-group

__global__ __launch_bounds__(256) void fill_zero_2d(float* __restrict__ dst, int64_t ld, int64_t rows,
                                                    int n) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= n) return;
  for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) dst[r * ld + col] = 0.f;
}

template <typename T, bool POW2>
__global__ __launch_bounds__(256) void scatter_kernel(SketchParams p, const T* __restrict__ A,
                                                      int64_t lda, int n, float* __restrict__ acc,
                                                      int64_t ldacc) {
  const int col = blockIdx.y * 256 + threadIdx.x;
  if (col >= n) return;
  const uint32_t bk = block_key(p.key1, 0u, 0u, 1u);
  const uint32_t u_beg = blockIdx.x * (uint32_t)kScatterRows;
  const uint32_t u_end = min(u_beg + (uint32_t)kScatterRows, (uint32_t)min((int64_t)p.Bc, p.d));
  for (uint32_t u = u_beg; u < u_end; ++u) {
    const float v = Elt<T>::load(A + (int64_t)u * lda + col) * p.scale;
    const RowHash rh = POW2 ? row_hash_pow2(bk, u, p.Br) : row_hash_any(bk, u, p.Br);
    uint32_t r = rh.shift;
    for (uint32_t i = 0; i < p.s; ++i) {
      unsafeAtomicAdd(acc + (int64_t)r * ldacc + col, ((rh.signs >> i) & 1u) ? -v : v);
      r += rh.stride;
      if (r >= p.Br) r -= p.Br;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void scatter_finalize(const float* __restrict__ acc, int64_t rows, int n,
                                                        T* __restrict__ out, int64_t ldo) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= n) return;
  for (int64_t r = blockIdx.y; r < rows; r += gridDim.y)
    Elt<T>::store(out + r * ldo + col, acc[r * (int64_t)n + col]);
}

size_t scatter_workspace_bytes(const SketchParams& p, int64_t n, fs_dtype dt) {
  return dt != FS_F32 ? (size_t)p.k * (size_t)n * sizeof(float) : 0;
}

hipError_t launch_scatter(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                          int64_t ldo, fs_dtype dt, void* ws, hipStream_t st, EventPair ev) {
  const unsigned jt = (unsigned)((n + 255) / 256);
  const unsigned slabs = (p.Bc + kScatterRows - 1) / kScatterRows;
  if (jt > 65535u) return hipErrorInvalidValue;
  float* acc = dt == FS_F32 ? (float*)out : (float*)ws;
  const int64_t ldacc = dt == FS_F32 ? ldo : n;
  const unsigned zrows = (unsigned)(p.k < 4096 ? p.k : 4096);
  hipLaunchKernelGGL(fill_zero_2d, dim3(jt, zrows), dim3(256), 0, st, acc, ldacc, p.k, (int)n);
  dim3 grid(slabs, jt), block(256);
#define FS_GO(T, P2) \
  hipLaunchKernelGGL((scatter_kernel<T, P2>), grid, block, 0, st, p, (const T*)A, lda, (int)n, acc, ldacc)
  if (ev.start) (void)hipEventRecord(ev.start, st);
  if (dt == FS_F32)       { if (p.br_pow2) FS_GO(float, true); else FS_GO(float, false); }
  else if (dt == FS_BF16) { if (p.br_pow2) FS_GO(uint16_t, true); else FS_GO(uint16_t, false); }
  else                    { if (p.br_pow2) FS_GO(f16, true); else FS_GO(f16, false); }
#undef FS_GO
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  if (dt == FS_BF16)
    hipLaunchKernelGGL(scatter_finalize<uint16_t>, dim3(jt, zrows), dim3(256), 0, st, acc, p.k, (int)n,
                       (uint16_t*)out, ldo);
  else if (dt == FS_F16)
    hipLaunchKernelGGL(scatter_finalize<f16>, dim3(jt, zrows), dim3(256), 0, st, acc, p.k, (int)n, (f16*)out, ldo);
  return hipGetLastError();
}

}  // namespace fs
