// Materialises the nonzeros of S (rows and signs) from the handle's integers.
// One thread per (column of S, wiring slot); the output block g of slot l is
// found by walking the inverse affine map l times from the column's input
// block (Appendix E: pi_l(g) = f^l(g), so g = f^{-l}(h)).
#include "handle.h"
#include "spec.h"

namespace fs {

__global__ __launch_bounds__(256) void export_kernel(SketchParams p, int32_t* __restrict__ rows,
                                                     int8_t* __restrict__ signs) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // c * kappa + (l - 1)
  if (idx >= p.d * p.kappa) return;
  const int64_t c = idx / p.kappa;
  const uint32_t l = (uint32_t)(idx % p.kappa) + 1u;
  const uint32_t h = (uint32_t)(c / p.Bc), u = (uint32_t)(c % p.Bc);
  uint32_t g = h;
  for (uint32_t t = 0; t < l; ++t) g = wire_prev(g, p.a_inv, p.b, p.M);
  const uint32_t bk = block_key(p.key1, g, h, p.M);
  const RowHash rh = p.br_pow2 ? row_hash_pow2(bk, u, p.Br) : row_hash_any(bk, u, p.Br);
  uint32_t r = rh.shift;
  const int64_t o = idx * p.s;
  for (uint32_t i = 0; i < p.s; ++i) {
    rows[o + i] = (int32_t)(g * p.Br + r);
    signs[o + i] = ((rh.signs >> i) & 1u) ? (int8_t)-1 : (int8_t)1;
    r += rh.stride;
    if (r >= p.Br) r -= p.Br;
  }
}

hipError_t launch_export(const SketchParams& p, int32_t* rows, int8_t* signs, hipStream_t st) {
  const int64_t total = p.d * p.kappa;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(export_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, rows, signs);
  return hipGetLastError();
}

}  // namespace fs
