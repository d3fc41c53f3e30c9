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

// Orbit table of the wiring map: tab[q] = f^q(0) for q in [0, M), tab[M + f^q(0)] = q.
// f^q is itself affine, x -> (A_q x + B_q) mod M, and powers compose as
// (A, B) o (A', B') = (A A', A B' + B), so thread q reaches f^q(0) = B_q by binary
// exponentiation (M <= 2^24: every product fits 64 bits).  f has full period (Appendix E,
// "Full-cycle affine construction"), so the M values are distinct and both halves are
// written exactly once.
__global__ __launch_bounds__(256) void orbit_kernel(uint32_t* __restrict__ tab, uint32_t M, uint32_t a,
                                                    uint32_t b) {
  const uint32_t q = blockIdx.x * 256 + threadIdx.x;
  if (q >= M) return;
  uint64_t ra = 1, rb = 0;   // f^0
  uint64_t pa = a, pb = b;   // f^(2^i)
  for (uint32_t e = q; e; e >>= 1) {
    if (e & 1u) { rb = (pa * rb + pb) % M; ra = (pa * ra) % M; }
    pb = (pa * pb + pb) % M;
    pa = (pa * pa) % M;
  }
  tab[q] = (uint32_t)rb;
  tab[M + (uint32_t)rb] = q;
}

hipError_t launch_orbit(const SketchParams& p, uint32_t* tab, hipStream_t st) {
  hipLaunchKernelGGL(orbit_kernel, dim3((p.M + 255) / 256), dim3(256), 0, st, tab, p.M, p.a, p.b);
  return hipGetLastError();
}

hipError_t launch_export(const SketchParams& p, int32_t* rows, int8_t* signs, hipStream_t st) {
  const int64_t total = p.d * p.kappa;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(export_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, rows, signs);
  return hipGetLastError();
}

}  // namespace fs
