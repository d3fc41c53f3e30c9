// Integer recipe that turns (seed, g, h, u) into the nonzeros of S.
// Paper Appendix E ("Within-block hashing") asks for a fast 32-bit mixing hash
// giving, per input row of a block, s distinct destination rows in [Br] (an
// affine progression with hash-derived shift and stride) and s independent
// signs; the concrete words below are this library's reading of it.
// All arithmetic is on uint32 with wrap-around.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FS_HD __host__ __device__ __forceinline__
#else
#define FS_HD inline
#endif

namespace fs {

constexpr uint32_t kC1 = 0x6A09E667u;  // frac(sqrt 2)
constexpr uint32_t kC2 = 0xBB67AE85u;  // frac(sqrt 3)
constexpr uint32_t kC3 = 0x3C6EF373u;  // frac(sqrt 5) | 1

FS_HD uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= kC1;
  x ^= x >> 15; x *= kC2;
  x ^= x >> 16; x *= kC3;
  x ^= x >> 15;
  return x;
}

// Key of the nonzero block (g, h) of an M x M block grid.
FS_HD uint32_t block_key(uint32_t key1, uint32_t g, uint32_t h, uint32_t M) {
  return mix32(key1 ^ mix32(g * M + h + kC3));
}

FS_HD uint32_t gcd_u32(uint32_t a, uint32_t b) {
  while (b) { uint32_t t = a % b; a = b; b = t; }
  return a;
}

// Row recipe for local input row u of a block with key bk:
//   r_i = (shift + i*stride) mod Br, sign_i = bit i of signs (1 = negative).
struct RowHash {
  uint32_t shift, stride, signs;
};

// Br a power of two (Br >= 1): stride is forced odd, which is exactly "advance
// to the next unit modulo Br".
FS_HD RowHash row_hash_pow2(uint32_t bk, uint32_t u, uint32_t Br) {
  const uint32_t h1 = mix32(bk ^ u);
  RowHash r;
  r.signs = mix32(h1 ^ kC2);
  r.shift = (h1 & 0xFFFFu) & (Br - 1);
  r.stride = Br > 1 ? (((h1 >> 16) & (Br - 1)) | 1u) : 0u;
  return r;
}

// Any Br in [1, 65536].
FS_HD RowHash row_hash_any(uint32_t bk, uint32_t u, uint32_t Br) {
  const uint32_t h1 = mix32(bk ^ u);
  RowHash r;
  r.signs = mix32(h1 ^ kC2);
  r.shift = (h1 & 0xFFFFu) % Br;
  uint32_t c = (h1 >> 16) % Br;
  while (gcd_u32(c, Br) != 1u) c = (c + 1u) % Br;
  r.stride = c;
  return r;
}

// f(x) = (a x + b) mod M, M <= 2^24 so the product fits 64 bits comfortably.
FS_HD uint32_t wire_next(uint32_t x, uint32_t a, uint32_t b, uint32_t M) {
  return (uint32_t)(((uint64_t)a * x + b) % M);
}
// f^{-1}(y) = a_inv (y - b) mod M
FS_HD uint32_t wire_prev(uint32_t y, uint32_t a_inv, uint32_t b, uint32_t M) {
  return (uint32_t)(((uint64_t)a_inv * ((y + M - b) % M)) % M);
}

}  // namespace fs
