// Pieces shared by the matrix-core kernels: tile constants, the HBM -> register ->
// MFMA-operand transposition of a row-major input, the exact 3-way bf16 split of
// fp32 values, and the MFMA wrapper.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "convert.h"

namespace fs {
namespace mm {

constexpr int KC = 64;           // rows of A per stage
constexpr int KSTEPS = KC / 16;  // MFMA k-steps per stage
constexpr int PHI_LD = KC + 8;   // bf16 per LDS row of Phi (144 B: conflict-free b128 reads)
constexpr int WCOLS = 128;       // columns per wave (4 per lane x 32 lanes)
constexpr int MAX_KAPPA = 128;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// What one lane loads from one row: CPL consecutive columns as one vector V; PFD = depth
// (in k-steps) of the register prefetch ring, sized to 64 VGPRs per wave.
template <typename T, int CPL> struct LdN;
template <> struct LdN<uint16_t, 4> { using V = uint2; static constexpr int PFD = 4; };
template <> struct LdN<f16, 4>      { using V = uint2; static constexpr int PFD = 4; };
template <> struct LdN<float, 4>    { using V = uint4; static constexpr int PFD = 2; };
template <typename T> using Ld = LdN<T, 4>;

__device__ __forceinline__ uint32_t perm(uint32_t hi_src, uint32_t lo_src, uint32_t sel) {
  return __builtin_amdgcn_perm(hi_src, lo_src, sel);
}

// 4 consecutive columns of one row, element by element; columns >= n read as 0.
template <typename T, int CPL = 4>
__device__ __forceinline__ typename LdN<T, CPL>::V load4_guarded(const T* p4, int col0, int n) {
  using V = typename LdN<T, CPL>::V;
  T e[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) e[c] = (col0 + c < n) ? p4[c] : (T)0;
  return *reinterpret_cast<V*>(e);
}

// MFMA B operands of the four column residues from 8 rows x 4 columns (bf16).
__device__ __forceinline__ void make_ops(const uint2 (&r)[8], uint4 (&op)[4]) {
  uint32_t* o0 = reinterpret_cast<uint32_t*>(&op[0]);
  uint32_t* o1 = reinterpret_cast<uint32_t*>(&op[1]);
  uint32_t* o2 = reinterpret_cast<uint32_t*>(&op[2]);
  uint32_t* o3 = reinterpret_cast<uint32_t*>(&op[3]);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    o0[q] = perm(r[2 * q + 1].x, r[2 * q].x, 0x05040100u);
    o1[q] = perm(r[2 * q + 1].x, r[2 * q].x, 0x07060302u);
    o2[q] = perm(r[2 * q + 1].y, r[2 * q].y, 0x05040100u);
    o3[q] = perm(r[2 * q + 1].y, r[2 * q].y, 0x07060302u);
  }
}

// fp32 column c of 8 rows -> three exact bf16 pieces (x = hi + mid + lo).
__device__ __forceinline__ void split_ops(const uint32_t (&x)[8], uint4& hi, uint4& mid, uint4& lo) {
  uint32_t m[8], l[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float xf = __uint_as_float(x[j]);
    const float r1 = xf - __uint_as_float(x[j] & 0xFFFF0000u);   // exact, <= 16 significant bits
    const uint32_t r1b = __float_as_uint(r1);
    const float r2 = r1 - __uint_as_float(r1b & 0xFFFF0000u);    // exact, <= 8 significant bits
    m[j] = r1b;
    l[j] = __float_as_uint(r2);
  }
  uint32_t* h = reinterpret_cast<uint32_t*>(&hi);
  uint32_t* mm = reinterpret_cast<uint32_t*>(&mid);
  uint32_t* ll = reinterpret_cast<uint32_t*>(&lo);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    h[q] = perm(x[2 * q + 1], x[2 * q], 0x07060302u);
    mm[q] = perm(m[2 * q + 1], m[2 * q], 0x07060302u);
    ll[q] = perm(l[2 * q + 1], l[2 * q], 0x07060302u);
  }
}

// The 16-bit format of the MFMA operands for element type T: half for half inputs, bf16 for
// bf16 inputs and for the bf16 pieces that fp32 inputs are split into.  `one` is +1 in that
// format (the sign is bit 15 in both); op() is D = A*B + C on 32 x 32 x 16 tiles, fp32 accumulate.
template <typename T> struct Fmt {
  static constexpr uint16_t one = 0x3F80;
  static __device__ __forceinline__ f32x16 op(uint4 a, uint4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Fmt<f16> {
  static constexpr uint16_t one = 0x3C00;
  static __device__ __forceinline__ f32x16 op(uint4 a, uint4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};

template <typename T>
__device__ __forceinline__ f32x16 mfma(uint4 a, uint4 b, f32x16 c) {
  return Fmt<T>::op(a, b, c);
}

}  // namespace mm
}  // namespace fs
