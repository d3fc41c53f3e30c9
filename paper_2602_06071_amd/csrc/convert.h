// 16-bit element types and their fp32 conversions.  bf16 is carried as raw uint16_t bits,
// IEEE half as the compiler's _Float16 (conversions round to nearest even, subnormals kept).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fs {

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float((uint32_t)b << 16);
}

// round-to-nearest-even; NaN stays NaN (quiet)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

typedef _Float16 f16;

__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
  return __builtin_bit_cast(uint16_t, (f16)f);
}

template <typename T> struct Elt;
template <> struct Elt<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elt<uint16_t> {
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = f32_to_bf16_rne(v); }
};

template <> struct Elt<f16> {
  static __device__ __forceinline__ float load(const f16* p) { return (float)*p; }
  static __device__ __forceinline__ void store(f16* p, float v) { *p = (f16)v; }
};

// four fp32 values -> four 16-bit elements of type T (bf16 or half), as two dwords
template <typename T> __device__ __forceinline__ uint2 pack4(const float (&v)[4]);
template <> __device__ __forceinline__ uint2 pack4<uint16_t>(const float (&v)[4]) {
  uint2 w;
  w.x = (uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16);
  w.y = (uint32_t)f32_to_bf16_rne(v[2]) | ((uint32_t)f32_to_bf16_rne(v[3]) << 16);
  return w;
}
template <> __device__ __forceinline__ uint2 pack4<f16>(const float (&v)[4]) {
  uint2 w;
  w.x = (uint32_t)f32_to_f16_bits(v[0]) | ((uint32_t)f32_to_f16_bits(v[1]) << 16);
  w.y = (uint32_t)f32_to_f16_bits(v[2]) | ((uint32_t)f32_to_f16_bits(v[3]) << 16);
  return w;
}

// the reverse: two dwords holding four 16-bit elements -> fp32
template <typename T> __device__ __forceinline__ void unpack4(uint2 w, float (&v)[4]);
template <> __device__ __forceinline__ void unpack4<uint16_t>(uint2 w, float (&v)[4]) {
  v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xFFFF0000u);
  v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xFFFF0000u);
}
template <> __device__ __forceinline__ void unpack4<f16>(uint2 w, float (&v)[4]) {
  v[0] = (float)__builtin_bit_cast(f16, (uint16_t)w.x); v[1] = (float)__builtin_bit_cast(f16, (uint16_t)(w.x >> 16));
  v[2] = (float)__builtin_bit_cast(f16, (uint16_t)w.y); v[3] = (float)__builtin_bit_cast(f16, (uint16_t)(w.y >> 16));
}

}  // namespace fs
