// FlashBlockRow (paper Appendix D, Alg. 2): the gather-only block-row sampling sketch.
// Output row (g, r) adds s signed rows of A from each of the kappa input blocks its block
// row samples and scales by sqrt(d/k)/sqrt(kappa*s).  No accumulation conflicts at all:
// one wave owns one output row of a column tile, every index and sign is wave-uniform
// (scalar ALU), every load is a contiguous row segment.  It reads k*kappa*s rows of A,
// not all d: the paper's "fast but fragile" point (some input coordinates are never read).
//
// Where the paper is silent: the kappa blocks of block row g are the wiring neighbours
// f^l(g); update t of row r in block (g, h) uses w1 = mix32(BK(g,h) ^ C1 ^ (r*32 + t)),
// index w1 mod Bc, sign = low bit of mix32(w1 ^ C2).  Rows beyond d read as zero.
#include "convert.h"
#include "handle.h"
#include "spec.h"

namespace fs {

namespace {

struct RowPick { uint32_t idx; bool neg; };

__device__ __forceinline__ RowPick pick(uint32_t bk, uint32_t r, uint32_t t, uint32_t Bc) {
  const uint32_t w1 = mix32(bk ^ kC1 ^ (r * 32u + t));
  return {w1 % Bc, (mix32(w1 ^ kC2) & 1u) != 0u};
}

// VEC: 4 columns per lane through one vector load (aligned A, lda % 4 == 0); else 1 column.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void blockrow_kernel(SketchParams p, const T* __restrict__ A,
                                                       int64_t lda, int n, T* __restrict__ out,
                                                       int64_t ldo, int out_vec) {
  constexpr int CPL = VEC ? 4 : 1;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row = (int64_t)blockIdx.x * 4 + wave;
  if (row >= p.k) return;
  const int lane = threadIdx.x & 63;
  const int col0 = ((int)blockIdx.y * 64 + lane) * CPL;
  const uint32_t g = (uint32_t)(row / p.Br), r = (uint32_t)(row % p.Br);
  const bool full = col0 + CPL <= n;

  float acc[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) acc[c] = 0.f;

  uint32_t h = g;
  for (uint32_t l = 0; l < p.kappa; ++l) {
    h = wire_next(h, p.a, p.b, p.M);
    const uint32_t bk = block_key(p.key1, g, h, p.M);
    for (uint32_t t = 0; t < p.s; ++t) {
      const RowPick pk = pick(bk, r, t, p.Bc);
      const int64_t src = (int64_t)h * p.Bc + pk.idx;
      if (src >= p.d) continue;  // zero padding of a partly filled last block
      const T* sp = A + src * lda + col0;
      float v[CPL];
      if constexpr (VEC) {
        if (full) {
          if constexpr (sizeof(T) == 2) {
            unpack4<T>(*reinterpret_cast<const uint2*>(sp), v);
          } else {
            const float4 w = *reinterpret_cast<const float4*>(sp);
            v[0] = w.x; v[1] = w.y; v[2] = w.z; v[3] = w.w;
          }
        } else {
#pragma unroll
          for (int c = 0; c < CPL; ++c) v[c] = col0 + c < n ? Elt<T>::load(sp + c) : 0.f;
        }
      } else {
        v[0] = col0 < n ? Elt<T>::load(sp) : 0.f;
      }
#pragma unroll
      for (int c = 0; c < CPL; ++c) acc[c] += pk.neg ? -v[c] : v[c];
    }
  }

  T* dst = out + row * ldo + col0;
  if (VEC && full && out_vec) {
    if constexpr (sizeof(T) == 2) {
      const float sc[4] = {acc[0] * p.scale, acc[CPL > 1 ? 1 : 0] * p.scale, acc[CPL > 2 ? 2 : 0] * p.scale,
                           acc[CPL > 3 ? 3 : 0] * p.scale};
      *reinterpret_cast<uint2*>(dst) = pack4<T>(sc);
    } else {
      *reinterpret_cast<float4*>(dst) = make_float4(acc[0] * p.scale, acc[CPL > 1 ? 1 : 0] * p.scale,
                                                    acc[CPL > 2 ? 2 : 0] * p.scale, acc[CPL > 3 ? 3 : 0] * p.scale);
    }
  } else {
#pragma unroll
    for (int c = 0; c < CPL; ++c)
      if (col0 + c < n) Elt<T>::store(dst + c, acc[c] * p.scale);
  }
}

// cols[row*kappa*s + l*s + t] = global column index (may lie in the padding), signs = +-1
__global__ __launch_bounds__(256) void blockrow_export_kernel(SketchParams p, int32_t* __restrict__ cols,
                                                              int8_t* __restrict__ signs) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // row * kappa + l
  if (idx >= p.k * p.kappa) return;
  const int64_t row = idx / p.kappa;
  const uint32_t l = (uint32_t)(idx % p.kappa);
  const uint32_t g = (uint32_t)(row / p.Br), r = (uint32_t)(row % p.Br);
  uint32_t h = g;
  for (uint32_t i = 0; i <= l; ++i) h = wire_next(h, p.a, p.b, p.M);
  const uint32_t bk = block_key(p.key1, g, h, p.M);
  for (uint32_t t = 0; t < p.s; ++t) {
    const RowPick pk = pick(bk, r, t, p.Bc);
    cols[idx * p.s + t] = (int32_t)((int64_t)h * p.Bc + pk.idx);
    signs[idx * p.s + t] = pk.neg ? (int8_t)-1 : (int8_t)1;
  }
}

}  // namespace

hipError_t launch_blockrow(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                           int64_t ldo, fs_dtype dt, hipStream_t st, EventPair ev) {
  const size_t esz = dt == FS_F32 ? 4 : 2;
  const bool vec = (uintptr_t)A % (4 * esz) == 0 && lda % 4 == 0;
  const int out_vec = ((uintptr_t)out % (4 * esz) == 0 && ldo % 4 == 0) ? 1 : 0;
  const int64_t cols_per_wg = vec ? 256 : 64;
  const int64_t col_tiles = (n + cols_per_wg - 1) / cols_per_wg;
  const int64_t row_groups = (p.k + 3) / 4;
  if (col_tiles > 65535 || row_groups > 0x7fffffff) return hipErrorInvalidValue;
  dim3 grid((unsigned)row_groups, (unsigned)col_tiles), block(256);
  if (ev.start) (void)hipEventRecord(ev.start, st);
#define FS_GO(T, V) hipLaunchKernelGGL((blockrow_kernel<T, V>), grid, block, 0, st, p, (const T*)A, lda, (int)n, (T*)out, ldo, out_vec)
  if (dt == FS_F32)       { if (vec) FS_GO(float, true); else FS_GO(float, false); }
  else if (dt == FS_BF16) { if (vec) FS_GO(uint16_t, true); else FS_GO(uint16_t, false); }
  else                    { if (vec) FS_GO(f16, true); else FS_GO(f16, false); }
#undef FS_GO
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  return hipGetLastError();
}

hipError_t launch_blockrow_export(const SketchParams& p, int32_t* cols, int8_t* signs, hipStream_t st) {
  const int64_t total = p.k * p.kappa;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(blockrow_export_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, cols, signs);
  return hipGetLastError();
}

}  // namespace fs
