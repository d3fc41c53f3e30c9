// General BlockPerm-SJLT apply: any Br, any s, any alignment.
//
// Work-group (g, j[, pass]) owns the output tile Y[g*Br : (g+1)*Br, j*TN : (j+1)*TN]
// (Alg. 1: one thread-block per output tile, no global atomics).  Unlike the
// paper's kernel there are no shared-memory atomics either: each lane owns one
// column, rows are walked wave-uniformly, so two lanes never touch the same
// accumulator.  The tile lives in LDS as [row][lane] (bank = lane, conflict
// free).  A is re-read once per wiring slot (kappa times in total).
//
// When Br*TN floats exceed the LDS budget the rows are split over grid.z
// passes; a pass skips the updates that fall outside its row range.
#include "convert.h"
#include "handle.h"
#include "spec.h"

namespace fs {

constexpr int kGenericLdsBytes = 64 * 1024;
constexpr int kRowUnroll = 8;

// ONEPASS: the whole block height fits the LDS tile (one row pass), so no update is filtered.
template <typename T, bool POW2, bool ONEPASS>
__global__ __launch_bounds__(256) void generic_kernel(SketchParams p, const T* __restrict__ A,
                                                      int64_t lda, int n, T* __restrict__ out,
                                                      int64_t ldo, int rows_per_pass) {
  extern __shared__ float sY[];  // [R][TN]
  const int tn = blockDim.x, tid = threadIdx.x;
  const uint32_t g = blockIdx.x;
  const uint32_t r0 = blockIdx.z * (uint32_t)rows_per_pass;
  const uint32_t R = min((uint32_t)rows_per_pass, p.Br - r0);
  const int col = blockIdx.y * tn + tid;
  const bool active = col < n;

  for (uint32_t r = 0; r < R; ++r) sY[r * tn + tid] = 0.f;

  uint32_t h = g;
  for (uint32_t l = 0; l < p.kappa; ++l) {
    h = wire_next(h, p.a, p.b, p.M);
    const uint32_t bk = block_key(p.key1, g, h, p.M);
    // Every load goes to a valid address (row and column clamped into the block) and what should
    // not count is zeroed afterwards: unconditional loads are issued back to back, conditional
    // ones were waited for one by one.  Rows at or beyond d (padding of a partly filled last
    // block) and lanes beyond column n read as 0.
    const uint32_t rows_here = (uint32_t)min((int64_t)p.Bc, p.d - (int64_t)h * p.Bc);  // >= 1
    const T* src = A + (int64_t)h * p.Bc * lda + min(col, n - 1);
    RowHash lane_rh{0u, 0u, 0u};
    static_assert(64 % kRowUnroll == 0, "a group of 64 hashed rows is a whole number of load batches");
    for (uint32_t u0 = 0; u0 < p.Bc; u0 += kRowUnroll) {
      // The hashes of 64 rows at a time, one lane per row, handed to the wave-uniform walk below
      // with v_readlane: the walk runs on the CU's one scalar unit, which would otherwise also
      // compute every row's hash once per wave.
      if (u0 % 64 == 0) lane_rh = POW2 ? row_hash_pow2(bk, u0 + (tid & 63), p.Br) : row_hash_any(bk, u0 + (tid & 63), p.Br);
      float v[kRowUnroll];
#pragma unroll
      for (int q = 0; q < kRowUnroll; ++q)
        v[q] = Elt<T>::load(src + (int64_t)min(u0 + q, rows_here - 1) * lda);
#pragma unroll
      for (int q = 0; q < kRowUnroll; ++q)
        if (!active || u0 + q >= rows_here) v[q] = 0.f;
#pragma unroll
      for (int q = 0; q < kRowUnroll; ++q) {
        if (u0 + q >= p.Bc) break;
        const int src_lane = (int)((u0 + q) & 63u);
        RowHash rh;
        rh.shift = (uint32_t)__builtin_amdgcn_readlane((int)lane_rh.shift, src_lane);
        rh.stride = (uint32_t)__builtin_amdgcn_readlane((int)lane_rh.stride, src_lane);
        rh.signs = (uint32_t)__builtin_amdgcn_readlane((int)lane_rh.signs, src_lane);
        uint32_t r = rh.shift;
        for (uint32_t i = 0; i < p.s; ++i) {
          const uint32_t rel = ONEPASS ? r : r - r0;
          if (ONEPASS || rel < R) {
            const float x = ((rh.signs >> i) & 1u) ? -v[q] : v[q];
            sY[rel * tn + tid] += x;
          }
          r += rh.stride;
          if (POW2) r &= p.Br - 1;
          else if (r >= p.Br) r -= p.Br;
        }
      }
    }
  }

  if (active) {
    T* dst = out + ((int64_t)g * p.Br + r0) * ldo + col;
    for (uint32_t r = 0; r < R; ++r) Elt<T>::store(dst + (int64_t)r * ldo, sY[r * tn + tid] * p.scale);
  }
}

// The same for vectors held as rows: out (n x k) = G S^T, G (n x d) row-major.  Thread e of a
// work-group owns example ex0 + e; a chunk of kChunk consecutive entries of TE examples is
// loaded with consecutive threads on consecutive addresses of one example, turned through LDS
// ([entry][example], odd stride), and then walked exactly as the column kernel walks rows:
// wave-uniform hash, lane-private accumulators, no atomics.  The output tile goes back through
// LDS so that consecutive threads store consecutive elements of one output row.
constexpr int kChunk = 32;

template <typename T, bool POW2, bool ONEPASS>
__global__ __launch_bounds__(128) void generic_rows_kernel(SketchParams p, const T* __restrict__ G,
                                                           int64_t ldg, int n, T* __restrict__ out,
                                                           int64_t ldo, int rows_per_pass) {
  extern __shared__ float smem_rows[];
  const int te = blockDim.x, tid = threadIdx.x, ld = te + 1;
  float* sG = smem_rows;                 // [kChunk][ld]
  float* sY = smem_rows + kChunk * ld;   // [R][ld]
  const uint32_t g = blockIdx.x;
  const uint32_t r0 = blockIdx.z * (uint32_t)rows_per_pass;
  const uint32_t R = min((uint32_t)rows_per_pass, p.Br - r0);
  const int64_t ex0 = (int64_t)blockIdx.y * te;

  for (uint32_t r = 0; r < R; ++r) sY[r * ld + tid] = 0.f;

  uint32_t h = g;
  for (uint32_t l = 0; l < p.kappa; ++l) {
    h = wire_next(h, p.a, p.b, p.M);
    const uint32_t bk = block_key(p.key1, g, h, p.M);
    for (uint32_t u0 = 0; u0 < p.Bc; u0 += kChunk) {
      __syncthreads();  // the previous chunk has been consumed
      // (loads at clamped, always valid addresses, zeroed afterwards where they do not count:
      // see the column kernel)
      // thread tid takes entry q = tid % 32 of the examples tid/32, tid/32 + te/32, ...: the
      // column is fixed per thread and the row pointer advances by a constant
      {
        const int q = tid % kChunk;
        const int64_t col = (int64_t)h * p.Bc + u0 + q;  // entry of the vector; padding reads as 0
        const bool col_ok = u0 + q < p.Bc && col < p.d;
        const T* colp = G + min(col, p.d - 1);
        const int64_t last = ((int64_t)n - 1) * ldg;  // offset of the last example's row
        const int e_step = te / kChunk;
        int e = tid / kChunk;
        int64_t row = (ex0 + e) * ldg;
#pragma unroll 8
        for (int it = 0; it < kChunk; ++it, e += e_step, row += (int64_t)e_step * ldg) {
          const bool row_ok = ex0 + e < n;
          const float x = Elt<T>::load(colp + (row_ok ? row : last));
          sG[q * ld + e] = (row_ok && col_ok) ? x : 0.f;
        }
      }
      __syncthreads();
      // the chunk's hashes, one lane per entry (the upper half-wave repeats the lower one)
      const RowHash lane_rh = POW2 ? row_hash_pow2(bk, u0 + (tid & (kChunk - 1)), p.Br)
                                   : row_hash_any(bk, u0 + (tid & (kChunk - 1)), p.Br);
      for (int q = 0; q < kChunk; ++q) {
        if (u0 + q >= p.Bc) break;
        const float v = sG[q * ld + tid];
        RowHash rh;
        rh.shift = (uint32_t)__builtin_amdgcn_readlane((int)lane_rh.shift, q);
        rh.stride = (uint32_t)__builtin_amdgcn_readlane((int)lane_rh.stride, q);
        rh.signs = (uint32_t)__builtin_amdgcn_readlane((int)lane_rh.signs, q);
        uint32_t r = rh.shift;
        for (uint32_t i = 0; i < p.s; ++i) {
          const uint32_t rel = ONEPASS ? r : r - r0;
          if (ONEPASS || rel < R) sY[rel * ld + tid] += ((rh.signs >> i) & 1u) ? -v : v;
          r += rh.stride;
          if (POW2) r &= p.Br - 1;
          else if (r >= p.Br) r -= p.Br;
        }
      }
    }
  }
  __syncthreads();
  for (uint32_t idx = tid; idx < (uint32_t)te * R; idx += te) {
    const uint32_t e = idx / R, r = idx % R;
    if (ex0 + e < n)
      Elt<T>::store(out + (ex0 + e) * ldo + (int64_t)g * p.Br + r0 + r, sY[r * ld + e] * p.scale);
  }
}

hipError_t launch_generic_rows(const SketchParams& p, const void* G, int64_t ldg, int64_t n, void* out,
                               int64_t ldo, fs_dtype dt, hipStream_t st, EventPair ev) {
  const int te = n <= 64 ? 64 : 128;
  const int ld = te + 1;
  const int max_rows = (kGenericLdsBytes - kChunk * ld * 4) / (ld * 4);
  const int rows_per_pass = (int)p.Br < max_rows ? (int)p.Br : max_rows;
  const unsigned passes = (p.Br + rows_per_pass - 1) / rows_per_pass;
  const int64_t ex_tiles = (n + te - 1) / te;
  if (ex_tiles > 65535 || passes > 65535u) return hipErrorInvalidValue;
  dim3 grid(p.M, (unsigned)ex_tiles, passes), block(te);
  const size_t lds = (size_t)(kChunk + rows_per_pass) * ld * 4;
#define FS_GO(T, P2)                                                                                         \
  do {                                                                                                       \
    if (passes == 1)                                                                                         \
      hipLaunchKernelGGL((generic_rows_kernel<T, P2, true>), grid, block, lds, st, p, (const T*)G, ldg,      \
                         (int)n, (T*)out, ldo, rows_per_pass);                                               \
    else                                                                                                     \
      hipLaunchKernelGGL((generic_rows_kernel<T, P2, false>), grid, block, lds, st, p, (const T*)G, ldg,     \
                         (int)n, (T*)out, ldo, rows_per_pass);                                               \
  } while (0)
  if (ev.start) (void)hipEventRecord(ev.start, st);
  if (dt == FS_F32)       { if (p.br_pow2) FS_GO(float, true); else FS_GO(float, false); }
  else if (dt == FS_BF16) { if (p.br_pow2) FS_GO(uint16_t, true); else FS_GO(uint16_t, false); }
  else                    { if (p.br_pow2) FS_GO(f16, true); else FS_GO(f16, false); }
#undef FS_GO
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  return hipGetLastError();
}

hipError_t launch_generic(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                          int64_t ldo, fs_dtype dt, hipStream_t st, EventPair ev) {
  int tn = 256;
  if (n <= 64) tn = 64; else if (n <= 128) tn = 128;
  while (tn > 64 && (int64_t)p.Br * tn * 4 > kGenericLdsBytes) tn >>= 1;
  int rows_per_pass = (int)p.Br;
  const int max_rows = kGenericLdsBytes / (tn * 4);
  if (rows_per_pass > max_rows) rows_per_pass = max_rows;
  const unsigned passes = (p.Br + rows_per_pass - 1) / rows_per_pass;
  const unsigned jt = (unsigned)((n + tn - 1) / tn);
  if (jt > 65535u || passes > 65535u) return hipErrorInvalidValue;
  dim3 grid(p.M, jt, passes), block(tn);
  const size_t lds = (size_t)rows_per_pass * tn * 4;
#define FS_GO(T, P2)                                                                                        \
  do {                                                                                                      \
    if (passes == 1)                                                                                        \
      hipLaunchKernelGGL((generic_kernel<T, P2, true>), grid, block, lds, st, p, (const T*)A, lda, (int)n,  \
                         (T*)out, ldo, rows_per_pass);                                                      \
    else                                                                                                    \
      hipLaunchKernelGGL((generic_kernel<T, P2, false>), grid, block, lds, st, p, (const T*)A, lda, (int)n, \
                         (T*)out, ldo, rows_per_pass);                                                      \
  } while (0)
  if (ev.start) (void)hipEventRecord(ev.start, st);
  if (dt == FS_F32)       { if (p.br_pow2) FS_GO(float, true); else FS_GO(float, false); }
  else if (dt == FS_BF16) { if (p.br_pow2) FS_GO(uint16_t, true); else FS_GO(uint16_t, false); }
  else                    { if (p.br_pow2) FS_GO(f16, true); else FS_GO(f16, false); }
#undef FS_GO
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  return hipGetLastError();
}

}  // namespace fs
