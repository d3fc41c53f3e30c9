// Dense Gaussian sketch S_ij ~ N(0, 1/k) (paper Section 1 and Section 3: the
// canonical JL / OSE sketch) applied as a GEMM on the matrix cores: the
// dense-contraction reference point next to the sparse BlockPerm apply.
//
// S is materialised once at create time from a counter-based generator:
//   c  = mix32(lo32(i*d+j) ^ mix32(hi32(i*d+j) ^ key1 ^ C1))
//   u1 = ((mix32(c ^ 0x9E3779B9) >> 8) + 1) / 2^24,  u2 = (mix32(c ^ 0x85EBCA6B) >> 8) / 2^24
//   S_ij = (float)( sqrt(-2 ln u1) cos(2 pi u2) / sqrt(k) )          (Box-Muller, in fp64)
// and kept as fp32 (export), as bf16 and as half, each rounded to nearest (bf16 and half
// applies), and as an exact three-way bf16 split hi+mid+lo (fp32 applies).
//
// The GEMM reuses the data path of the sparse kernel: A goes HBM -> registers ->
// MFMA operand (4 columns x 8 rows per lane, transposed with v_perm_b32), S tiles of
// RW rows x 64 columns are staged in LDS (double buffered, one barrier per stage).
// fp32 applies use six bf16 MFMAs per tile (hi*hi, hi*mid, mid*hi, hi*lo, lo*hi,
// mid*mid); the dropped cross terms are below 2^-23 relative.
#include <type_traits>

#include "handle.h"
#include "mfma_common.h"
#include "spec.h"

namespace fs {

namespace {

using namespace mm;

__global__ __launch_bounds__(256) void gauss_fill_kernel(float* __restrict__ S32, uint16_t* __restrict__ Sbf,
                                                         uint16_t* __restrict__ Shi, uint16_t* __restrict__ Smid,
                                                         uint16_t* __restrict__ Slo, uint16_t* __restrict__ Sh,
                                                         int64_t k, int64_t d, uint32_t key1) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= k * d) return;
  const uint32_t c = mix32((uint32_t)idx ^ mix32((uint32_t)((uint64_t)idx >> 32) ^ key1 ^ kC1));
  const double u1 = (double)((mix32(c ^ 0x9E3779B9u) >> 8) + 1u) * (1.0 / 16777216.0);
  const double u2 = (double)(mix32(c ^ 0x85EBCA6Bu) >> 8) * (1.0 / 16777216.0);
  const double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
  const float s = (float)(z / sqrt((double)k));
  S32[idx] = s;
  Sbf[idx] = f32_to_bf16_rne(s);
  Sh[idx] = f32_to_f16_bits(s);
  const uint32_t sb = __float_as_uint(s);
  const float r1 = s - __uint_as_float(sb & 0xFFFF0000u);
  const uint32_t r1b = __float_as_uint(r1);
  const float r2 = r1 - __uint_as_float(r1b & 0xFFFF0000u);
  Shi[idx] = (uint16_t)(sb >> 16);
  Smid[idx] = (uint16_t)(r1b >> 16);
  Slo[idx] = (uint16_t)(__float_as_uint(r2) >> 16);
}

struct GaussArgs {
  const uint16_t* S[3];  // bf16 and half: S[0] only; fp32: hi, mid, lo
  const void* A;
  void* out;
  int64_t k, d, lda, ldo;
  int n, stages, out_vec;
};

// Work-group: RW = 32*MT*NRG rows of S x 128*NCG columns of A; wave: 32*MT rows x 128 columns.
// MT = 4 keeps the 256 accumulators in AGPRs with one wave per SIMD: four times the MFMA work per
// loaded (and, for fp32, per split) element of A than MT = 1.
template <typename T, int MT, int NRG, int NCG>
__global__ __launch_bounds__(64 * NRG * NCG) __attribute__((amdgpu_waves_per_eu(MT > 2 ? 1 : 2)))
void gauss_kernel(GaussArgs a) {
  using V = typename Ld<T>::V;
  constexpr int PFD = Ld<T>::PFD;
  constexpr int PARTS = sizeof(T) == 4 ? 3 : 1;
  constexpr int NW = NRG * NCG, NT = 64 * NW;
  constexpr int RW = 32 * MT * NRG;
  constexpr int TILE = RW * PHI_LD;
  constexpr int SREG = RW * 8 / NT;  // 16-byte pieces of one S tile per thread
  static_assert(RW * 8 % NT == 0, "tile copy must divide evenly");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* s_tile = reinterpret_cast<uint16_t*>(smem);  // [2][PARTS][TILE]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = wave / NCG, cg = wave % NCG, kg = lane >> 5;
  const int col0 = (int)blockIdx.y * (WCOLS * NCG) + cg * WCOLS + 4 * (lane & 31);
  const int64_t row_base = (int64_t)blockIdx.x * RW;
  const int T_stages = a.stages;
  const char* Abase = reinterpret_cast<const char*>(a.A);
  const int64_t row_bytes = a.lda * (int64_t)sizeof(T);
  const uint32_t voff = (uint32_t)(((int64_t)(kg * 8) * a.lda + col0) * (int64_t)sizeof(T));

  f32x16 acc[MT][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][c][i] = 0.f;

  uint4 sreg[PARTS][SREG];
  auto s_fetch = [&](int t) {
#pragma unroll
    for (int pt = 0; pt < PARTS; ++pt)
#pragma unroll
      for (int i = 0; i < SREG; ++i) {
        const int e = tid + i * NT, row = e >> 3, c16 = e & 7;
        sreg[pt][i] = *reinterpret_cast<const uint4*>(a.S[pt] + (row_base + row) * a.d + (int64_t)t * KC + c16 * 8);
      }
  };
  auto s_store = [&](int buf) {
#pragma unroll
    for (int pt = 0; pt < PARTS; ++pt)
#pragma unroll
      for (int i = 0; i < SREG; ++i) {
        const int e = tid + i * NT, row = e >> 3, c16 = e & 7;
        *reinterpret_cast<uint4*>(s_tile + (buf * PARTS + pt) * TILE + row * PHI_LD + c16 * 8) = sreg[pt][i];
      }
  };

  auto body = [&](auto ragged_tag) {
    constexpr bool RAGGED = decltype(ragged_tag)::value;
    V ld[PFD][8];
    auto issue = [&](int kk, V (&dst)[8]) {
      const char* sb = Abase + (int64_t)kk * 16 * row_bytes;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if constexpr (RAGGED) {
          dst[j] = load4_guarded<T>(reinterpret_cast<const T*>(sb + j * row_bytes + voff), col0, a.n);
        } else {
          // the whole of A is one buffer; offsets fit 32 bits (checked on the host)
          const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
              const_cast<char*>(Abase), 0, (int)((a.d - 1) * row_bytes + (int64_t)a.n * (int64_t)sizeof(T)),
              0x00020000);
          const uint32_t soj = (uint32_t)(kk * 16 + j) * (uint32_t)row_bytes;
          if constexpr (sizeof(T) == 2)
            dst[j] = __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soj, 0));
          else
            dst[j] = __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soj, 0));
        }
      }
    };

    auto stage = [&](int t, auto last_tag) {
      constexpr bool LAST = decltype(last_tag)::value;
      __syncthreads();
      if constexpr (!LAST) s_fetch(t + 1);
      const uint16_t* tile = s_tile + (t & 1) * PARTS * TILE;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        uint4 pa[PARTS][MT];
#pragma unroll
        for (int pt = 0; pt < PARTS; ++pt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            pa[pt][mt] = *reinterpret_cast<const uint4*>(
                tile + pt * TILE + ((rg * MT + mt) * 32 + (lane & 31)) * PHI_LD + ks * 16 + kg * 8);
        V(&cur)[8] = ld[ks % PFD];
        const bool fetch = !LAST || ks + PFD < KSTEPS;
        if constexpr (sizeof(T) == 2) {
          uint4 op[4];
          make_ops(cur, op);
          if (fetch) issue(t * KSTEPS + ks + PFD, cur);
#pragma unroll
          for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[0][mt], op[c], acc[mt][c]);
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            uint32_t xs[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
              xs[j] = c == 0 ? cur[j].x : c == 1 ? cur[j].y : c == 2 ? cur[j].z : cur[j].w;
            uint4 hi, mid, lo;
            split_ops(xs, hi, mid, lo);
            // product by product over the row tiles: with MT = 4 an accumulator is reused only
            // after three other MFMAs (back-to-back dependent MFMAs stall the matrix pipe)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[0][mt], hi, acc[mt][c]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[0][mt], mid, acc[mt][c]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[1][mt], hi, acc[mt][c]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[0][mt], lo, acc[mt][c]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[2][mt], hi, acc[mt][c]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[1][mt], mid, acc[mt][c]);
          }
          if (fetch) issue(t * KSTEPS + ks + PFD, cur);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (!LAST) s_store((t + 1) & 1);
    };

    s_fetch(0);
    s_store(0);
#pragma unroll
    for (int i = 0; i < PFD; ++i) issue(i, ld[i]);
    for (int t = 0; t + 1 < T_stages; ++t) stage(t, std::false_type{});
    stage(T_stages - 1, std::true_type{});
  };
  const bool full_tile = ((int)blockIdx.y + 1) * (WCOLS * NCG) <= a.n;
  if (full_tile) body(std::false_type{}); else body(std::true_type{});

  if (col0 >= a.n) return;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int64_t row = row_base + (rg * MT + mt) * 32 + 8 * (i >> 2) + 4 * kg + (i & 3);
      const float v[4] = {acc[mt][0][i], acc[mt][1][i], acc[mt][2][i], acc[mt][3][i]};
      T* dst = reinterpret_cast<T*>(a.out) + row * a.ldo + col0;
      if (a.out_vec && col0 + 3 < a.n) {
        if constexpr (sizeof(T) == 2) {
          const uint2 w = pack4<T>(v);
          *reinterpret_cast<uint2*>(dst) = w;
        } else {
          *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        }
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (col0 + c < a.n) Elt<T>::store(dst + c, v[c]);
      }
    }
  }
}

template <typename K>
hipError_t go(K kernel, dim3 grid, unsigned threads, size_t lds, hipStream_t st, const GaussArgs& a) {
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kernel, grid, dim3(threads), lds, st, a);
  return hipGetLastError();
}

}  // namespace

size_t gauss_bytes(int64_t k, int64_t d) { return (size_t)k * (size_t)d * (4 + 5 * 2); }

hipError_t gauss_fill(void* storage, int64_t k, int64_t d, uint32_t key1, hipStream_t st) {
  float* S32 = (float*)storage;
  uint16_t* b = (uint16_t*)(S32 + k * d);
  const int64_t blocks = (k * d + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gauss_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, st, S32, b, b + k * d,
                     b + 2 * k * d, b + 3 * k * d, b + 4 * k * d, k, d, key1);
  return hipGetLastError();
}

bool gauss_supported(int64_t k, int64_t d, const void* A, int64_t lda, int64_t n, fs_dtype dt) {
  const int64_t esz = dt == FS_F32 ? 4 : 2;
  if (d % KC || k % 128 || n < 1) return false;
  if ((uintptr_t)A % (4 * esz) || lda % 4) return false;
  if (d * lda * esz >= ((int64_t)1 << 31)) return false;  // 32-bit buffer offsets over all of A
  return (n + 255) / 256 <= 65535;  // (the widest column tile is 512)
}

hipError_t launch_gauss(const void* storage, int64_t k, int64_t d, const void* A, int64_t lda,
                        int64_t n, void* out, int64_t ldo, fs_dtype dt, hipStream_t st, EventPair ev) {
  const float* S32 = (const float*)storage;
  const uint16_t* b = (const uint16_t*)(S32 + k * d);
  const size_t esz = dt == FS_F32 ? 4 : 2;
  GaussArgs a;
  a.A = A; a.out = out; a.k = k; a.d = d; a.lda = lda; a.ldo = ldo; a.n = (int)n;
  a.stages = (int)(d / KC);
  a.out_vec = ((uintptr_t)out % (4 * esz) == 0 && (ldo * esz) % (4 * esz) == 0) ? 1 : 0;
  const unsigned col_tiles = (unsigned)((n + 255) / 256);
  if (ev.start) (void)hipEventRecord(ev.start, st);
  hipError_t e;
  if (dt == FS_BF16) {
    a.S[0] = b; a.S[1] = a.S[2] = nullptr;
    constexpr int RW = 128;
    e = go(gauss_kernel<uint16_t, 2, 2, 2>, dim3((unsigned)(k / RW), col_tiles), 256, 2 * RW * PHI_LD * 2, st, a);
  } else if (dt == FS_F16) {
    a.S[0] = b + 4 * k * d; a.S[1] = a.S[2] = nullptr;
    constexpr int RW = 128;
    e = go(gauss_kernel<f16, 2, 2, 2>, dim3((unsigned)(k / RW), col_tiles), 256, 2 * RW * PHI_LD * 2, st, a);
  } else {
    a.S[0] = b + k * d; a.S[1] = b + 2 * k * d; a.S[2] = b + 3 * k * d;
    // 128-row x 512-column work-groups when they still fill most of the chip, else 64 x 256
    const int64_t wide_tiles = (n + 511) / 512;
    if ((k / 128) * wide_tiles >= 192) {
      constexpr int RW = 128;
      e = go(gauss_kernel<float, 4, 1, 4>, dim3((unsigned)(k / RW), (unsigned)wide_tiles), 256,
             2 * 3 * RW * PHI_LD * 2, st, a);
    } else {
      constexpr int RW = 64;
      e = go(gauss_kernel<float, 1, 2, 2>, dim3((unsigned)(k / RW), col_tiles), 256, 2 * 3 * RW * PHI_LD * 2, st, a);
    }
  }
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  return e;
}

}  // namespace fs
