// BlockPerm-SJLT apply on the matrix cores (gfx950 MFMA).
//
// The s signed additions per input element of Alg. 1 cost kappa*s fp32 adds per
// element of A, which for 2-byte inputs exceeds what the vector ALUs can do at
// HBM speed.  Here a Br x Bc block Phi_{g,h} (entries 0, +1, -1) is instead
// treated as a dense bf16 matrix and Phi * A_tile is computed with
// v_mfma_f32_32x32x16_bf16 into fp32 accumulators: products with 0/+-1 are
// exact, so the result is the same sum in a different order.
//
//  * Phi is never stored in HBM: per 64-row stage of A, the work-group hashes the
//    (block, row) pairs it needs (one lane per pair, Appendix E "Within-block
//    hashing"), scatters the s nonzeros of each into a zeroed LDS tile
//    [stacked row][64 + 8 pad] and every wave reads its MFMA operand from there
//    with one 128-bit LDS read.  Three LDS tiles rotate (consume / fill / clear),
//    one barrier per stage.
//  * A goes HBM -> registers directly: a lane loads 4 consecutive columns of 8
//    rows (coalesced 256 B / 512 B row segments per half-wave) and transposes
//    them in registers with v_perm_b32 into four MFMA operands, one per column
//    residue; a wave owns 128 columns.  fp32 inputs are split exactly into three
//    bf16 pieces (8+8+8 significant bits) and take three MFMAs.
//  * Two work decompositions, both free of global atomics (Section 5, "Eliminating
//    Global Atomics"):
//      OUT-stationary  work-group = (output block g, column tile); loops over the
//                      kappa input blocks f^l(g) as in Alg. 1 (A re-read kappa times,
//                      served by L2 / Infinity Cache);
//      IN-stationary   work-group = (input block h, column tile, row split); reads
//                      its rows of A once and accumulates the kappa stacked
//                      destination blocks g_l = f^{-l}(h) (kappa*Br MFMA rows), writes
//                      them as fp32 partial planes; a second kernel adds the planes
//                      in fixed order, scales and stores (deterministic).
//
// Inputs must be finite: a dense product multiplies every element by the zeros of
// Phi as well, so an Inf/NaN in A spreads to all rows of the blocks that read it.
#include "convert.h"
#include "handle.h"
#include "spec.h"

namespace fs {

namespace {

constexpr int KC = 64;           // rows of A per stage
constexpr int KSTEPS = KC / 16;  // MFMA k-steps per stage
constexpr int PHI_LD = KC + 8;   // bf16 per LDS row of Phi (144 B: conflict-free b128 reads)
constexpr int WCOLS = 128;       // columns per wave (4 per lane x 32 lanes)
constexpr int MAX_KAPPA = 128;
constexpr uint16_t kOne = 0x3F80, kMinusOne = 0xBF80;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct MfmaArgs {
  SketchParams p;
  const void* A;
  void* out;
  float* ws;
  int64_t lda, ldo, ldw;
  int n;
  int zsplit;       // IN: row splits of an input block
  int stages;       // stages per work-group
  int out_vec;      // out rows allow 4-column vector stores
};

template <typename T> struct Ld;
template <> struct Ld<uint16_t> { using V = uint2; static constexpr int PFD = 4; };
template <> struct Ld<float>    { using V = uint4; static constexpr int PFD = 2; };

__device__ __forceinline__ uint32_t perm(uint32_t hi_src, uint32_t lo_src, uint32_t sel) {
  return __builtin_amdgcn_perm(hi_src, lo_src, sel);
}

// 4 consecutive columns of one row; lanes beyond n read nothing.
template <typename T>
__device__ __forceinline__ typename Ld<T>::V load4(const T* rowp, int col0, int n) {
  using V = typename Ld<T>::V;
  V v;
  if (col0 + 3 < n) {
    v = *reinterpret_cast<const V*>(rowp + col0);
  } else {
    T e[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) e[c] = (col0 + c < n) ? rowp[col0 + c] : (T)0;
    v = *reinterpret_cast<V*>(e);
  }
  return v;
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

__device__ __forceinline__ f32x16 mfma(uint4 a, uint4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <typename T, int MT, int NRG, int NCG, bool IN_STAT>
__global__ __launch_bounds__(64 * NRG * NCG) __attribute__((amdgpu_waves_per_eu(2)))
void mfma_kernel(MfmaArgs a) {
  using V = typename Ld<T>::V;
  constexpr int PFD = Ld<T>::PFD;
  constexpr int NW = NRG * NCG, NT = 64 * NW;
  constexpr int RW = 32 * MT * NRG;  // stacked Phi rows per work-group
  constexpr int PHI_ELEMS = RW * PHI_LD;

  __shared__ __attribute__((aligned(16))) uint16_t s_phi[3][PHI_ELEMS];
  __shared__ uint32_t s_bk[MAX_KAPPA];   // block keys per slot
  __shared__ uint32_t s_blk[MAX_KAPPA];  // IN: destination block g_l;  OUT: source block h_l

  const SketchParams& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = wave / NCG, cg = wave % NCG;
  const int kg = lane >> 5;
  const int col0 = (int)blockIdx.y * (WCOLS * NCG) + cg * WCOLS + 4 * (lane & 31);
  const uint32_t blk = blockIdx.x;  // IN: h, OUT: g
  const int z = IN_STAT ? (int)blockIdx.z : 0;
  const int T_stages = a.stages;
  const uint32_t rows_per_blk_stage = p.Bc / KC;  // stages per input block (OUT)

  // ---- slot tables -------------------------------------------------------
  for (int sl = tid; sl < (int)p.kappa; sl += NT) {
    uint32_t x = blk;
    for (int l = 0; l <= sl; ++l)
      x = IN_STAT ? wire_prev(x, p.a_inv, p.b, p.M) : wire_next(x, p.a, p.b, p.M);
    s_blk[sl] = x;
    s_bk[sl] = IN_STAT ? block_key(p.key1, x, blk, p.M) : block_key(p.key1, blk, x, p.M);
  }
  {
    uint4* z4 = reinterpret_cast<uint4*>(&s_phi[0][0]);
    for (int i = tid; i < 3 * PHI_ELEMS / 8; i += NT) z4[i] = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();

  // first row of A of global k-step kk (16 rows each) of this work-group
  auto row_of = [&](int kk) -> int64_t {
    if (IN_STAT) {
      return (int64_t)blk * p.Bc + (int64_t)z * T_stages * KC + (int64_t)kk * 16;
    } else {
      const uint32_t per_blk = p.Bc / 16;
      const uint32_t l = (uint32_t)kk / per_blk, kr = (uint32_t)kk % per_blk;
      return (int64_t)s_blk[l] * p.Bc + (int64_t)kr * 16;
    }
  };
  const T* Abase = reinterpret_cast<const T*>(a.A);
  const int total_ksteps = T_stages * KSTEPS;

  V ld[PFD][8];
  auto issue = [&](int kk, V (&dst)[8]) {
    if (kk < total_ksteps) {
      const T* rp = Abase + (row_of(kk) + kg * 8) * a.lda;
#pragma unroll
      for (int j = 0; j < 8; ++j) dst[j] = load4<T>(rp + (int64_t)j * a.lda, col0, a.n);
    }
  };

  // Scatter the nonzeros of stage t into tile `buf` (one lane per (slot, row) pair).
  auto produce = [&](int t, int buf) {
    uint16_t* phi = &s_phi[buf][0];
    if (IN_STAT) {
      const uint32_t u = (uint32_t)(z * T_stages + t) * KC + lane;
      for (uint32_t slot = wave; slot < p.kappa; slot += NW) {
        const RowHash rh = row_hash_pow2(s_bk[slot], u, p.Br);
        uint32_t r = rh.shift;
        for (uint32_t i = 0; i < p.s; ++i) {
          phi[(slot * p.Br + r) * PHI_LD + lane] = ((rh.signs >> i) & 1u) ? kMinusOne : kOne;
          r = (r + rh.stride) & (p.Br - 1);
        }
      }
    } else if (wave == 0) {
      const uint32_t l = (uint32_t)t / rows_per_blk_stage;
      const uint32_t u = ((uint32_t)t % rows_per_blk_stage) * KC + lane;
      const RowHash rh = row_hash_pow2(s_bk[l], u, p.Br);
      uint32_t r = rh.shift;
      for (uint32_t i = 0; i < p.s; ++i) {
        phi[r * PHI_LD + lane] = ((rh.signs >> i) & 1u) ? kMinusOne : kOne;
        r = (r + rh.stride) & (p.Br - 1);
      }
    }
  };

  f32x16 acc[MT][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][c][i] = 0.f;

  produce(0, 0);
#pragma unroll
  for (int i = 0; i < PFD; ++i) issue(i, ld[i]);

  for (int t = 0; t < T_stages; ++t) {
    __syncthreads();
    {  // clear the tile consumed in the previous stage, fill the next one
      uint4* z4 = reinterpret_cast<uint4*>(&s_phi[(t + 2) % 3][0]);
      for (int i = tid; i < PHI_ELEMS / 8; i += NT) z4[i] = make_uint4(0, 0, 0, 0);
      if (t + 1 < T_stages) produce(t + 1, (t + 1) % 3);
    }
    const uint16_t* phi = &s_phi[t % 3][0];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      uint4 pa[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        pa[mt] = *reinterpret_cast<const uint4*>(
            phi + ((rg * MT + mt) * 32 + (lane & 31)) * PHI_LD + ks * 16 + kg * 8);
      V(&cur)[8] = ld[ks % PFD];
      if constexpr (sizeof(T) == 2) {
        uint4 op[4];
        make_ops(cur, op);
        issue(t * KSTEPS + ks + PFD, cur);
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma(pa[mt], op[c], acc[mt][c]);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint32_t xs[8];
#pragma unroll
          for (int j = 0; j < 8; ++j)
            xs[j] = c == 0 ? cur[j].x : c == 1 ? cur[j].y : c == 2 ? cur[j].z : cur[j].w;
          uint4 hi, mid, lo;
          split_ops(xs, hi, mid, lo);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            acc[mt][c] = mfma(pa[mt], hi, acc[mt][c]);
            acc[mt][c] = mfma(pa[mt], mid, acc[mt][c]);
            acc[mt][c] = mfma(pa[mt], lo, acc[mt][c]);
          }
        }
        issue(t * KSTEPS + ks + PFD, cur);
      }
    }
  }

  // ---- epilogue ------------------------------------------------------------
  if (col0 >= a.n) return;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t row_s = (uint32_t)((rg * MT + mt) * 32 + 8 * (i >> 2) + 4 * kg + (i & 3));
      float v[4] = {acc[mt][0][i], acc[mt][1][i], acc[mt][2][i], acc[mt][3][i]};
      if (IN_STAT) {
        const uint32_t slot = row_s / p.Br, r = row_s & (p.Br - 1);
        const int64_t plane = (int64_t)z * p.kappa + slot;
        float* dst = a.ws + (plane * p.k + (int64_t)s_blk[slot] * p.Br + r) * a.ldw + col0;
        *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
      } else {
        T* dst = reinterpret_cast<T*>(a.out) + ((int64_t)blk * p.Br + row_s) * a.ldo + col0;
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] *= p.scale;
        if (a.out_vec && col0 + 3 < a.n) {
          if constexpr (sizeof(T) == 2) {
            uint2 w;
            w.x = (uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16);
            w.y = (uint32_t)f32_to_bf16_rne(v[2]) | ((uint32_t)f32_to_bf16_rne(v[3]) << 16);
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
}

// out[row][col] = scale * sum_p ws[p][row][col], planes added in index order.
template <typename T>
__global__ __launch_bounds__(256) void reduce_planes_kernel(const float* __restrict__ ws, int planes,
                                                            int64_t k, int64_t ldw, int n,
                                                            T* __restrict__ out, int64_t ldo,
                                                            float scale, int out_vec) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // over k * ldw/4
  const int64_t q = ldw / 4;
  if (idx >= k * q) return;
  const int64_t row = idx / q;
  const int col0 = (int)(idx % q) * 4;
  if (col0 >= n) return;
  const float* src = ws + row * ldw + col0;
  float4 s = *reinterpret_cast<const float4*>(src);
  for (int pl = 1; pl < planes; ++pl) {
    const float4 v = *reinterpret_cast<const float4*>(src + (int64_t)pl * k * ldw);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  float v[4] = {s.x * scale, s.y * scale, s.z * scale, s.w * scale};
  T* dst = out + row * ldo + col0;
  if (out_vec && col0 + 3 < n) {
    if constexpr (sizeof(T) == 2) {
      uint2 w;
      w.x = (uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16);
      w.y = (uint32_t)f32_to_bf16_rne(v[2]) | ((uint32_t)f32_to_bf16_rne(v[3]) << 16);
      *reinterpret_cast<uint2*>(dst) = w;
    } else {
      *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
    }
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (col0 + c < n) Elt<T>::store(dst + c, v[c]);
  }
}

// ---- host-side planning ----------------------------------------------------
struct Plan {
  bool ok = false;
  bool in_stat = false;
  int mt = 0, nrg = 0, ncg = 0, zsplit = 1, stages = 0;
  int64_t ldw = 0;
  int planes = 0;
};

bool tile_shape(uint32_t rw, int* mt, int* nrg) {
  if (rw == 32) { *mt = 1; *nrg = 1; return true; }
  if (rw == 64) { *mt = 2; *nrg = 1; return true; }
  if (rw == 128) { *mt = 2; *nrg = 2; return true; }
  return false;
}

Plan make_plan(const SketchParams& p, const void* A, int64_t lda, int64_t n, fs_dtype dt) {
  Plan pl;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  if (!p.br_pow2 || p.Bc % KC || p.kappa > (uint32_t)MAX_KAPPA || n < 1) return pl;
  if ((uintptr_t)A % (4 * esz) || (lda * esz) % (4 * esz)) return pl;  // 4-column vector loads
  pl.ncg = n > WCOLS ? 2 : 1;
  const int64_t col_tiles = (n + WCOLS * pl.ncg - 1) / (WCOLS * pl.ncg);
  if (col_tiles > 65535) return pl;

  int mt_i, nrg_i, mt_o, nrg_o;
  const bool can_in = (uint64_t)p.kappa * p.Br <= 128 && tile_shape(p.kappa * p.Br, &mt_i, &nrg_i);
  const bool can_out = tile_shape(p.Br, &mt_o, &nrg_o);
  if (!can_in && !can_out) return pl;

  // IN-stationary row split: enough work-groups to fill 256 CUs a few times over
  int zs = 1;
  while ((int64_t)p.M * col_tiles * zs < 1024 && zs < 16 && (p.Bc / (zs * 2)) % KC == 0 &&
         p.Bc / (zs * 2) >= (uint32_t)KC)
    zs *= 2;
  // workspace traffic (write + read of the partial planes) relative to reading A once
  const double rho = 2.0 * zs * p.kappa * (double)p.k * 4.0 / ((double)p.d * esz);
  const bool out_starved = (int64_t)p.M * col_tiles < 256;  // fewer output tiles than CUs
  pl.in_stat = can_in && (!can_out || rho <= 0.6 || out_starved);
  if (pl.in_stat) {
    pl.mt = mt_i; pl.nrg = nrg_i; pl.zsplit = zs;
    pl.stages = (int)(p.Bc / zs / KC);
    pl.ldw = (n + 3) & ~(int64_t)3;
    pl.planes = zs * (int)p.kappa;
    if (zs > 65535) return pl;
  } else {
    pl.mt = mt_o; pl.nrg = nrg_o; pl.zsplit = 1;
    pl.stages = (int)((uint64_t)p.kappa * p.Bc / KC);
  }
  pl.ok = true;
  return pl;
}

template <typename T, bool IN_STAT>
hipError_t launch_shape(const Plan& pl, const MfmaArgs& a, dim3 grid, hipStream_t st) {
#define FS_GO(MT, NRG, NCG) \
  hipLaunchKernelGGL((mfma_kernel<T, MT, NRG, NCG, IN_STAT>), grid, dim3(64 * NRG * NCG), 0, st, a)
  if (pl.ncg == 1) {
    if (pl.mt == 1) FS_GO(1, 1, 1); else if (pl.nrg == 1) FS_GO(2, 1, 1); else FS_GO(2, 2, 1);
  } else {
    if (pl.mt == 1) FS_GO(1, 1, 2); else if (pl.nrg == 1) FS_GO(2, 1, 2); else FS_GO(2, 2, 2);
  }
#undef FS_GO
  return hipGetLastError();
}

}  // namespace

bool mfma_supported(const SketchParams& p, const void* A, int64_t lda, int64_t n, const void* out,
                    int64_t ldo, fs_dtype dt) {
  (void)out; (void)ldo;
  return make_plan(p, A, lda, n, dt).ok;
}

size_t mfma_workspace_bytes(const SketchParams& p, int64_t n, fs_dtype dt) {
  const int64_t ld = (n + 7) & ~(int64_t)7;
  const Plan pl = make_plan(p, (const void*)(uintptr_t)256, ld, n, dt);
  if (!pl.ok || !pl.in_stat) return 0;
  return (size_t)pl.planes * (size_t)p.k * (size_t)pl.ldw * sizeof(float);
}

hipError_t launch_mfma(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                       int64_t ldo, fs_dtype dt, void* ws, hipStream_t st, EventPair ev) {
  const Plan pl = make_plan(p, A, lda, n, dt);
  if (!pl.ok) return hipErrorInvalidValue;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  MfmaArgs a;
  a.p = p; a.A = A; a.out = out; a.ws = (float*)ws;
  a.lda = lda; a.ldo = ldo; a.ldw = pl.ldw; a.n = (int)n;
  a.zsplit = pl.zsplit; a.stages = pl.stages;
  a.out_vec = ((uintptr_t)out % (4 * esz) == 0 && (ldo * esz) % (4 * esz) == 0) ? 1 : 0;
  const unsigned col_tiles = (unsigned)((n + WCOLS * pl.ncg - 1) / (WCOLS * pl.ncg));
  dim3 grid(p.M, col_tiles, pl.in_stat ? pl.zsplit : 1);

  if (ev.start) (void)hipEventRecord(ev.start, st);
  hipError_t e;
  if (dt == FS_BF16)
    e = pl.in_stat ? launch_shape<uint16_t, true>(pl, a, grid, st) : launch_shape<uint16_t, false>(pl, a, grid, st);
  else
    e = pl.in_stat ? launch_shape<float, true>(pl, a, grid, st) : launch_shape<float, false>(pl, a, grid, st);
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  if (e != hipSuccess || !pl.in_stat) return e;

  const int64_t work = p.k * (pl.ldw / 4);
  const unsigned blocks = (unsigned)((work + 255) / 256);
  if (dt == FS_BF16)
    hipLaunchKernelGGL(reduce_planes_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, a.ws, pl.planes,
                       p.k, pl.ldw, (int)n, (uint16_t*)out, ldo, p.scale, a.out_vec);
  else
    hipLaunchKernelGGL(reduce_planes_kernel<float>, dim3(blocks), dim3(256), 0, st, a.ws, pl.planes,
                       p.k, pl.ldw, (int)n, (float*)out, ldo, p.scale, a.out_vec);
  return hipGetLastError();
}

}  // namespace fs
