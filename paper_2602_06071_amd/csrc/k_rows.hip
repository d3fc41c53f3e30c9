// BlockPerm-SJLT apply for inputs held "examples as rows": G is n x d row-major (every row is
// one vector to sketch, e.g. one example's gradient) and out = G S^T is n x k row-major, i.e.
// out[i, :] = S G[i, :].  The same linear map as the column layout (Alg. 1), only transposed.
//
// On the matrix cores this layout is the natural one: with D (examples x stacked output rows)
// = G_tile (examples x K) * Phi^T (K x stacked rows) a lane's MFMA operand is 8 consecutive
// K-values of ONE example row, which is 16 contiguous bytes of G: the operand is loaded
// straight from HBM with one 128-bit buffer load, no register transposition.  K-values may be
// assigned to MFMA k-steps in any order as long as both operands agree, so lane half kg takes
// the K-range [32 kg, 32 kg + 32) of a 64-row stage and k-step j its j-th group of 8: the two
// halves of a wave then read 128 contiguous bytes of every example row per stage.
//
//  * input-stationary (one wave = one work-group): (input block h, 32*ET examples, row split z)
//    reads its K-range of G once and accumulates the kappa stacked destination blocks
//    g_l = f^{-l}(h) (kappa*Br = 32*MT MFMA columns); fp32 partial planes [plane][example][k]
//    and the fixed-order plane reduction give `out` without atomics on data;
//  * Phi^T is generated exactly as in the column layout: per 64-row stage one lane per input
//    row hashes its kappa slots (Appendix E, "Within-block hashing") and scatters +-1 as bf16
//    into the wave's own LDS tile [stacked row][64 + 8]; two tiles alternate, no barrier;
//  * fp32 inputs: exact three-way bf16 split of the 8 values a lane holds, three MFMAs.
//
// Shapes: power-of-two Br with kappa*Br in {32, 64, 128}, Bc a multiple of 64 that divides d,
// 16-byte aligned rows.  Inputs must be finite (a dense product also multiplies by the zeros).
#include <type_traits>

#include "handle.h"
#include "mfma_common.h"
#include "spec.h"

namespace fs {

namespace {

using namespace mm;

struct RowsArgs {
  SketchParams p;
  const void* G;
  float* ws;
  int64_t ldg, ldw;
  int n;        // examples
  int stages;   // 64-row stages per work-group
  uint32_t log2_br;
};

template <typename T> struct RowLd;  // what a lane loads per (example tile, k-step): 8 K-values
template <> struct RowLd<uint16_t> { static constexpr int NV = 1; };  // one b128
template <> struct RowLd<float>    { static constexpr int NV = 2; };  // two b128

template <typename T, int MT, int ET>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2)))
void rows_kernel(RowsArgs a) {
  constexpr int NV = RowLd<T>::NV;
  constexpr int RWV = 32 * MT;         // stacked output rows = kappa * Br
  constexpr int TILE = RWV * PHI_LD;   // bf16 elements of one Phi tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const SketchParams& p = a.p;
  const int lane = (int)threadIdx.x;
  const int m = lane & 31, kg = lane >> 5;
  uint32_t* s_bk = reinterpret_cast<uint32_t*>(smem);   // [MAX_KAPPA] block keys per slot
  uint32_t* s_blk = s_bk + MAX_KAPPA;                   // [MAX_KAPPA] destination block g_l
  uint16_t* s_phi = reinterpret_cast<uint16_t*>(smem + 2 * MAX_KAPPA * 4);

  const uint32_t blk = blockIdx.x;  // input block h
  const int ex0 = (int)blockIdx.y * (32 * ET);
  const int z = (int)blockIdx.z;
  const int T_stages = a.stages;
  const uint32_t lbr = a.log2_br;

  // slot tables and empty tiles
  for (int sl = lane; sl < (int)p.kappa; sl += 64) {
    uint32_t x = blk;
    for (int l = 0; l <= sl; ++l) x = wire_prev(x, p.a_inv, p.b, p.M);
    s_blk[sl] = x;
    s_bk[sl] = block_key(p.key1, x, blk, p.M);
  }
  {
    uint4* z4 = reinterpret_cast<uint4*>(s_phi);
    static_assert((2 * TILE / 8) % 64 == 0, "two tiles are a whole number of 64-lane stores");
#pragma unroll
    for (int i = 0; i < 2 * TILE / 8 / 64; ++i) z4[lane + i * 64] = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();  // one wave: orders the table writes before the reads by other lanes

  // ---- loads ---------------------------------------------------------------------------
  // One descriptor per wave: base = first example row of the wave at the first K of its range;
  // the range ends with the last valid example row, so rows at or beyond n read as 0 without
  // touching memory (lanes of such rows get the out-of-range offset 2^31 outright).
  const int64_t row_bytes = a.ldg * (int64_t)sizeof(T);
  const int rows_valid = min(32 * ET, a.n - ex0);
  const int64_t k_first = (int64_t)blk * p.Bc + (int64_t)z * T_stages * KC;
  const int64_t range =
      rows_valid > 0 ? (int64_t)(rows_valid - 1) * row_bytes + (int64_t)T_stages * KC * (int64_t)sizeof(T) : 0;
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(reinterpret_cast<const char*>(a.G) + (int64_t)ex0 * row_bytes +
                        k_first * (int64_t)sizeof(T)),
      0, (int)(uint32_t)range, 0x00020000);
  uint32_t voff[ET];
#pragma unroll
  for (int c = 0; c < ET; ++c)
    voff[c] = c * 32 + m < rows_valid
                  ? (uint32_t)((int64_t)(c * 32 + m) * row_bytes + (int64_t)kg * 32 * (int64_t)sizeof(T))
                  : 0x80000000u;

  // Prefetch ring of R example tiles, each with all four k-steps of a stage: the four 16-byte
  // pieces a lane takes from one 128-byte line (bf16; two lines for fp32) are requested back to
  // back, so the line is fetched once.  (Requesting them one k-step at a time, a stage apart,
  // re-fetched every line four times: 1.9 TB/s instead of the rate below.)
  constexpr int R = sizeof(T) == 2 ? ET : 2;
  static_assert(ET % R == 0, "the ring divides a stage");
  uint4 ld[R][KSTEPS][NV];
  auto issue_tile = [&](int t, int c, uint4 (&dst)[KSTEPS][NV]) {
    // stage t, example tile c: K offset 64 t + 8 j for k-step j (+ 32 kg in voff)
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j)
#pragma unroll
      for (int v = 0; v < NV; ++v)
        dst[j][v] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(
            rs, voff[c], (uint32_t)(t * KC + j * 8) * (uint32_t)sizeof(T) + 16u * v, 0));
  };

  f32x16 acc[ET][MT];
#pragma unroll
  for (int c = 0; c < ET; ++c)
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[c][rt][i] = 0.f;

  // ---- Phi^T: part `part` of a stage takes every 4th slot ---------------------------------
  auto produce = [&](int t, int buf, int part) {
    uint16_t* phi = s_phi + buf * TILE;
    const uint32_t u = (uint32_t)(z * T_stages + t) * KC + lane;
    for (uint32_t slot = part; slot < p.kappa; slot += KSTEPS) {
      const RowHash rh = row_hash_pow2(s_bk[slot], u, p.Br);
      uint32_t r = rh.shift;
      const uint32_t base = slot << lbr;
      for (uint32_t i = 0; i < p.s; ++i) {
        phi[__umul24(base + r, (uint32_t)PHI_LD) + lane] = (uint16_t)(((rh.signs >> i) << 15) | kOne);
        r = (r + rh.stride) & (p.Br - 1);
      }
    }
  };
  auto clear_tile = [&](int buf) {
    uint4* z4 = reinterpret_cast<uint4*>(s_phi + buf * TILE);
#pragma unroll
    for (int i = 0; i < (TILE / 8 + 63) / 64; ++i)
      if (TILE / 8 % 64 == 0 || lane + i * 64 < TILE / 8) z4[lane + i * 64] = make_uint4(0, 0, 0, 0);
  };

  auto stage = [&](int t, auto last_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    const uint16_t* phi = s_phi + (t & 1) * TILE;
    uint4 pb[KSTEPS][MT];  // Phi^T operands: stacked row rt*32 + m, K = 32 kg + 8 j .. + 7
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j)
#pragma unroll
      for (int rt = 0; rt < MT; ++rt)
        pb[j][rt] = *reinterpret_cast<const uint4*>(phi + (rt * 32 + m) * PHI_LD + kg * 32 + j * 8);
#pragma unroll
    for (int c = 0; c < ET; ++c) {
      if constexpr (!LAST) {
#pragma unroll
        for (int part = c * KSTEPS / ET; part < (c + 1) * KSTEPS / ET; ++part) produce(t + 1, (t + 1) & 1, part);
      }
      uint4(&cur)[KSTEPS][NV] = ld[c % R];
      // the tile R places further on: same stage, or the next one
      const int CN = (c + R) % ET;  // compile-time after unrolling
      const bool wrap = c + R >= ET;
      const bool fetch = !(LAST && wrap);  // compile-time after unrolling
      if constexpr (sizeof(T) == 2) {
        uint4 g[KSTEPS];
#pragma unroll
        for (int j = 0; j < KSTEPS; ++j) g[j] = cur[j][0];
        if (fetch) issue_tile(wrap ? t + 1 : t, CN, cur);
#pragma unroll
        for (int j = 0; j < KSTEPS; ++j)
#pragma unroll
          for (int rt = 0; rt < MT; ++rt) acc[c][rt] = mfma(g[j], pb[j][rt], acc[c][rt]);
      } else {
#pragma unroll
        for (int jj = 0; jj < KSTEPS; jj += 2) {
          uint4 pc[2][3];
#pragma unroll
          for (int cc = 0; cc < 2; ++cc) {
            const uint32_t xs[8] = {cur[jj + cc][0].x, cur[jj + cc][0].y, cur[jj + cc][0].z, cur[jj + cc][0].w,
                                    cur[jj + cc][1].x, cur[jj + cc][1].y, cur[jj + cc][1].z, cur[jj + cc][1].w};
            split_ops(xs, pc[cc][0], pc[cc][1], pc[cc][2]);
          }
#pragma unroll
          for (int piece = 0; piece < 3; ++piece)
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
              for (int rt = 0; rt < MT; ++rt)
                acc[c][rt] = mfma(pc[cc][piece], pb[jj + cc][rt], acc[c][rt]);
        }
        if (fetch) issue_tile(wrap ? t + 1 : t, CN, cur);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (!LAST) clear_tile(t & 1);
  };

  if (rows_valid > 0) {
#pragma unroll
    for (int c = 0; c < R; ++c) issue_tile(0, c, ld[c]);
#pragma unroll
    for (int part = 0; part < KSTEPS; ++part) produce(0, 0, part);
    for (int t = 0; t + 1 < T_stages; ++t) stage(t, std::false_type{});
    stage(T_stages - 1, std::true_type{});
  }

  // ---- epilogue: accumulator v of tile (c, rt) is example ex0 + 32 c + 8 (v/4) + 4 kg + v%4,
  // stacked row 32 rt + m; a half-wave writes 32 consecutive stacked rows of one example
#pragma unroll
  for (int rt = 0; rt < MT; ++rt) {
    const uint32_t srow = (uint32_t)(rt * 32 + m);
    const uint32_t slot = srow >> lbr, r = srow & (p.Br - 1);
    if (slot >= p.kappa) continue;
    const int64_t plane = (int64_t)z * p.kappa + slot;
    float* col = a.ws + plane * a.n * a.ldw + (int64_t)s_blk[slot] * p.Br + r;
#pragma unroll
    for (int c = 0; c < ET; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ex = c * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
        if (ex < rows_valid) col[(int64_t)(ex0 + ex) * a.ldw] = acc[c][rt][v];
      }
  }
}

struct RowsPlan {
  bool ok = false;
  int mt = 0, et = 0, zsplit = 1, stages = 0, planes = 0;
  int64_t ldw = 0;
  size_t lds = 0;
};

RowsPlan make_rows_plan(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt) {
  RowsPlan pl;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  if (!p.br_pow2 || p.Bc % KC || p.d % p.Bc || p.kappa > (uint32_t)MAX_KAPPA || n < 1) return pl;
  const uint64_t rw = (uint64_t)p.kappa * p.Br;
  if (rw == 32) { pl.mt = 1; pl.et = 4; }
  else if (rw == 64) { pl.mt = 2; pl.et = 4; }
  else if (rw == 128) { pl.mt = 4; pl.et = 2; }
  else return pl;
  if ((uintptr_t)G % 16 || (ldg * (int64_t)esz) % 16) return pl;         // 128-bit loads
  if (128 * ldg * (int64_t)esz >= ((int64_t)1 << 31)) return pl;          // 32-bit lane offsets and range
  const int64_t ex_tiles = (n + 32 * pl.et - 1) / (32 * pl.et);
  if (ex_tiles > 65535) return pl;
  // row split: the traffic model of the column layout (G at ~6 TB/s once 1024 waves exist,
  // planes written at ~3.4 TB/s and read back at ~6 TB/s)
  const double g_bytes = (double)p.d * (double)n * esz;
  double best = 0;
  for (int zc = 1; zc <= 16; zc *= 2) {
    if (zc > 1 && ((p.Bc / zc) % KC != 0 || p.Bc / zc < (uint32_t)KC)) break;
    const double waves = (double)p.M * ex_tiles * zc;
    const double plane_bytes = (double)zc * p.kappa * (double)p.k * (double)n * 4.0;
    const double t = g_bytes / (6e12 * (waves < 1024 ? waves / 1024 : 1.0)) + plane_bytes / 3.4e12 +
                     plane_bytes / 6e12;
    if (zc == 1 || t < best) { best = t; pl.zsplit = zc; }
  }
  pl.stages = (int)(p.Bc / pl.zsplit / KC);
  pl.planes = pl.zsplit * (int)p.kappa;
  pl.ldw = (p.k + 3) & ~(int64_t)3;
  pl.lds = 2 * MAX_KAPPA * 4 + 2 * (size_t)(32 * pl.mt) * PHI_LD * 2;
  pl.ok = true;
  return pl;
}

template <typename K>
hipError_t go(K kernel, dim3 grid, size_t lds, hipStream_t st, const RowsArgs& a) {
  hipLaunchKernelGGL(kernel, grid, dim3(64), lds, st, a);
  return hipGetLastError();
}

}  // namespace

bool rows_supported(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt) {
  return make_rows_plan(p, G, ldg, n, dt).ok;
}

size_t rows_workspace_bytes(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt) {
  const RowsPlan pl = make_rows_plan(p, G, ldg, n, dt);
  if (!pl.ok) return 0;
  return (size_t)pl.planes * (size_t)n * (size_t)pl.ldw * sizeof(float);
}

hipError_t launch_rows(const SketchParams& p, const void* G, int64_t ldg, int64_t n, void* out,
                       int64_t ldo, fs_dtype dt, void* ws, hipStream_t st, EventPair ev) {
  const RowsPlan pl = make_rows_plan(p, G, ldg, n, dt);
  if (!pl.ok) return hipErrorInvalidValue;
  RowsArgs a;
  a.p = p; a.G = G; a.ws = (float*)ws;
  a.ldg = ldg; a.ldw = pl.ldw; a.n = (int)n;
  a.stages = pl.stages;
  a.log2_br = 0;
  while ((1u << a.log2_br) < p.Br) ++a.log2_br;
  const dim3 grid(p.M, (unsigned)((n + 32 * pl.et - 1) / (32 * pl.et)), pl.zsplit);

  if (ev.start) (void)hipEventRecord(ev.start, st);
  hipError_t e;
  if (dt == FS_BF16) {
    e = pl.mt == 1   ? go(rows_kernel<uint16_t, 1, 4>, grid, pl.lds, st, a)
        : pl.mt == 2 ? go(rows_kernel<uint16_t, 2, 4>, grid, pl.lds, st, a)
                     : go(rows_kernel<uint16_t, 4, 2>, grid, pl.lds, st, a);
  } else {
    e = pl.mt == 1   ? go(rows_kernel<float, 1, 4>, grid, pl.lds, st, a)
        : pl.mt == 2 ? go(rows_kernel<float, 2, 4>, grid, pl.lds, st, a)
                     : go(rows_kernel<float, 4, 2>, grid, pl.lds, st, a);
  }
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  if (e != hipSuccess) return e;
  // out[i][c] = scale * sum over planes: the plane reduction of the column layout with the
  // roles of rows and columns exchanged (n example rows of k columns)
  return launch_reduce_planes(a.ws, pl.planes, n, pl.ldw, p.k, out, ldo, p.scale, dt, st);
}

}  // namespace fs
