// BlockPerm-SJLT apply for inputs held "examples as rows": G is n x d row-major (every row is
// one vector to sketch, e.g. one example's gradient) and out = G S^T is n x k row-major, i.e.
// out[i, :] = S G[i, :].  The same linear map as the column layout (Alg. 1), only transposed.
//
// With D (examples x stacked output rows) = G_tile (examples x K) * Phi^T (K x stacked rows) a
// lane's MFMA operand is 8 consecutive K-values of ONE example row: 16 contiguous bytes of G,
// no register transposition.  Loading the operands in that very lane order would touch 32
// different rows with 32 bytes each per instruction, which the memory system serves at less
// than half the streaming rate (measured with a read-only probe: 2.6 TB/s at a power-of-two row
// stride, 5.4 TB/s at best).  So G is loaded coalesced -- 8 (bf16) or 16 (fp32) lanes cover the
// 128 / 256 contiguous bytes a row contributes to a 64-value stage, 5.9-6.3 TB/s in the same
// probe -- and each 32-example tile is passed through a small padded LDS tile of the wave to
// reach the operand order (LDS operations of one wave complete in order: no barrier).
//
//  * input-stationary (one wave = one work-group): (input block h, 32*ET examples, row split z)
//    reads its K-range of G once and accumulates the kappa stacked destination blocks
//    g_l = f^{-l}(h) (kappa*Br <= 32*MT MFMA columns); fp32 partial results stored by input
//    block and a fixed-order gather-reduction give `out` without atomics on data;
//  * Phi^T is generated exactly as in the column layout: per 64-row stage one lane per input
//    row hashes its kappa slots (Appendix E, "Within-block hashing") and scatters +-1 as bf16
//    into the wave's own LDS tile [stacked row][64 + 8] (one tile: a stage reads all its
//    operands first, then the tile is cleared and refilled behind those reads);
//  * fp32 inputs: exact three-way bf16 split of the 8 values a lane holds, three MFMAs;
//  * the prefetch ring holds whole example tiles (all lines of a tile are requested together).
//
// Shapes: power-of-two Br (kappa*Br <= 128: tile height 32, 64 or 128, rows above kappa*Br idle;
// more: Br < 32 in groups of wiring slots, Br in {32, 64, 128} output-stationary), any Bc and
// alignment (128-bit loads need G, ldg and Bc to be multiples of 16 bytes).  Inputs must be finite (a dense
// product also multiplies by the zeros).
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
  const uint32_t* orbit;  // 2M words: block at each orbit position of f from block 0, then the inverse (or NULL)
  void* out;              // OUT mode: the result itself
  int64_t ldg, ldo;
  int n;        // examples
  int stages;   // 64-row stages per work-group
  int zsplit;       // IN: row splits of an input block
  int group_slots;  // IN: wiring slots one work-group stacks (grid.z = zsplit * slot groups)
  int nsub;         // OUT, Br > 128: 128-row slices of an output block (grid.y = example tiles * nsub)
  uint32_t log2_br;
};

// OUT: output-stationary instead (Alg. 1's order): the wave owns output block g for its examples,
// walks the kappa input blocks f^l(g) with Br = 32*MT MFMA columns, and stores the scaled result
// itself; G is read kappa times (the re-reads hit L2 when neighbouring waves are in step), there
// are no partial results.  Used when kappa*Br is more than one wave can accumulate.
// fp32 with 64 stacked rows and every type with 128 get the whole register file of a SIMD (one
// wave): with two waves fp32 spills its accumulators and split operands, and a 128-row tile with
// four example tiles (256 accumulators, in AGPRs) reuses every Phi^T operand twice as often.
// UNAL = 1: rows are only 4-byte aligned (G or ldg*sizeof(T) not a multiple of 16): every 16-byte
// piece is loaded as four dwords.  UNAL = 2 (16-bit types): rows are only 2-byte aligned (odd
// ldg): eight element loads per piece, and a ring of two example tiles.
// BIG (input-stationary only): rows so long that 128 of them span 2^31 bytes get one buffer
// descriptor per 32-example tile instead of one per wave (2 % slower on the gradient workload).
template <typename T, int MT, int ET, bool OUT, int UNAL = 0, bool BIG = false>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu((sizeof(T) == 4 && MT >= 2) || MT == 4 ? 1 : 2)))
void rows_kernel(RowsArgs a) {
  constexpr int RWV = 32 * MT;         // tile height: kappa * Br stacked output rows, rounded up
  constexpr int TILE = RWV * PHI_LD;   // bf16 elements of the Phi tile
  constexpr int ROWB = KC * (int)sizeof(T);   // bytes of a row per stage: 128 / 256
  constexpr int GLD = ROWB + 16;              // LDS row of the transposition tile (conflict-free b128)
  constexpr int LPR = ROWB / 16;              // lanes per row: 8 / 16
  constexpr int RPI = 64 / LPR;               // rows per load instruction: 8 / 4
  constexpr int NLD = 32 / RPI;               // 16-byte loads per lane and 32-example tile: 4 / 8
  constexpr int NV = (int)sizeof(T) / 2;      // 16-byte loads per k-step operand: 1 / 2
  static_assert(NLD == KSTEPS * NV, "what a lane loads of a tile is what it uses as operands of a stage");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const SketchParams& p = a.p;
  const int lane = (int)threadIdx.x;
  const int m = lane & 31, kg = lane >> 5;
  uint32_t* s_bk = reinterpret_cast<uint32_t*>(smem);   // [MAX_KAPPA] block keys per slot
  uint32_t* s_blk = s_bk + MAX_KAPPA;                   // [MAX_KAPPA] destination block g_l
  uint16_t* s_phi = reinterpret_cast<uint16_t*>(smem + 2 * MAX_KAPPA * 4);
  unsigned char* s_g = smem + 2 * MAX_KAPPA * 4 + TILE * 2;  // transposition tile: [32][GLD] bytes

  // Which (block, example tile) this wave takes.  OUT with an orbit table: work-groups are
  // renumbered so that the ones an XCD runs side by side (the hardware deals linear ids
  // round-robin over the 8 XCDs) are consecutive orbit positions of one example tile, and each
  // visits its kappa neighbours in the order of their orbit position modulo kappa: the kappa
  // readers of an input block then touch it at the same time and the re-reads hit that XCD's L2.
  uint32_t blk = blockIdx.x;  // input block h (OUT: output block g)
  uint32_t ey = blockIdx.y, opos = 0;
  const bool remap = OUT && a.orbit != nullptr;
  if (remap) {
    const uint32_t total = gridDim.x * gridDim.y;
    uint32_t id = blockIdx.y * gridDim.x + blockIdx.x;
    if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
    opos = id % gridDim.x;
    ey = id / gridDim.x;
    blk = __builtin_amdgcn_readfirstlane(a.orbit[opos]);
  }
  // OUT with blocks higher than the tile: the wave owns rows [row_lo, row_lo + 32*MT) of its block
  uint32_t row_lo = 0;
  if (OUT && a.nsub > 1) {
    row_lo = (ey % (uint32_t)a.nsub) * RWV;
    ey /= (uint32_t)a.nsub;
  }
  const int ex0 = (int)ey * (32 * ET);
  // IN with kappa*Br above the tile height: grid.z also numbers groups of `group_slots` wiring
  // slots; a work-group serves the slots [slot0, slot0 + kap) and G is read once per group
  const int z = OUT ? 0 : (int)(blockIdx.z % (uint32_t)a.zsplit);
  const uint32_t slot0 = OUT ? 0u : (blockIdx.z / (uint32_t)a.zsplit) * (uint32_t)a.group_slots;
  const uint32_t kap = OUT ? p.kappa : min(p.kappa - slot0, (uint32_t)a.group_slots);
  const int T_stages = a.stages;
  const uint32_t lbr = a.log2_br;

  // slot tables and an empty tile
  for (int sl = lane; sl < (int)kap; sl += 64) {
    uint32_t x = blk;
    if (remap) {
      const uint32_t l = (sl + p.kappa - (opos + 1) % p.kappa) % p.kappa;  // 0 .. kappa-1
      x = a.orbit[(opos + 1 + l) % p.M];
    } else {
      for (int l = 0; l <= (int)slot0 + sl; ++l) x = OUT ? wire_next(x, p.a, p.b, p.M) : wire_prev(x, p.a_inv, p.b, p.M);
    }
    s_blk[sl] = x;
    s_bk[sl] = OUT ? block_key(p.key1, blk, x, p.M) : block_key(p.key1, x, blk, p.M);
  }
  auto clear_tile = [&]() {
    uint4* z4 = reinterpret_cast<uint4*>(s_phi);
#pragma unroll
    for (int i = 0; i < (TILE / 8 + 63) / 64; ++i)
      if (TILE / 8 % 64 == 0 || lane + i * 64 < TILE / 8) z4[lane + i * 64] = make_uint4(0, 0, 0, 0);
  };
  clear_tile();
  __syncthreads();  // one wave: orders the table writes before the reads by other lanes

  // ---- loads ---------------------------------------------------------------------------
  // One descriptor per wave (BIG: per 32-example tile): base = its first example row; the range
  // ends with its last valid example row, so rows at or beyond n read as 0 without touching
  // memory.  The scalar offset selects example tile (not BIG), row group and the stage's K-range;
  // the lane offset the row in the group and the 16-byte piece.
  // K-values of k-step j in lane half kg: 16 j + 8 kg.
  const int64_t row_bytes = a.ldg * (int64_t)sizeof(T);
  const int rows_valid = min(32 * ET, a.n - ex0);
  const int64_t last_row_bytes =
      // (the last row's end rounded up to a dword: range checks are per dword, and the dword that
      // holds entry d-1 must not count as outside; its other half lies in the same aligned word,
      // hence in mapped memory, and is cleared with the rest of the tail.  Element loads, UNAL = 2,
      // are checked per element and get the exact end: their rows need not start on a dword.)
      UNAL == 2 ? p.d * (int64_t)sizeof(T) : (p.d * (int64_t)sizeof(T) + 3) & ~(int64_t)3;
  constexpr int ND = BIG ? ET : 1;      // descriptors
  constexpr int DR = BIG ? 32 : 32 * ET;  // example rows each covers
  __amdgpu_buffer_rsrc_t rs_t[ND];
#pragma unroll
  for (int c = 0; c < ND; ++c) {
    const int valid = min(DR, rows_valid - DR * c);
    const int64_t range = valid > 0 ? (int64_t)(valid - 1) * row_bytes + last_row_bytes : 0;
    rs_t[c] = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(a.G) + (int64_t)(ex0 + DR * c) * row_bytes), 0,
        (int)(uint32_t)range, 0x00020000);
  }
  // Byte offset in a row of a stage's first K-value.  IN: the wave's own K-range.  OUT: stage t
  // lies in input block s_blk[t / spb]; (sl_n, st_n, kb_n) describe stage "current + 1" and are
  // stepped once per stage, kb_c is the current stage's offset.
  // stages per input block; the last one may reach past the block (Bc not a multiple of 64):
  // Phi^T gets no nonzeros for those K-values, so the neighbouring block's entries count as 0
  const uint32_t spb = (p.Bc + KC - 1) / KC;
  uint32_t sl_n = 0, st_n = 0;
  uint32_t kb_c = OUT ? (uint32_t)__builtin_amdgcn_readfirstlane(s_blk[0]) * p.Bc * (uint32_t)sizeof(T)
                      : (uint32_t)(((int64_t)blk * p.Bc + (int64_t)z * T_stages * KC) * (int64_t)sizeof(T));
  uint32_t kb_n = kb_c;
  auto step_next = [&]() {  // (sl_n, st_n, kb_n) <- the stage after the one they describe
    if constexpr (OUT) {
      if (++st_n == spb) { st_n = 0; ++sl_n; }
      const uint32_t hb = __builtin_amdgcn_readfirstlane(s_blk[min(sl_n, p.kappa - 1)]);
      kb_n = (hb * p.Bc + st_n * KC) * (uint32_t)sizeof(T);
    } else {
      kb_n += ROWB;
    }
  };
  const uint32_t voff = (uint32_t)((int64_t)(lane / LPR) * row_bytes + (lane % LPR) * 16);
  unsigned char* g_wr = s_g + (lane / LPR) * GLD + (lane % LPR) * 16;
  const unsigned char* g_rd = s_g + m * GLD + kg * (8 * (int)sizeof(T));
  const int phi_k = kg * 8;  // + 16 j

  // Prefetch ring of R example tiles, a whole stage of each: the lines of a tile are requested
  // back to back, once.  (Requesting them one k-step at a time, a stage apart, re-fetched every
  // line four times.)
  constexpr int R = sizeof(T) == 2 && UNAL != 2 ? ET : 2;
  static_assert(ET % R == 0, "the ring divides a stage");
  uint4 ld[R][NLD];
  auto issue_tile = [&](uint32_t kb, int c, uint4 (&dst)[NLD]) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const __amdgpu_buffer_rsrc_t rs = rs_t[BIG ? c : 0];
      const uint32_t so = (uint32_t)((BIG ? 0 : c * 32) + i * RPI) * (uint32_t)row_bytes + kb;
      if constexpr (UNAL == 2) {
        typedef unsigned short us8 __attribute__((ext_vector_type(8)));
        us8 e;
#pragma unroll
        for (int c = 0; c < 8; ++c)
          e[c] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, voff + 2u * c, so, 0);
        dst[i] = __builtin_bit_cast(uint4, e);
      } else if constexpr (UNAL == 1) {
        dst[i].x = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, voff, so, 0);
        dst[i].y = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, voff + 4u, so, 0);
        dst[i].z = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, voff + 8u, so, 0);
        dst[i].w = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, voff + 12u, so, 0);
      } else {
        dst[i] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, so, 0));
      }
    }
  };

  f32x16 acc[ET][MT];
#pragma unroll
  for (int c = 0; c < ET; ++c)
#pragma unroll
    for (int rt = 0; rt < MT; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[c][rt][i] = 0.f;

  // ---- Phi^T of the stage (sl_n, st_n) / t: IN: part `part` takes every 4th slot; OUT: the one
  // block of the stage, in part 0 -----------------------------------------------------------
  auto produce = [&](int t, int part) {
    if constexpr (OUT) {
      if (part != 0) return;
      const uint32_t u = st_n * KC + lane;
      const RowHash rh = row_hash_pow2(s_bk[sl_n], u, p.Br);
      uint32_t r = rh.shift;
      const uint32_t cnt = u < p.Bc ? p.s : 0u;
      if (a.nsub > 1) {  // (wave-uniform) keep the nonzeros that fall into this wave's slice
        for (uint32_t i = 0; i < cnt; ++i) {
          const uint32_t local = r - row_lo;  // unsigned: rows below the slice wrap high
          if (local < (uint32_t)RWV)
            s_phi[__umul24(local, (uint32_t)PHI_LD) + lane] = (uint16_t)(((rh.signs >> i) << 15) | Fmt<T>::one);
          r = (r + rh.stride) & (p.Br - 1);
        }
      } else {
        for (uint32_t i = 0; i < cnt; ++i) {
          s_phi[__umul24(r, (uint32_t)PHI_LD) + lane] = (uint16_t)(((rh.signs >> i) << 15) | Fmt<T>::one);
          r = (r + rh.stride) & (p.Br - 1);
        }
      }
      return;
    }
    const uint32_t u = (uint32_t)(z * T_stages + t) * KC + lane;
    if (u >= p.Bc) return;  // past the block
    if (!p.br_pow2) {  // (wave-uniform) slots of 2^lbr >= Br rows; the general row hash, wrap by compare
      for (uint32_t slot = part; slot < kap; slot += KSTEPS) {
        const RowHash rh = row_hash_any(s_bk[slot], u, p.Br);
        uint32_t r = rh.shift;
        const uint32_t base = slot << lbr;
        for (uint32_t i = 0; i < p.s; ++i) {
          s_phi[__umul24(base + r, (uint32_t)PHI_LD) + lane] = (uint16_t)(((rh.signs >> i) << 15) | Fmt<T>::one);
          r += rh.stride;
          if (r >= p.Br) r -= p.Br;
        }
      }
      return;
    }
    for (uint32_t slot = part; slot < kap; slot += KSTEPS) {
      const RowHash rh = row_hash_pow2(s_bk[slot], u, p.Br);
      uint32_t r = rh.shift;
      const uint32_t base = slot << lbr;
      for (uint32_t i = 0; i < p.s; ++i) {
        s_phi[__umul24(base + r, (uint32_t)PHI_LD) + lane] = (uint16_t)(((rh.signs >> i) << 15) | Fmt<T>::one);
        r = (r + rh.stride) & (p.Br - 1);
      }
    }
  };

  // One stage.  All Phi^T operands of the stage are read into registers first; LDS operations
  // of a wave complete in order, so the one tile can be cleared and refilled for the next stage
  // right behind those reads.
  // Entries of a vector at or beyond d (the zero padding of a partly filled last input block) are
  // whatever follows in memory: the row's own padding or the next example.  They are cleared in
  // registers, in the few stages that reach that far.
  const int d_bytes = (int)(p.d * (int64_t)sizeof(T));
  auto dword_mask = [](int rem) -> uint32_t {  // rem = valid bytes from this dword on
    return rem >= 4 ? 0xFFFFFFFFu : rem >= 2 ? 0x0000FFFFu : 0u;
  };
  auto stage = [&](int t, auto last_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    const int tail_bytes = d_bytes - (int)kb_c;  // bytes of this stage's K-range that lie before entry d
    const bool tail = tail_bytes < ROWB;
    uint4 pb[KSTEPS][MT];  // stacked row rt*32 + m, the K-values of (k-step j, half kg)
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j)
#pragma unroll
      for (int rt = 0; rt < MT; ++rt)
        pb[j][rt] = *reinterpret_cast<const uint4*>(s_phi + (rt * 32 + m) * PHI_LD + phi_k +
                                                    16 * j);
    if constexpr (!LAST) { clear_tile(); step_next(); }
#pragma unroll
    for (int c = 0; c < ET; ++c) {
      if constexpr (!LAST) {
#pragma unroll
        for (int part = c * KSTEPS / ET; part < (c + 1) * KSTEPS / ET; ++part) produce(t + 1, part);
      }
      uint4(&cur)[NLD] = ld[c % R];
      if (tail) {  // wave-uniform: only the stages of a partly filled last block that reach entry d
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          // bytes of this 16-byte piece that lie before entry d (<= 0: none, >= 16: all)
          const int vb = tail_bytes - (lane % LPR) * 16;
          cur[i].x &= dword_mask(vb);
          cur[i].y &= dword_mask(vb - 4);
          cur[i].z &= dword_mask(vb - 8);
          cur[i].w &= dword_mask(vb - 12);
        }
      }
      uint4 g[NLD];  // operand pieces: k-step j is g[j*NV .. j*NV + NV)
#pragma unroll
      for (int i = 0; i < NLD; ++i) *reinterpret_cast<uint4*>(g_wr + i * RPI * GLD) = cur[i];
      // refill the slot with the tile R places further on: same stage, or the next one
      const int CN = (c + R) % ET;  // compile-time after unrolling
      const bool wrap = c + R >= ET;
      if (!(LAST && wrap)) issue_tile(wrap ? kb_n : kb_c, CN, cur);
#pragma unroll
      for (int i = 0; i < NLD; ++i)
        g[i] = *reinterpret_cast<const uint4*>(g_rd + (i / NV) * (16 * (int)sizeof(T)) + (i % NV) * 16);
      if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int j = 0; j < KSTEPS; ++j)
#pragma unroll
          for (int rt = 0; rt < MT; ++rt) acc[c][rt] = mfma<T>(g[j], pb[j][rt], acc[c][rt]);
      } else {
#pragma unroll
        for (int jj = 0; jj < KSTEPS; jj += 2) {
          uint4 pc[2][3];
#pragma unroll
          for (int cc = 0; cc < 2; ++cc) {
            const uint4 x0 = g[(jj + cc) * 2], x1 = g[(jj + cc) * 2 + 1];
            const uint32_t xs[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
            split_ops(xs, pc[cc][0], pc[cc][1], pc[cc][2]);
          }
#pragma unroll
          for (int piece = 0; piece < 3; ++piece)
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
              for (int rt = 0; rt < MT; ++rt)
                acc[c][rt] = mfma<T>(pc[cc][piece], pb[jj + cc][rt], acc[c][rt]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    kb_c = kb_n;
  };

  if (rows_valid > 0) {
#pragma unroll
    for (int c = 0; c < R; ++c) issue_tile(kb_c, c, ld[c]);
#pragma unroll
    for (int part = 0; part < KSTEPS; ++part) produce(0, part);
    for (int t = 0; t + 1 < T_stages; ++t) stage(t, std::false_type{});
    stage(T_stages - 1, std::true_type{});
  }

  // ---- epilogue: accumulator v of tile (c, rt) is example ex0 + 32 c + 8 (v/4) + 4 kg + v%4,
  // stacked row 32 rt + m.
  if constexpr (OUT) {  // the finished block: scale, convert, 32 consecutive columns per half-wave
    T* base = reinterpret_cast<T*>(a.out) + (int64_t)ex0 * a.ldo + (int64_t)blk * p.Br + row_lo + m;
#pragma unroll
    for (int c = 0; c < ET; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ex = c * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
        if (ex < rows_valid) {
#pragma unroll
          for (int rt = 0; rt < MT; ++rt) Elt<T>::store(base + (int64_t)ex * a.ldo + rt * 32, acc[c][rt][v] * p.scale);
        }
      }
    return;
  }
  // IN: the partial results are stored as [z][example][record][stacked row]: a wave's 32*MT
  // stacked rows of one example are contiguous, so every store instruction writes whole 128-byte
  // lines (stored by destination block they were 32-byte runs for Br = 8, and the stores cost
  // 15 % of the kernel).  The reduction gathers them by output block.
  // Records are ordered by the ORBIT POSITION of the input block when the orbit table exists:
  // the kappa records an output block needs are then adjacent (positions p+1 .. p+kappa of the
  // output's position p), and neighbouring outputs read neighbouring records.
  {
    const uint32_t rec = a.orbit ? __builtin_amdgcn_readfirstlane(a.orbit[p.M + blk]) : blk;
    float* base = a.ws + (((int64_t)blockIdx.z * a.n + ex0) * p.M + rec) * RWV + m;  // set (group, z)
    const int64_t ex_stride = (int64_t)p.M * RWV;
#pragma unroll
    for (int c = 0; c < ET; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ex = c * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
        if (ex < rows_valid) {
#pragma unroll
          for (int rt = 0; rt < MT; ++rt) base[ex * ex_stride + rt * 32] = acc[c][rt][v];
        }
      }
  }
}

// out[ex][g*Br + r] = scale * sum over slots l = 1..kappa (outer) and row splits z (inner) of
// part[z][ex][record of f^l(g)][(l-1)*Br + r]: fixed order, no atomics.  One thread per VEC output
// columns (VEC = 4 when 4 | Br, else 1).  With the orbit table (2M words: block at each orbit
// position of f from block 0, then the inverse) threads are numbered by the orbit position pos of
// their output block and the records are those at positions pos+1 .. pos+kappa: a sliding window
// of contiguous memory.  Without it records are indexed by block and f is evaluated directly.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void reduce_rows_kernel(const float* __restrict__ part, int zsplit, int n,
                                                          SketchParams p, uint32_t lbr, uint32_t rw,
                                                          uint32_t group_slots,
                                                          const uint32_t* __restrict__ orbit,
                                                          T* __restrict__ out, int64_t ldo) {
  const int64_t q = p.k / VEC;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)n * q) return;
  const int64_t ex = idx / q;
  const uint32_t col0 = (uint32_t)(idx % q) * VEC;
  // orbit position (or block) and row in block; lbr = log2 of the rows a slot takes in a record
  // (Br, or the next power of two when Br is not one)
  const uint32_t bi = p.br_pow2 ? col0 >> lbr : col0 / p.Br;
  const uint32_t r = p.br_pow2 ? col0 & (p.Br - 1) : col0 - bi * p.Br;
  const uint32_t g = orbit ? orbit[bi] : bi;
  const int64_t z_stride = (int64_t)n * p.M * rw;
  const float* src = part + ex * (int64_t)p.M * rw + r;
  float s[VEC];
#pragma unroll
  for (int c = 0; c < VEC; ++c) s[c] = 0.f;
  // The kappa * zsplit addends in the order (slot l, row split z), four at a time: their loads are
  // issued together, then added in that order.  (One load per pass of a loop made the kernel wait
  // for memory once per addend.)
  using Vec = std::conditional_t<VEC == 4, float4, float>;
  const uint32_t total = p.kappa * (uint32_t)zsplit;
  uint32_t rec = bi, l = 0, zc = 0, lg = 0, grp = 0;  // record of slot l; l = grp * group_slots + lg
  rec = orbit ? (rec + 1 == p.M ? 0u : rec + 1) : wire_next(rec, p.a, p.b, p.M);
  for (uint32_t t0 = 0; t0 < total; t0 += 4) {
    Vec v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // (past the last addend the cursor stays on it: the load is valid and ignored)
      const float* ph = src + ((int64_t)grp * zsplit + zc) * z_stride + (int64_t)rec * rw + (lg << lbr);
      v[j] = *reinterpret_cast<const Vec*>(ph);
      if (t0 + j + 1 < total) {
        if (++zc == (uint32_t)zsplit) {
          zc = 0;
          ++l;
          if (++lg == group_slots) { lg = 0; ++grp; }
          rec = orbit ? (rec + 1 == p.M ? 0u : rec + 1) : wire_next(rec, p.a, p.b, p.M);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (t0 + j < total) {
        if constexpr (VEC == 4) { s[0] += v[j].x; s[1] += v[j].y; s[2] += v[j].z; s[3] += v[j].w; }
        else s[0] += v[j];
      }
    }
  }
  (void)l;
  T* dst = out + ex * ldo + (int64_t)g * p.Br + r;
#pragma unroll
  for (int c = 0; c < VEC; ++c) s[c] *= p.scale;
  if constexpr (VEC == 4) {
    if ((uintptr_t)dst % (4 * sizeof(T)) == 0) {  // one 8- or 16-byte store
      if constexpr (sizeof(T) == 2) {
        const uint2 w = pack4<T>(s);
        *reinterpret_cast<uint2*>(dst) = w;
      } else {
        *reinterpret_cast<float4*>(dst) = make_float4(s[0], s[1], s[2], s[3]);
      }
      return;
    }
  }
#pragma unroll
  for (int c = 0; c < VEC; ++c) Elt<T>::store(dst + c, s[c]);
}

struct RowsPlan {
  bool ok = false;
  int mt = 0, et = 0, zsplit = 1, stages = 0, planes = 0, groups = 1, group_slots = 0;
  bool out_stat = false;
  int unal = 0;  // 0: 128-bit loads, 1: dword loads, 2: element loads (16-bit types)
  int nsub = 1;  // OUT: 128-row slices of an output block
  bool big = false;  // IN: one descriptor per 32-example tile (very long rows)
  size_t lds = 0;
};

RowsPlan make_rows_plan(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt) {
  RowsPlan pl;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  if (n < 1) return pl;
  const int64_t blk_stages = ((int64_t)p.Bc + KC - 1) / KC;  // the last one may be partly filled
  // Br not a power of two: input-stationary only, every slot padded to the next power of two
  uint32_t brp = 1;
  while (brp < p.Br) brp <<= 1;
  if (!p.br_pow2 && brp > 128) return pl;
  const uint64_t rw = (uint64_t)p.kappa * brp;
  // 32, 64, 128, or 128-row slices of a higher block (OUT tables all kappa neighbours: at most MAX_KAPPA)
  const bool br_tile = p.br_pow2 && p.Br >= 32 && p.kappa <= (uint32_t)MAX_KAPPA;
  const int out_mt = (int)(p.Br > 128 ? 128 : p.Br) / 32;
  const int out_nsub = p.Br > 128 ? (int)(p.Br / 128) : 1;
  if (p.kappa == 1 && br_tile) {  // nothing is re-read: output-stationary stores the result directly
    pl.out_stat = true;
    pl.mt = out_mt; pl.nsub = out_nsub;
    pl.et = 4;
  } else if (rw <= 32) { pl.mt = 1; pl.et = 4; }   // the smallest tile that holds the stacked rows
  else if (rw <= 64) { pl.mt = 2; pl.et = 4; }
  else if (rw <= 128) { pl.mt = 4; pl.et = 4; }
  else if (br_tile) {  // too many stacked rows: output-stationary
    pl.out_stat = true;
    pl.mt = out_mt; pl.nsub = out_nsub;
    pl.et = 4;
  } else if (brp <= 64) {  // ... and no OUT for them (small blocks, Br not a power of two, kappa > 128):
    pl.mt = 4; pl.et = 4;  // groups of 128/Br slots, G read once per group
    pl.group_slots = (int)(128 / brp);
    pl.groups = (int)((p.kappa + pl.group_slots - 1) / pl.group_slots);
  } else return pl;
  if ((uintptr_t)G % esz) return pl;
  // what every piece address G + example*ldg + block*Bc + 64*stage (in bytes) is a multiple of
  const int64_t bc_bytes = (int64_t)p.Bc * (int64_t)esz;
  if ((uintptr_t)G % 4 || (ldg * (int64_t)esz) % 4 || bc_bytes % 4) pl.unal = 2;         // element loads
  else if ((uintptr_t)G % 16 || (ldg * (int64_t)esz) % 16 || bc_bytes % 16) pl.unal = 1;  // four dwords each
  // 32-bit offsets: within the wave's 128 examples, or (input-stationary only) within a 32-example tile
  if (34 * ldg * (int64_t)esz >= ((int64_t)1 << 31)) return pl;
  pl.big = 130 * ldg * (int64_t)esz >= ((int64_t)1 << 31);
  if (pl.big && pl.out_stat) return pl;
  const int64_t ex_tiles = (n + 32 * pl.et - 1) / (32 * pl.et);
  if (ex_tiles * pl.nsub > 65535) return pl;
  // row split: the traffic model of the column layout (G at ~6 TB/s once 1024 waves exist,
  // planes written at ~3.4 TB/s and read back at ~6 TB/s)
  if (pl.group_slots == 0) pl.group_slots = (int)p.kappa;
  const double g_bytes = (double)p.d * (double)n * esz * pl.groups;
  double best = 0;
  for (int zc = 1; zc <= 16; zc *= 2) {
    if (zc > 1 && p.Bc % (uint32_t)(zc * KC) != 0) break;  // splits are whole stages
    const double waves = (double)p.M * ex_tiles * zc * pl.groups;
    const double plane_bytes = (double)zc * p.kappa * (double)p.k * (double)n * 4.0;
    const double t = g_bytes / (6e12 * (waves < 1024 ? waves / 1024 : 1.0)) + plane_bytes / 3.4e12 +
                     plane_bytes / 6e12;
    if (zc == 1 || t < best) { best = t; pl.zsplit = zc; }
  }
  if (pl.out_stat) pl.zsplit = 1;
  pl.stages = pl.out_stat ? (int)(p.kappa * blk_stages) : (int)(blk_stages / pl.zsplit);
  pl.planes = pl.out_stat ? 0 : pl.zsplit * (int)p.kappa;
  // slot tables, the Phi^T tile and the transposition tile
  pl.lds = 2 * MAX_KAPPA * 4 + (size_t)(32 * pl.mt) * PHI_LD * 2 + 32 * (KC * esz + 16);
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

bool rows_describe(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt, int* mode,
                   int* flags, size_t* workspace) {
  const RowsPlan pl = make_rows_plan(p, G, ldg, n, dt);
  if (!pl.ok) return false;
  *mode = pl.out_stat ? 1 : 2;
  *flags = (pl.unal ? FS_PLAN_ELEMENT_LOADS : 0) | (pl.nsub > 1 ? FS_PLAN_ROW_SLICES : 0) |
           (pl.groups > 1 ? FS_PLAN_SLOT_GROUPS : 0) | (pl.zsplit > 1 ? FS_PLAN_SPLIT : 0);
  *workspace = rows_workspace_bytes(p, G, ldg, n, dt);
  return true;
}

size_t rows_workspace_bytes(const SketchParams& p, const void* G, int64_t ldg, int64_t n, fs_dtype dt) {
  const RowsPlan pl = make_rows_plan(p, G, ldg, n, dt);
  if (!pl.ok) return 0;
  // [z][example][block][tile height]
  return pl.out_stat ? 0 : (size_t)pl.groups * (size_t)pl.zsplit * (size_t)n * (size_t)p.M * (size_t)(32 * pl.mt) *
                               sizeof(float);
}

hipError_t launch_rows(const SketchParams& p, const void* G, int64_t ldg, int64_t n, void* out,
                       int64_t ldo, fs_dtype dt, void* ws, const uint32_t* orbit, hipStream_t st,
                       EventPair ev) {
  const RowsPlan pl = make_rows_plan(p, G, ldg, n, dt);
  if (!pl.ok) return hipErrorInvalidValue;
  RowsArgs a;
  a.p = p; a.G = G; a.ws = (float*)ws; a.orbit = orbit; a.out = out;
  a.ldg = ldg; a.ldo = ldo; a.n = (int)n;
  a.stages = pl.stages;
  a.log2_br = 0;
  while ((1u << a.log2_br) < p.Br) ++a.log2_br;
  a.zsplit = pl.zsplit; a.group_slots = pl.group_slots; a.nsub = pl.nsub;
  const dim3 grid(p.M, (unsigned)((n + 32 * pl.et - 1) / (32 * pl.et)) * pl.nsub, pl.zsplit * pl.groups);

  if (ev.start) (void)hipEventRecord(ev.start, st);
  hipError_t e;
#define FS_ROWS_U(T, MT, ET, U)                                                   \
  (pl.out_stat ? go(rows_kernel<T, MT, ET, true, U>, grid, pl.lds, st, a)         \
   : pl.big    ? go(rows_kernel<T, MT, ET, false, U, true>, grid, pl.lds, st, a)  \
               : go(rows_kernel<T, MT, ET, false, U>, grid, pl.lds, st, a))
// (U2: what pl.unal == 2 selects -- element loads exist for the 16-bit types only; fp32 rows are
// always dword aligned)
#define FS_ROWS(T, MT, ET, U2) \
  (pl.unal == 0 ? FS_ROWS_U(T, MT, ET, 0) : pl.unal == 1 ? FS_ROWS_U(T, MT, ET, 1) : FS_ROWS_U(T, MT, ET, U2))
  if (dt == FS_BF16)
    e = pl.mt == 1 ? FS_ROWS(uint16_t, 1, 4, 2) : pl.mt == 2 ? FS_ROWS(uint16_t, 2, 4, 2) : FS_ROWS(uint16_t, 4, 4, 2);
  else if (dt == FS_F16)
    e = pl.mt == 1 ? FS_ROWS(f16, 1, 4, 2) : pl.mt == 2 ? FS_ROWS(f16, 2, 4, 2) : FS_ROWS(f16, 4, 4, 2);
  else
    e = pl.mt == 1 ? FS_ROWS(float, 1, 4, 1) : pl.mt == 2 ? FS_ROWS(float, 2, 4, 1) : FS_ROWS(float, 4, 4, 1);
#undef FS_ROWS
#undef FS_ROWS_U
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  if (e != hipSuccess || pl.out_stat) return e;
  const int vec = p.Br % 4 == 0 ? 4 : 1;
  const int64_t work = n * (p.k / vec);
  const dim3 rgrid((unsigned)((work + 255) / 256));
#define FS_RED(T, VEC)                                                                                   \
  hipLaunchKernelGGL((reduce_rows_kernel<T, VEC>), rgrid, dim3(256), 0, st, a.ws, pl.zsplit, (int)n, p, \
                     a.log2_br, (uint32_t)(32 * pl.mt), (uint32_t)pl.group_slots, orbit, (T*)out, ldo)
  if (dt == FS_BF16)     { if (vec == 4) FS_RED(uint16_t, 4); else FS_RED(uint16_t, 1); }
  else if (dt == FS_F16) { if (vec == 4) FS_RED(f16, 4); else FS_RED(f16, 1); }
  else                   { if (vec == 4) FS_RED(float, 4); else FS_RED(float, 1); }
#undef FS_RED
  return hipGetLastError();
}

}  // namespace fs
