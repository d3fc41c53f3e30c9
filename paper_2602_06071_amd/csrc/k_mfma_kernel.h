// The matrix-core kernels of k_mfma.hip and their launch table, as a header: one translation
// unit per element type includes it (k_mfma_f32.hip, k_mfma_bf16.hip, k_mfma_f16.hip) so that
// the three sets of instantiations compile side by side.
#pragma once
#include <type_traits>

#include "handle.h"
#include "mfma_common.h"
#include "spec.h"

namespace fs {
namespace mm {


struct MfmaArgs {
  SketchParams p;
  const void* A;
  void* out;
  float* ws;
  const uint32_t* pos2blk;  // orbit order of the blocks (RUN > 1 only)
  int64_t lda, ldo, ldw;
  int n;
  int zsplit;       // IN: row splits of an input block; OUT: splits of the kappa*Bc rows
  int group_slots;  // IN: wiring slots one work-group stacks (grid.z = zsplit * slot groups)
  int nsub;         // OUT, Br > 128: 128-row slices of an output block (grid.y = column tiles * nsub)
  int stages;       // stages per work-group
  int out_vec;      // out rows allow 4-column vector stores
  uint32_t log2_br;
};

// What the host decided for one launch (make_plan in k_mfma.hip).
struct Plan {
  bool ok = false;
  bool in_stat = false;
  int mt = 0, nrg = 0, ncg = 0, zsplit = 1, stages = 0, run = 1, cpl = 4, pfx = 1;
  int groups = 1, group_slots = 0;  // IN: slot groups (A is read once per group)
  int nsub = 1;                     // OUT: 128-row slices of an output block
  bool unal = false;                // A or lda not aligned to 4 columns: element-wise loads
  bool stacked = false;             // several output blocks per wave: the kernel of k_stacked.hip
  bool outs = false;                // OUT, 16-bit: the kernel of k_outs.hip (work-group-shared Phi tiles)
  int64_t ldw = 0;
  int planes = 0;
  size_t lds = 0;
};

}  // namespace mm

namespace {

using namespace mm;

// PFX multiplies the depth of the register prefetch ring (1 or 2).  A ring deeper than one
// stage (bf16, PFX = 2: 8 k-steps) needs an even number of stages, which the host checks.
// SUB (OUT, Br > 128): a work-group owns one 128-row slice of its output block; it walks the same
// input blocks and keeps only the nonzeros that fall into its slice.
// UNAL: A or lda is not a multiple of 4 columns, so a lane's 4 columns are not one aligned
// vector: they are loaded element by element (same registers afterwards, four times the load
// instructions).
template <typename T, int MT, int NRG, int NCG, bool IN_STAT, int RUN, int CPL, int PFX = 1, bool SUB = false,
          bool UNAL = false>
__global__ __launch_bounds__(64 * NRG * NCG * RUN) __attribute__((amdgpu_waves_per_eu(MT > 2 ? 1 : 2)))
void mfma_kernel(MfmaArgs a) {
  using V = typename LdN<T, CPL>::V;
  // (element loads hold four registers per row until they are packed: half the ring)
  constexpr int PFD = UNAL ? 2 : LdN<T, CPL>::PFD * PFX;
  static_assert(PFD <= KSTEPS || PFD == 2 * KSTEPS, "ring depth: within a stage, or exactly two stages");
  constexpr int WC = 32 * CPL;                 // columns per wave
  constexpr int NW = NRG * NCG, NT = 64 * NW;  // waves / threads of one sub-group
  constexpr int RWV = 32 * MT;                 // stacked Phi rows of one wave
  constexpr int TILE = RWV * PHI_LD;           // bf16 elements of one Phi tile
  static_assert(RUN == 1 || IN_STAT, "orbit runs are an IN-stationary mode");
  static_assert(!SUB || (!IN_STAT && NRG == 1), "row slices are an OUT-stationary mode");

  // dynamic LDS: per sub-group [MAX_KAPPA] keys and blocks, then per wave two Phi tiles
  // [RWV][PHI_LD] bf16 (consume / refill: a wave makes exactly the rows it consumes, so the
  // steady state needs no barrier).  The tile region is reused as the merge buffer of the
  // RUN > 1 epilogue.
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const SketchParams& p = a.p;
  const int sg = RUN > 1 ? (int)threadIdx.x / NT : 0;  // sub-group: one input block each
  const int tid = RUN > 1 ? (int)threadIdx.x % NT : (int)threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  constexpr size_t kTabBytes = (size_t)RUN * 2 * MAX_KAPPA * 4;
  uint32_t* s_bk = reinterpret_cast<uint32_t*>(smem) + sg * 2 * MAX_KAPPA;  // block keys per slot
  uint32_t* s_blk = s_bk + MAX_KAPPA;    // IN: destination block g_l;  OUT: source block h_l
  uint16_t* s_phi = reinterpret_cast<uint16_t*>(smem + kTabBytes) + (size_t)(sg * NW + wave) * 2 * TILE;

  const int rg = wave / NCG, cg = wave % NCG;
  const int kg = lane >> 5;
  // Which (block, column tile) this work-group takes.  OUT with an orbit table: work-groups
  // are renumbered so that the ones an XCD runs side by side (the hardware deals linear ids
  // round-robin over the 8 XCDs) are consecutive orbit positions of one column tile; together
  // with the phase order below they then read the same input block at the same time, and the
  // kappa re-reads of A are served by that XCD's L2 instead of the fabric.
  uint32_t bx = blockIdx.x, jt = blockIdx.y, opos = 0;
  const bool remap = !IN_STAT && a.pos2blk != nullptr;
  if (remap) {
    const uint32_t total = gridDim.x * gridDim.y;
    uint32_t id = blockIdx.y * gridDim.x + blockIdx.x;
    if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
    opos = id % gridDim.x;
    jt = id / gridDim.x;
  }
  uint32_t slice = 0;
  if constexpr (SUB) {
    slice = jt % (uint32_t)a.nsub;
    jt /= (uint32_t)a.nsub;
  }
  const int col0 = (int)jt * (WC * NCG) + cg * WC + CPL * (lane & 31);
  // IN: input block h (RUN > 1: the block at orbit position blockIdx.x*RUN + sg); OUT: g
  uint32_t blk = bx;
  if (RUN > 1) blk = __builtin_amdgcn_readfirstlane(a.pos2blk[blockIdx.x * RUN + sg]);
  if (remap) blk = __builtin_amdgcn_readfirstlane(a.pos2blk[opos]);
  // IN with kappa*Br above the tile height: grid.z also numbers groups of `group_slots` wiring
  // slots; a work-group then serves the slots [slot0, slot0 + kap) and A is read once per group
  const int z = (int)(blockIdx.z % (uint32_t)a.zsplit);
  const uint32_t slot0 = IN_STAT ? (blockIdx.z / (uint32_t)a.zsplit) * (uint32_t)a.group_slots : 0u;
  const uint32_t kap = IN_STAT ? min(p.kappa - slot0, (uint32_t)a.group_slots) : p.kappa;
  const int T_stages = a.stages;
  // stages per input block (OUT).  Bc need not be a multiple of the stage: the rows of the last
  // stage at or beyond Bc lie outside the block's buffer range and read as 0.
  const uint32_t rows_per_blk_stage = (p.Bc + KC - 1) / KC;
  const uint32_t lbr = a.log2_br;

  // ---- slot tables and empty tiles ------------------------------------------------
  auto clear_tile = [&](int buf) {
    uint4* z4 = reinterpret_cast<uint4*>(s_phi + buf * TILE);
#pragma unroll
    for (int i = 0; i < (TILE / 8 + 63) / 64; ++i)
      if (TILE / 8 % 64 == 0 || lane + i * 64 < TILE / 8) z4[lane + i * 64] = make_uint4(0, 0, 0, 0);
  };
  auto setup_tables = [&]() {
    for (int sl = tid; sl < (int)kap; sl += NT) {
      uint32_t x = blk;
      if (remap) {
        // phase sl handles the neighbour whose (unwrapped) orbit position is sl mod kappa:
        // every work-group of a column tile is then on the same input block in the same phase
        const uint32_t l = (sl + p.kappa - (opos + 1) % p.kappa) % p.kappa;  // 0 .. kappa-1
        x = a.pos2blk[(opos + 1 + l) % p.M];
      } else {
        for (int l = 0; l <= (int)slot0 + sl; ++l)
          x = IN_STAT ? wire_prev(x, p.a_inv, p.b, p.M) : wire_next(x, p.a, p.b, p.M);
      }
      s_blk[sl] = x;
      s_bk[sl] = IN_STAT ? block_key(p.key1, x, blk, p.M) : block_key(p.key1, blk, x, p.M);
    }
    clear_tile(0);
    clear_tile(1);
    __syncthreads();
  };

  const char* Abase = reinterpret_cast<const char*>(a.A);
  // per-lane byte offset of its first row inside a 16-row k-step (fits 32 bits: checked on
  // the host); the other 7 rows are reached through the scalar base
  // (a lane whose columns all lie at or beyond n gets an offset outside every descriptor range
  // instead, 2^31: its loads return 0 and move no data)
  const uint32_t voff = col0 < a.n ? (uint32_t)(((int64_t)(kg * 8) * a.lda + col0) * (int64_t)sizeof(T))
                                   : 0x80000000u;
  const int64_t row_bytes = a.lda * (int64_t)sizeof(T);

  f32x16 acc[MT][CPL];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][c][i] = 0.f;

  // Scatter into tile `buf` the nonzeros of stage t that fall in this wave's stacked rows
  // [row_lo, row_lo + RWV): one lane per row of the stage, the wave's slots in turn.  Part
  // `part` (of KSTEPS) takes every KSTEPS-th slot so the hashing spreads over the stage.
  const uint32_t row_lo = SUB ? slice * RWV : (uint32_t)rg * RWV;
  // `whole`: the slot lies entirely inside this wave's rows, so no nonzero is filtered out.
  auto scatter = [&](uint16_t* phi, uint32_t key, uint32_t u, uint32_t slot_row0, bool whole) {
    if (!p.br_pow2) {
      // (wave-uniform; IN only) Br not a power of two: a slot takes 2^log2_br >= Br tile rows, of
      // which the first Br are used; the general row hash, and the wrap as a compare
      const RowHash rg_ = row_hash_any(key, u, p.Br);
      uint32_t rr = rg_.shift;
      for (uint32_t i = 0; i < p.s; ++i) {
        phi[__umul24(slot_row0 - row_lo + rr, (uint32_t)PHI_LD) + lane] =
            (uint16_t)(((rg_.signs >> i) << 15) | Fmt<T>::one);
        rr += rg_.stride;
        if (rr >= p.Br) rr -= p.Br;
      }
      return;
    }
    const RowHash rh = row_hash_pow2(key, u, p.Br);
    uint32_t r = rh.shift;
    // tile index of (row, lane) = row*72 + lane (24-bit multiply-add); the stored half-word is
    // +-1.0 in bf16: 0x3F80 with sign bit i of the hash word moved to bit 15 (bits above 15 of
    // the 32-bit value are dropped by the 16-bit store)
    const uint32_t base = slot_row0 - row_lo;
    auto put = [&](uint32_t local, uint32_t i) {
      phi[__umul24(local, (uint32_t)PHI_LD) + lane] = (uint16_t)(((rh.signs >> i) << 15) | Fmt<T>::one);
    };
    if (whole) {
      // s >= 1; the first two updates are peeled (s = 2 and 4 are the common cases)
      put(base + r, 0);
      if (p.s >= 2) {
        r = (r + rh.stride) & (p.Br - 1);
        put(base + r, 1);
        for (uint32_t i = 2; i < p.s; ++i) {
          r = (r + rh.stride) & (p.Br - 1);
          put(base + r, i);
        }
      }
    } else {
      for (uint32_t i = 0; i < p.s; ++i) {
        const uint32_t local = base + r;  // unsigned: rows below row_lo wrap high
        if (local < (uint32_t)RWV) put(local, i);
        r = (r + rh.stride) & (p.Br - 1);
      }
    }
  };
  auto produce = [&](int t, int buf, int part) {
    uint16_t* phi = s_phi + buf * TILE;
    if (IN_STAT) {
      const uint32_t u = (uint32_t)(z * T_stages + t) * KC + lane;
      const uint32_t slot_lo = row_lo >> lbr;
      const uint32_t slot_hi = min(kap, ((row_lo + RWV - 1) >> lbr) + 1);
      const bool whole = p.Br <= (uint32_t)RWV;  // power-of-two Br: slots tile the wave's rows
      for (uint32_t slot = slot_lo + part; slot < slot_hi; slot += KSTEPS)
        scatter(phi, s_bk[slot], u, slot << lbr, whole);
    } else if (part == 0) {
      const uint32_t tg = (uint32_t)(z * T_stages + t);  // stage among all kappa blocks
      const uint32_t l = tg / rows_per_blk_stage;
      const uint32_t u = (tg % rows_per_blk_stage) * KC + lane;
      scatter(phi, s_bk[l], u, 0u, p.Br <= (uint32_t)RWV);
    }
  };

  // The main loop, once for full column tiles and once for the ragged last tile (the same
  // vector loads, masked at the point of use); the choice is uniform per work-group.
  auto body = [&](auto ragged_tag) {
    constexpr bool RAGGED = decltype(ragged_tag)::value;
    V ld[PFD][8];
    // Buffer descriptor over the rows this work-group reads from one input block
    // (dword 3 = 32-bit data format for gfx9-family raw buffers).  The scalar offset
    // walks the rows, the lane offset (voff) selects row-in-k-step and column.
    // Rows at or beyond d (the zero padding of a partly filled last input block) lie outside
    // the descriptor's range, and out-of-range buffer loads return 0 without touching memory.
    // The range ends with the last valid row's columns, rounded up to the 4-column vector: in the
    // ragged tile a lane's vector may straddle column n; what it reads beyond n (the row's own
    // padding, inside the same aligned 8/16-byte granule as a valid element) is masked to zero.
    auto make_rsrc = [&](int64_t first_row, int64_t nrows) {
      const int64_t valid = min(nrows, p.d - first_row);
      // (element loads, UNAL, never reach past column n-1 of the last valid row)
      const int64_t ncols = UNAL ? (int64_t)a.n : ((int64_t)a.n + 3) & ~(int64_t)3;
      const int64_t bytes = valid > 0 ? (valid - 1) * row_bytes + ncols * (int64_t)sizeof(T) : 0;
      return __builtin_amdgcn_make_buffer_rsrc(
          const_cast<char*>(Abase + first_row * row_bytes), 0, (int)bytes, 0x00020000);
    };
    // Fetch cursor.  k-steps are issued strictly in order, so the OUT mode
    // keeps (descriptor of the current input block, byte offset, k-step within the block) in
    // scalar registers and only rebuilds the descriptor when it crosses into the next block.
    __amdgpu_buffer_rsrc_t f_rs = make_rsrc(0, 0);
    uint32_t f_so = 0, f_kr = 0, f_l = 0;
    const uint32_t per_blk_k = rows_per_blk_stage * KSTEPS;
    auto cursor_init = [&]() {
      if (IN_STAT) {
        const int64_t row0 = (int64_t)z * T_stages * KC;  // the range ends with the block's last row
        f_rs = make_rsrc((int64_t)blk * p.Bc + row0, min((int64_t)T_stages * KC, (int64_t)p.Bc - row0));
      } else {
        const uint32_t kg0 = (uint32_t)(z * T_stages * KSTEPS);
        f_l = kg0 / per_blk_k;
        f_kr = kg0 % per_blk_k;
        const uint32_t hb = __builtin_amdgcn_readfirstlane(s_blk[f_l]);
        f_rs = make_rsrc((int64_t)hb * p.Bc, p.Bc);
        f_so = f_kr * 16u * (uint32_t)row_bytes;
      }
    };
    // OUT mode, after every issue: step the cursor (wave-uniform; the branch is taken once per
    // input block).  Kept apart from issue() so that it can sit at the end of a k-step and the
    // k-step stays one basic block.
    auto advance = [&]() {
      if constexpr (!IN_STAT) {
        f_so += 16u * (uint32_t)row_bytes;
        if (++f_kr == per_blk_k) {
          f_kr = 0;
          f_so = 0;
          if (++f_l < p.kappa) {
            const uint32_t hb = __builtin_amdgcn_readfirstlane(s_blk[f_l]);
            f_rs = make_rsrc((int64_t)hb * p.Bc, p.Bc);
          }
        }
      }
    };
    auto issue = [&](int kk, V (&dst)[8]) {
      const __amdgpu_buffer_rsrc_t rs = f_rs;
      const uint32_t so = IN_STAT ? (uint32_t)kk * 16u * (uint32_t)row_bytes : f_so;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t soj = so + (uint32_t)j * (uint32_t)row_bytes;
        if constexpr (UNAL && sizeof(V) == 8) {
          // (written as 16-bit vector inserts so that the halves of a register are loaded in
          // place, without a packing step)
          typedef unsigned short us4 __attribute__((ext_vector_type(4)));
          us4 e;
          e.x = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, voff, soj, 0);
          e.y = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, voff + 2u, soj, 0);
          e.z = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, voff + 4u, soj, 0);
          e.w = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, voff + 6u, soj, 0);
          dst[j] = __builtin_bit_cast(V, e);
        } else if constexpr (UNAL) {
          uint32_t* e = reinterpret_cast<uint32_t*>(&dst[j]);
#pragma unroll
          for (int c = 0; c < 4; ++c)
            e[c] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, voff + 4u * c, soj, 0);
        } else if constexpr (sizeof(V) == 8)
          dst[j] = __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soj, 0));
        else
          dst[j] = __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soj, 0));
      }
    };
    // Ragged tile: zero, at the point of use, the columns at or beyond n of what a lane loaded.
    V cmask;
    {
      const int vc = a.n - col0;  // valid columns of this lane's vector (may be <= 0 or >= 4)
      if constexpr (sizeof(V) == 8) {
        cmask.x = vc >= 2 ? 0xFFFFFFFFu : vc == 1 ? 0x0000FFFFu : 0u;
        cmask.y = vc >= 4 ? 0xFFFFFFFFu : vc == 3 ? 0x0000FFFFu : 0u;
      } else {
        cmask.x = vc >= 1 ? 0xFFFFFFFFu : 0u;
        cmask.y = vc >= 2 ? 0xFFFFFFFFu : 0u;
        cmask.z = vc >= 3 ? 0xFFFFFFFFu : 0u;
        cmask.w = vc >= 4 ? 0xFFFFFFFFu : 0u;
      }
    }
    auto mask_cur = [&](V (&cur)[8]) {
      if constexpr (RAGGED) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          cur[j].x &= cmask.x;
          cur[j].y &= cmask.y;
          if constexpr (sizeof(V) == 16) {
            cur[j].z &= cmask.z;
            cur[j].w &= cmask.w;
          }
        }
      }
    };

    // One stage: 4 MFMA k-steps on tile t%2 while a later stage is loaded and the next one is
    // hashed into the other tile.  FETCH (compile time): 2 = every k-step issues the loads PFD
    // k-steps ahead, 1 = only those that stay inside this stage, 0 = none; FILL: whether a next
    // stage exists.  The steady-state loop body thus has no conditional memory operations.
    // PAR is the stage's parity when the ring spans two stages (it makes the ring slot static).
    auto stage = [&](int t, auto par_tag, auto fetch_tag, auto fill_tag) {
      constexpr int PAR = decltype(par_tag)::value;
      constexpr int FETCH = decltype(fetch_tag)::value;
      constexpr bool LAST = !decltype(fill_tag)::value;
      const uint16_t* phi = s_phi + (t & 1) * TILE;
      const int fill_buf = (t + 1) & 1;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        uint4 pa[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          pa[mt] = *reinterpret_cast<const uint4*>(
              phi + (mt * 32 + (lane & 31)) * PHI_LD + ks * 16 + kg * 8);
        if constexpr (!LAST) produce(t + 1, fill_buf, ks);

        V(&cur)[8] = ld[(PAR * KSTEPS + ks) % PFD];
        const bool fetch = FETCH == 2 || (FETCH == 1 && ks + PFD < KSTEPS);  // compile-time
        mask_cur(cur);
        if constexpr (sizeof(T) == 2) {
          uint4 op[4];
          make_ops(cur, op);
          if (fetch) issue(t * KSTEPS + ks + PFD, cur);
#pragma unroll
          for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[mt], op[c], acc[mt][c]);
        } else {
          // two columns at a time, piece by piece: an accumulator is reused only after
          // 2*MT other MFMAs (back-to-back dependent MFMAs stall the matrix pipe)
#pragma unroll
          for (int c = 0; c < 4; c += 2) {
            uint4 pc[2][3];
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
              uint32_t xs[8];
#pragma unroll
              for (int j = 0; j < 8; ++j)
                xs[j] = c + cc == 0 ? cur[j].x : c + cc == 1 ? cur[j].y : c + cc == 2 ? cur[j].z : cur[j].w;
              split_ops(xs, pc[cc][0], pc[cc][1], pc[cc][2]);
            }
#pragma unroll
            for (int piece = 0; piece < 3; ++piece)
#pragma unroll
              for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                  acc[mt][c + cc] = mfma<T>(pa[mt], pc[cc][piece], acc[mt][c + cc]);
          }
          if (fetch) issue(t * KSTEPS + ks + PFD, cur);
        }
        if (fetch) advance();
        __builtin_amdgcn_sched_barrier(0);  // keep k-steps apart: bounds register pressure
      }
      // the tile just consumed becomes the fill target of the next stage
      if constexpr (!LAST) clear_tile(t & 1);
    };

    // OUT mode runs a software-pipelined variant of the stage, written as straight-line code so
    // that the scheduler can place the non-MFMA work between the MFMAs (with one wave per SIMD
    // nothing else would hide it):
    //  * the Phi operands of k-step ks+1 are read from LDS during k-step ks (two register sets);
    //  * the s nonzeros of a row of the next stage are written two per k-step, without a loop:
    //    updates beyond s go to a pad column of the tile that no MFMA reads (only s > 8 needs a
    //    loop, after the MFMAs of the last k-step);
    //  * the tile being consumed is cleared in 16-column slices, slice ks during k-step ks (its
    //    reads were issued one k-step earlier and LDS operations of a wave complete in order).
    uint4 pa2[2][MT];
    RowHash prh{0u, 0u, 0u};
    uint32_t pr = 0;
    const uint32_t pad_at = (uint32_t)((lane & 31) * PHI_LD + KC + (lane >> 5));
    auto read_pa = [&](const uint16_t* tile, int ks, uint4 (&dst)[MT]) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        dst[mt] = *reinterpret_cast<const uint4*>(tile + (mt * 32 + (lane & 31)) * PHI_LD + ks * 16 + kg * 8);
    };
    auto put_one = [&](uint16_t* tile, uint32_t i, bool real) {
      const uint32_t local = SUB ? pr - row_lo : pr;  // unsigned: rows below the slice wrap high
      const bool keep = SUB ? real && local < (uint32_t)RWV : real;
      tile[keep ? __umul24(local, (uint32_t)PHI_LD) + lane : pad_at] = (uint16_t)(((prh.signs >> i) << 15) | Fmt<T>::one);
      pr = (pr + prh.stride) & (p.Br - 1);
    };
    auto fill_part = [&](int t1, uint16_t* tile, int ks) {
      if (ks == 0) {
        const uint32_t tg = (uint32_t)(z * T_stages + t1);  // stage among all kappa blocks
        const uint32_t l = tg / rows_per_blk_stage;
        prh = row_hash_pow2(s_bk[l], (tg % rows_per_blk_stage) * KC + lane, p.Br);
        pr = prh.shift;
      }
      put_one(tile, 2u * ks, 2u * ks < p.s);
      put_one(tile, 2u * ks + 1u, 2u * ks + 1u < p.s);
    };
    auto clear_slice = [&](uint16_t* tile, int ks) {
#pragma unroll
      for (int i = 0; i < MT; ++i) {  // RWV rows x 32 bytes = 2*RWV 16-byte units
        const int unit = lane + 64 * i;
        *reinterpret_cast<uint4*>(tile + (unit >> 1) * PHI_LD + ks * 16 + (unit & 1) * 8) = make_uint4(0, 0, 0, 0);
      }
    };
    auto stage_out = [&](int t, auto par_tag, auto fetch_tag, auto fill_tag) {
      constexpr int PAR = decltype(par_tag)::value;
      constexpr int FETCH = decltype(fetch_tag)::value;
      constexpr bool FILL = decltype(fill_tag)::value;
      uint16_t* cur_tile = s_phi + (t & 1) * TILE;
      uint16_t* fill_tile = s_phi + ((t + 1) & 1) * TILE;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        V(&cur)[8] = ld[(PAR * KSTEPS + ks) % PFD];
        const bool fetch = FETCH == 2 || (FETCH == 1 && ks + PFD < KSTEPS);  // compile-time
        mask_cur(cur);
        uint4(&pa)[MT] = pa2[ks & 1];
        uint4(&pn)[MT] = pa2[(ks + 1) & 1];
        if constexpr (FILL) {
          fill_part(t + 1, fill_tile, ks);
          clear_slice(cur_tile, ks);
        }
        if (ks + 1 < KSTEPS) read_pa(cur_tile, ks + 1, pn);
        else if constexpr (FILL) read_pa(fill_tile, 0, pn);
        if constexpr (sizeof(T) == 2) {
          uint4 op[4];
          make_ops(cur, op);
          if (fetch) issue(t * KSTEPS + ks + PFD, cur);
#pragma unroll
          for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][c] = mfma<T>(pa[mt], op[c], acc[mt][c]);
          if constexpr (MT == 4) {  // one wave per SIMD: spread the rest between the MFMAs
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
#pragma unroll
            for (int i = 0; i < 4 * MT; ++i) {
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
              __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
              __builtin_amdgcn_sched_group_barrier(0x090, 2, 0);
            }
          }
        } else {
          // two columns at a time, piece by piece: an accumulator is reused only after
          // 2*MT other MFMAs (back-to-back dependent MFMAs stall the matrix pipe)
#pragma unroll
          for (int c = 0; c < 4; c += 2) {
            uint4 pc[2][3];
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
              uint32_t xs[8];
#pragma unroll
              for (int j = 0; j < 8; ++j)
                xs[j] = c + cc == 0 ? cur[j].x : c + cc == 1 ? cur[j].y : c + cc == 2 ? cur[j].z : cur[j].w;
              split_ops(xs, pc[cc][0], pc[cc][1], pc[cc][2]);
            }
#pragma unroll
            for (int piece = 0; piece < 3; ++piece)
#pragma unroll
              for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                  acc[mt][c + cc] = mfma<T>(pa[mt], pc[cc][piece], acc[mt][c + cc]);
          }
          if (fetch) issue(t * KSTEPS + ks + PFD, cur);
        }
        if (fetch) advance();
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (FILL) {
        if (p.s > 2u * KSTEPS) {  // rare: the remaining nonzeros, then re-read the first operands
          for (uint32_t i = 2u * KSTEPS; i < p.s; ++i) put_one(fill_tile, i, true);
          read_pa(fill_tile, 0, pa2[0]);
        }
      }
    };

    // (the barrier inside setup_tables waits for outstanding loads, so none are issued before it)
    setup_tables();
    if constexpr (RAGGED) {
      // a wave whose 128 columns all lie at or beyond n has nothing to add (its accumulators
      // stay zero and the epilogue stores nothing); it only had to take part in the barrier
      if ((int)jt * (WC * NCG) + cg * WC >= a.n) return;
    }
    cursor_init();
#pragma unroll
    for (int i = 0; i < PFD; ++i) { issue(i, ld[i]); advance(); }
#pragma unroll
    for (int part = 0; part < KSTEPS; ++part) produce(0, 0, part);
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    // (fp32 with two waves per SIMD has no registers to spare for the second operand set)
    constexpr bool PIPE = !IN_STAT && (sizeof(T) == 2 || MT == 4);
    auto run_stage = [&](int t, auto par_tag, auto fetch_tag, auto fill_tag) {
      if constexpr (PIPE) stage_out(t, par_tag, fetch_tag, fill_tag);
      else stage(t, par_tag, fetch_tag, fill_tag);
    };
    if constexpr (PIPE) read_pa(s_phi, 0, pa2[0]);
    if constexpr (PFD <= KSTEPS) {
      for (int t = 0; t + 1 < T_stages; ++t) run_stage(t, I0{}, I2{}, std::true_type{});
      run_stage(T_stages - 1, I0{}, I1{}, std::false_type{});
    } else {  // T_stages is even: the last two stages find all their loads already in flight
      for (int t = 0; t + 2 < T_stages; t += 2) {
        run_stage(t, I0{}, I2{}, std::true_type{});
        run_stage(t + 1, I1{}, I2{}, std::true_type{});
      }
      run_stage(T_stages - 2, I0{}, I0{}, std::true_type{});
      run_stage(T_stages - 1, I1{}, I0{}, std::false_type{});
    }
  };
  const bool full_tile = ((int)jt + 1) * (WC * NCG) <= a.n;
  if (full_tile) body(std::false_type{}); else body(std::true_type{});

  // ---- epilogue ------------------------------------------------------------
  // accumulator register i of tile (mt, c) holds stacked row (rg*MT+mt)*32 + 8*(i/4) + 4*kg + i%4
  // of column col0 + c; columns are handled four at a time (q).
  if constexpr (RUN > 1) {
    // Merge in LDS the tiles of the RUN sub-groups that go to the same output block:
    // sub-group j, slot l-1 lands on relative output position idx = j - l + kappa
    // (0 .. kappa+RUN-2).  Sub-groups take turns in index order, so the sum order is fixed.
    constexpr int TNW = WC * NCG;
    float* mbuf = reinterpret_cast<float*>(smem + kTabBytes);  // [kappa+RUN-1][Br][TNW]
    const int colw = cg * WC + CPL * (lane & 31);
    __syncthreads();  // every wave is done with the Phi tiles
    for (int j = 0; j < RUN; ++j) {
      if (sg == j) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
          for (int ib = 0; ib < 16; ib += 4) {  // four rows at a time: reads first, then adds
            float4* d[4];
            bool first[4];
            float4 o[4][CPL / 4];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
              const int i = ib + ii;
              const uint32_t row_s = (uint32_t)((rg * MT + mt) * 32 + 8 * (i >> 2) + 4 * kg + (i & 3));
              const uint32_t slot = row_s >> lbr, r = row_s & (p.Br - 1);
              const uint32_t idx = (uint32_t)j + p.kappa - 1u - slot;
              first[ii] = slot == 0 || j == 0;  // no earlier sub-group reaches this tile
              d[ii] = reinterpret_cast<float4*>(mbuf + ((size_t)((idx << lbr) + r)) * TNW + colw);
              if (j > 0) {
#pragma unroll
                for (int q = 0; q < CPL / 4; ++q) o[ii][q] = d[ii][q];
              }
            }
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
              const int i = ib + ii;
#pragma unroll
              for (int q = 0; q < CPL / 4; ++q) {
                float4 v = make_float4(acc[mt][4 * q][i], acc[mt][4 * q + 1][i], acc[mt][4 * q + 2][i],
                                       acc[mt][4 * q + 3][i]);
                if (j > 0 && !first[ii]) {
                  v.x += o[ii][q].x; v.y += o[ii][q].y; v.z += o[ii][q].z; v.w += o[ii][q].w;
                }
                d[ii][q] = v;
              }
            }
          }
        }
      }
      __syncthreads();
    }
    // cooperative store of the kappa+RUN-1 merged tiles to their partial planes; the
    // destination block of tile idx is slot j+kappa-1-idx of any sub-group j that feeds it
    static_assert(TNW / 4 == 64, "index split below assumes 64 float4 per tile row");
    const uint32_t total = (p.kappa + RUN - 1) << (lbr + 6);
    const uint32_t* blk_tab = reinterpret_cast<const uint32_t*>(smem);
    for (uint32_t e = threadIdx.x; e < total; e += NT * RUN) {
      const uint32_t idx = e >> (lbr + 6), r = (e >> 6) & (p.Br - 1), c4 = e & 63u;
      const int col = (int)blockIdx.y * TNW + (int)c4 * 4;
      if (col >= a.n) continue;
      const uint32_t j = min(idx, (uint32_t)(RUN - 1));
      const uint32_t g = blk_tab[j * 2 * MAX_KAPPA + MAX_KAPPA + (j + p.kappa - 1 - idx)];
      const int64_t plane = idx / RUN;
      float* dst = a.ws + (plane * p.k + ((int64_t)g << lbr) + r) * a.ldw + col;
      *reinterpret_cast<float4*>(dst) =
          *reinterpret_cast<const float4*>(mbuf + ((size_t)((idx << lbr) + r)) * TNW + c4 * 4);
    }
    return;
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t row_s = (uint32_t)((rg * MT + mt) * 32 + 8 * (i >> 2) + 4 * kg + (i & 3));
#pragma unroll
      for (int q = 0; q < CPL / 4; ++q) {
        const int colq = col0 + 4 * q;
        if (colq >= a.n) continue;
        float v[4] = {acc[mt][4 * q][i], acc[mt][4 * q + 1][i], acc[mt][4 * q + 2][i], acc[mt][4 * q + 3][i]};
        if (IN_STAT) {
          const uint32_t slot = row_s >> lbr, r = row_s & ((1u << lbr) - 1u);
          if (slot >= kap || r >= p.Br) continue;  // idle rows: above the stacked slots, or above Br in a slot
          const int64_t plane = (int64_t)z * p.kappa + slot0 + slot;
          float* dst = a.ws + (plane * p.k + (int64_t)s_blk[slot] * p.Br + r) * a.ldw + colq;
          *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        } else if (a.zsplit > 1) {  // OUT with split rows: plane z, summed by the reduce kernel
          float* dst = a.ws + ((int64_t)z * p.k + (int64_t)blk * p.Br + (SUB ? row_lo : 0u) + row_s) * a.ldw + colq;
          *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
          T* dst = reinterpret_cast<T*>(a.out) + ((int64_t)blk * p.Br + (SUB ? row_lo : 0u) + row_s) * a.ldo + colq;
#pragma unroll
          for (int c = 0; c < 4; ++c) v[c] *= p.scale;
          if (a.out_vec && colq + 3 < a.n) {
            if constexpr (sizeof(T) == 2) {
              const uint2 w = pack4<T>(v);
              *reinterpret_cast<uint2*>(dst) = w;
            } else {
              *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            }
          } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
              if (colq + c < a.n) Elt<T>::store(dst + c, v[c]);
          }
        }
      }
    }
  }
}

// out[row][col] = scale * sum_p ws[p][row][col], planes added in index order.
// RUN > 1: plane c of the output block at orbit position pos holds a tile only when
// delta = c*RUN + (pos%RUN + kappa)%RUN - kappa <= RUN-2 (the writer's relative position).
template <typename T>
__global__ __launch_bounds__(256) void reduce_planes_kernel(const float* __restrict__ ws, int planes,
                                                            int64_t k, int64_t ldw, int n,
                                                            T* __restrict__ out, int64_t ldo,
                                                            float scale, int out_vec, int run,
                                                            const uint32_t* __restrict__ blk2pos,
                                                            uint32_t Br, uint32_t kappa) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // over k * ldw/4
  const int64_t q = ldw / 4;
  if (idx >= k * q) return;
  const int64_t row = idx / q;
  const int col0 = (int)(idx % q) * 4;
  if (col0 >= n) return;
  uint32_t rho_k = 0;
  if (run > 1) rho_k = (blk2pos[row / Br] % (uint32_t)run + kappa) % (uint32_t)run;
  const float* src = ws + row * ldw + col0;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  // The planes that count are planes 0 .. nvalid-1 (RUN > 1: once a plane is empty the later ones
  // are too).  Four at a time: their loads are issued together, then added in index order; past
  // the last one the load repeats it (a cache hit) and is ignored.  One load per pass of a loop
  // made this kernel wait for memory once per plane.
  int nvalid = planes;
  if (run > 1) {
    nvalid = 0;
    while (nvalid < planes && (int)(nvalid * run + rho_k) - (int)kappa <= run - 2) ++nvalid;
  }
  for (int p0 = 0; p0 < nvalid; p0 += 4) {
    float4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      v[j] = *reinterpret_cast<const float4*>(src + (int64_t)min(p0 + j, nvalid - 1) * k * ldw);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (p0 + j < nvalid) { s.x += v[j].x; s.y += v[j].y; s.z += v[j].z; s.w += v[j].w; }
  }
  float v[4] = {s.x * scale, s.y * scale, s.z * scale, s.w * scale};
  T* dst = out + row * ldo + col0;
  if (out_vec && col0 + 3 < n) {
    if constexpr (sizeof(T) == 2) {
      const uint2 w = pack4<T>(v);
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

// One instantiation, and so one cached limit, per kernel (the kernel is a template argument).
template <auto kernel>
hipError_t go(dim3 grid, unsigned threads, size_t lds, hipStream_t st, const MfmaArgs& a) {
  static size_t raised = 64 * 1024;  // the dynamic-LDS limit set for this kernel so far
  if (lds > raised) {  // above the default dynamic-LDS limit: raise it for this kernel
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    raised = lds;
  }
  hipLaunchKernelGGL(kernel, grid, dim3(threads), lds, st, a);
  return hipGetLastError();
}

// Element-wise loads (Plan::unal): one ring depth, no orbit runs.
template <typename T, bool IN_STAT>
hipError_t launch_shape_unal(const Plan& pl, const MfmaArgs& a, dim3 grid, hipStream_t st) {
#define FS_GO(MT, NCG) \
  return go<mfma_kernel<T, MT, 1, NCG, IN_STAT, 1, 4, 1, false, true>>(grid, 64 * NCG, pl.lds, st, a)
#define FS_GO4(NCG)                                                                                      \
  do {                                                                                                   \
    if constexpr (!IN_STAT) {                                                                            \
      if (pl.nsub > 1)                                                                                   \
        return go<mfma_kernel<T, 4, 1, NCG, false, 1, 4, 1, true, true>>(grid, 64 * NCG, pl.lds, st, a); \
    }                                                                                                    \
    FS_GO(4, NCG);                                                                                       \
  } while (0)
  if (pl.ncg == 1) {
    if (pl.mt == 1) FS_GO(1, 1); else if (pl.mt == 2) FS_GO(2, 1); else FS_GO4(1);
  } else {
    if (pl.mt == 1) FS_GO(1, 2); else if (pl.mt == 2) FS_GO(2, 2); else FS_GO4(2);
  }
#undef FS_GO
#undef FS_GO4
}

template <typename T, bool IN_STAT>
hipError_t launch_shape(const Plan& pl, const MfmaArgs& a, dim3 grid, hipStream_t st) {
#define FS_GO(MT, NRG, NCG, RUN) \
  return go<mfma_kernel<T, MT, NRG, NCG, IN_STAT, RUN, 4>>(grid, 64 * NRG * NCG * RUN, pl.lds, st, a)
#define FS_GO4(NCG)                                                                            \
  do {                                                                                         \
    if constexpr (!IN_STAT) {                                                                  \
      if (pl.nsub > 1) {                                                                       \
        if constexpr (sizeof(T) == 2) {                                                        \
          if (pl.pfx == 2)                                                                     \
            return go<mfma_kernel<T, 4, 1, NCG, false, 1, 4, 2, true>>(grid, 64 * NCG, pl.lds, st, a); \
        }                                                                                      \
        return go<mfma_kernel<T, 4, 1, NCG, false, 1, 4, 1, true>>(grid, 64 * NCG, pl.lds, st, a);     \
      }                                                                                        \
    }                                                                                          \
    if constexpr (sizeof(T) == 2) {                                                            \
      if (pl.pfx == 2)                                                                         \
        return go<mfma_kernel<T, 4, 1, NCG, IN_STAT, 1, 4, 2>>(grid, 64 * NCG, pl.lds, st, a); \
    }                                                                                          \
    return go<mfma_kernel<T, 4, 1, NCG, IN_STAT, 1, 4, 1>>(grid, 64 * NCG, pl.lds, st, a);     \
  } while (0)
  if constexpr (IN_STAT) {
    if (pl.run == 4) FS_GO(2, 1, 2, 4);
  }
  if (pl.ncg == 1) {
    if (pl.mt == 1) FS_GO(1, 1, 1, 1); else if (pl.mt == 2) FS_GO(2, 1, 1, 1); else FS_GO4(1);
  } else {
    if (pl.mt == 1) FS_GO(1, 1, 2, 1); else if (pl.mt == 2) FS_GO(2, 1, 2, 1); else FS_GO4(2);
  }
#undef FS_GO
#undef FS_GO4
}


}  // namespace
}  // namespace fs
