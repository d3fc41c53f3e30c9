// BlockPerm-SJLT apply with S output blocks, consecutive on the orbit of the wiring, stacked in
// the accumulators of one wave: A travels from L2 into registers (kappa+S-1)/S times per output
// block instead of kappa times.
//
// Alg. 1 gives one output block to a work-group and streams its kappa input blocks, so every
// element of A is loaded kappa times; the output-stationary kernels keep all but one of those
// loads in L2, but the traffic from L2 into the compute units, and the work done on it there
// (the transposition or, for fp32, the split into bf16 pieces), is still kappa-fold, and those
// kernels are bound by it (Appendix D names the same bottleneck).  Every permutation of the
// wiring is a power of ONE full-cycle affine map f (Appendix E, "Full-cycle affine
// construction"), so in the order of f's orbit the output block at position o reads the input
// blocks at positions o+1 .. o+kappa.  S consecutive outputs o .. o+S-1 therefore need only the
// kappa+S-1 inputs o+1 .. o+S-1+kappa.  A wave keeps the S output blocks stacked in its
// accumulators (S*Br rows x 64 columns: all 256 accumulation registers); the input at position
// o+1+j feeds the slots i with 0 <= j-i < kappa, a contiguous range.  The result is stored
// directly, scaled, by the one wave that owns it: no partial planes, no second kernel, no
// atomics, a fixed summation order.
//
//  * Phases.  The inputs are taken in kappa phases: a phase takes the inputs whose orbit position
//    has one residue modulo kappa, the same residue in every work-group.  A work-group's window
//    of kappa+S-1 positions holds one such input or two; one feeds all S slots, two feed the slots
//    0..m-1 and m..S-1.  So every phase is the same matrix work in every work-group (each slot
//    gets exactly one block), all readers of an input block read it in the same phase, stage by
//    stage, and all but the first hit L2: with kappa = S HBM sees A once (measured: the same fetch
//    size as the output-stationary kernel).  With kappa = 2S, 3S, .. there are kappa/S kinds of
//    work-group whose two-block phases (a little slower: two loads, two splits per k-step) fall
//    on different residues; the residues are taken in an order that alternates between the kinds,
//    which keeps them within one such difference of each other (kappa = 2S: A is fetched 1.4
//    times; in plain residue order 1.75 times).
//  * A phase of two blocks walks both together: per k-step the 16 rows of the first block for its
//    slots, then the same rows of the second for the others, against ONE Phi tile whose slot i
//    was hashed with the block that feeds slot i.  Phi is made kappa times per output block, as in
//    Alg. 1, not kappa+S-1 times.
//  * Work-group = (group of S outputs, NW*64 columns): NW waves, one per SIMD, sharing one pair of
//    Phi tiles [S*Br][KC+8] in LDS.  A lane of wave w makes the nonzeros of one (input row, slot)
//    pair of a stage (Appendix E, "Within-block hashing": one row hash per lane and stage) in the
//    K-slice [w*KW, w*KW+KW), which wave w also clears; one work-group barrier per stage,
//    ordering LDS traffic only, placed one k-step before the stage ends.
//  * The slot range of a sub-step is a template argument: straight-line code, no test per slot.
//    With S | kappa the phases of two blocks come in one run (m = 1, 2, .. S-1), so the kernel is
//    a fixed sequence of loops, one per shape of phase, with no choice inside a loop.  (A choice
//    inside the loop, or a loop that touches different accumulators in its two halves, made the
//    register allocator move accumulators in and out of the accumulation registers on every
//    pass.)
//  * One wave per SIMD has nobody to hide behind, so the instruction stream is laid out by hand:
//    every k-step is cut into scheduling regions in which MFMAs alternate with a fixed number of
//    other instructions.  For fp32 the three pieces of a value go to the same accumulator, so each
//    piece gets a region of its own: within a region no two MFMAs depend on each other.
//  * A: HBM -> registers (2 columns x 8 rows per lane and sub-step, loop-invariant scalar row
//    offsets, one VGPR offset) -> v_perm transpose (16-bit types) or the exact 3-way bf16 split
//    (fp32) -> MFMA B operands.  Loads run PFD sub-steps ahead in a register ring.  Loads past the
//    last phase go to an empty descriptor range (they return 0 and move nothing) and the tile made
//    after the last stage is never read, so the stage code has no first/last variants.
//
// Needs the orbit table, S | M, S | kappa, an even number of 64-row stages per input block, and
// blocks exactly 64 (S = 4) or 128 (S = 2, fp32 only: for 16-bit types the kernel with one block
// per work-group is the faster one there) rows high.
// Inputs must be finite (a dense product also multiplies by the zeros of Phi).
//
// FS_ABLATE_LOADS / FS_ABLATE_FILL: compile-time switches for timing the kernel with the loads of A
// (after the prologue) or the making of Phi taken out (wrong results; never defined in the shipped build).
#include <stdio.h>

#include <type_traits>

#include "handle.h"
#include "mfma_common.h"
#include "spec.h"

namespace fs {
namespace {

using namespace mm;

constexpr int MAX_PHASES = MAX_KAPPA;  // one phase per permutation

struct StackedArgs {
  SketchParams p;
  const void* A;
  void* out;
  const uint32_t* pos2blk;  // orbit order of the blocks
  int64_t lda, ldo;
  int n;
  int spb;      // stages per input block: ceil(Bc / KC), even
  int out_vec;  // out and ldo allow stores of 2 elements
};

// the loaded vector of one lane and row: 2 consecutive columns
template <typename T> struct Ld2 { using V = uint32_t; };
template <> struct Ld2<float> { using V = uint2; };

template <typename T, int MTS, int S, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1)))
void stacked_kernel(StackedArgs a) {
  using V = typename Ld2<T>::V;
  constexpr bool F32 = sizeof(T) == 4;
  constexpr int CG = 2;                        // column groups of 32 per wave
  constexpr int C = 32 * CG;                   // columns per wave
  constexpr int BR = 32 * MTS;                 // rows of an output block
  constexpr int R = S * BR;                    // stacked rows = rows of a Phi tile
  constexpr int TILE = R * PHI_LD;             // 16-bit elements of one Phi tile
  constexpr int PFS = F32 ? 1 : 2;
  constexpr int PFD = PFS * KSTEPS;            // sub-steps the loads of A run ahead
  constexpr int NP = F32 ? 3 : 1;              // bf16 pieces per value
  constexpr int KW = KC / NW;                  // fill: K-columns per wave
  constexpr int LPR = 64 / (KW * S);           // fill: lanes that share one (input row, slot) pair
  constexpr int NPUT = 8 / LPR;                // fill: nonzeros per lane written by straight-line code (s <= 8)
  static_assert(KW * S * LPR == 64 && NPUT % 4 == 0, "fill layout");
  constexpr int UPR = KW / 8;                  // 16-byte units per tile row of a wave's K-slice
  constexpr int NT = 64 * NW;
  static_assert(S * MTS * CG * 16 == 256, "256 accumulator registers");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // per phase: the input block of the first half, of the second half (the same block when the
  // phase has one), how many slots the first feeds (S: the phase has one block), the block keys
  uint32_t* s_hx = reinterpret_cast<uint32_t*>(smem);
  uint32_t* s_hy = s_hx + MAX_PHASES;
  uint32_t* s_m = s_hy + MAX_PHASES;
  uint32_t* s_key = s_m + MAX_PHASES;  // [phase * S + slot]
  uint16_t* s_phi = reinterpret_cast<uint16_t*>(smem + (size_t)MAX_PHASES * (S + 3) * 4);  // two tiles

  const SketchParams& p = a.p;
  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6, kg = lane >> 5;
  const uint32_t NPH = p.kappa;  // phases

  // work-group -> (output group, column tile); linear ids are dealt round-robin over the 8 XCDs, so
  // the renumbering gives an XCD consecutive groups of one column tile (they share input blocks)
  uint32_t grp = blockIdx.x, jt = blockIdx.y;
  {
    const uint32_t total = gridDim.x * gridDim.y;
    uint32_t id = blockIdx.y * gridDim.x + blockIdx.x;
    if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
    grp = id % gridDim.x;
    jt = id / gridDim.x;
  }
  const uint32_t pos0 = grp * S;  // orbit position of slot 0
  // A phase takes the inputs whose orbit position has one residue modulo kappa.  The first of them
  // in the window pos0+1 .. pos0+kappa+S-1 is input j (position pos0+1+j) with j < kappa; it feeds
  // the slots 0..j.  If j <= S-2 the window holds a second one, input j+kappa, for the slots
  // j+1..S-1.  Phase number ph takes the residue (ph % KS) S + ph / KS, KS = kappa / S: a group
  // whose first position is t S modulo kappa has its two-block phases at the residues t S + 1 ..
  // t S + S-1, and in this order they are the phases t + KS, t + 2 KS, ..: between the two-block
  // phases of one kind of group come those of the others, so the kinds (their two-block phases
  // take a little longer) never get more than one such difference apart, and stay close enough
  // for the second reader of a block to find it in L2.
  const uint32_t KS = p.kappa / (uint32_t)S;
  for (uint32_t ph = tid; ph < NPH; ph += NT) {
    const uint32_t res = (ph % KS) * (uint32_t)S + ph / KS;
    const uint32_t j = (res + p.kappa - (pos0 + 1) % p.kappa) % p.kappa;
    const bool two = j + 1 < (uint32_t)S;
    const uint32_t hx = a.pos2blk[(pos0 + 1 + j) % p.M];
    const uint32_t hy = two ? a.pos2blk[(pos0 + 1 + j + p.kappa) % p.M] : hx;
    const uint32_t m = two ? j + 1 : (uint32_t)S;
    s_hx[ph] = hx;
    s_hy[ph] = hy;
    s_m[ph] = m;
#pragma unroll
    for (int i = 0; i < S; ++i)
      s_key[ph * S + i] = block_key(p.key1, a.pos2blk[pos0 + i], (uint32_t)i < m ? hx : hy, p.M);
  }
  for (int i = tid; i < 2 * TILE / 8; i += NT) reinterpret_cast<uint4*>(s_phi)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();

  // ---- addressing of A ------------------------------------------------------------------
  const int col0 = (int)jt * (C * NW) + wave * C + 2 * (lane & 31);
  const char* Abase = reinterpret_cast<const char*>(a.A);
  const int64_t row_bytes = a.lda * (int64_t)sizeof(T);
  // a lane whose columns lie at or beyond n gets an offset outside every descriptor range: its
  // loads return 0 and move no data.  (n is even here, so a lane's two columns are both valid or
  // both not.)
  const uint32_t voff0 = col0 < a.n ? (uint32_t)(((int64_t)(kg * 8) * a.lda + col0) * (int64_t)sizeof(T))
                                    : 0x80000000u;
  uint32_t soff[8];  // loop-invariant scalar offsets of the 8 rows of a k-step
#pragma unroll
  for (int j = 0; j < 8; ++j) soff[j] = (uint32_t)j * (uint32_t)row_bytes;
  const uint32_t kstep_bytes = 16u * (uint32_t)row_bytes;
  // Descriptor over the rows of input block hb; rows at or beyond d (zero padding of a partly
  // filled last block) and rows of a block's last stage at or beyond Bc lie outside its range and
  // read as 0; phases past the last get an empty range.
  auto make_rsrc = [&](uint32_t hb, bool live) {
    const int64_t first_row = (int64_t)hb * p.Bc;
    const int64_t valid = live ? min((int64_t)p.Bc, p.d - first_row) : 0;
    const int64_t bytes = valid > 0 ? (valid - 1) * row_bytes + (int64_t)a.n * (int64_t)sizeof(T) : 0;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(Abase + first_row * row_bytes), 0, (int)bytes,
                                             0x00020000);
  };

  f32x16 acc[S][MTS][CG];
#pragma unroll
  for (int i = 0; i < S; ++i)
#pragma unroll
    for (int mt = 0; mt < MTS; ++mt)
#pragma unroll
      for (int c = 0; c < CG; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][mt][c][r] = 0.f;

  // ---- cursors -------------------------------------------------------------------------------
  // The work is a sequence of sub-steps of 16 input rows: per phase, stage and k-step, the k-step's
  // rows of the first block (for the slots it feeds), then the same rows of the second block if
  // the phase has one.
  const uint32_t spb = (uint32_t)a.spb;
  // loads: PFD sub-steps ahead of the MFMAs in that sequence
  __amdgpu_buffer_rsrc_t f_rsx, f_rsy;
  uint32_t f_voff = voff0, f_ph = 0, f_left = 0;  // f_left: k-steps left in the phase being loaded
  bool f_two = false, f_second = false;
  auto load_fetch_phase = [&]() {
    const uint32_t ph = min(f_ph, NPH - 1);
    const bool live = f_ph < NPH;
    f_rsx = make_rsrc(__builtin_amdgcn_readfirstlane(s_hx[ph]), live);
    f_rsy = make_rsrc(__builtin_amdgcn_readfirstlane(s_hy[ph]), live);
    f_two = __builtin_amdgcn_readfirstlane(s_m[ph]) < (uint32_t)S;
    f_voff = voff0;
    f_left = spb * (uint32_t)KSTEPS;
  };
  load_fetch_phase();
  V ld[PFD][8];
#ifdef FS_ABLATE_LOADS
  bool loads_on = true;  // ablation build: only the prologue loads A, the ring keeps that data
#endif
  // the next sub-step of the sequence (no branches: a k-step stays one scheduling region)
  auto issue = [&](V (&dst)[8]) {
    const __amdgpu_buffer_rsrc_t rs = f_second ? f_rsy : f_rsx;
#ifdef FS_ABLATE_LOADS
    if (loads_on)
#endif
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if constexpr (F32)
        dst[j] = __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b64(rs, f_voff, soff[j], 0));
      else
        dst[j] = (V)__builtin_amdgcn_raw_buffer_load_b32(rs, f_voff, soff[j], 0);
    }
    const bool k_done = !f_two || f_second;  // that was the k-step's last sub-step
    f_second = f_two && !f_second;
    f_voff += k_done ? kstep_bytes : 0u;
    f_left -= k_done ? 1u : 0u;
  };
  // between k-steps: the phase being loaded may have ended (never between the two sub-steps of a
  // k-step: the loads run an even number of sub-steps ahead and a phase has an even number)
  auto fetch_phase_check = [&]() {
    if (f_left == 0) {
      ++f_ph;
      load_fetch_phase();
    }
  };
  // Phi, one stage ahead.  A lane makes the nonzeros of ONE (input row, slot) pair of a stage:
  // K-column sh_col of its wave's slice, slot sh_slot, and of that row's s nonzeros the ones
  // numbered sh_j, sh_j + LPR, ... (LPR lanes share a pair), so it evaluates one row hash a stage.
  uint32_t p_us = 0, p_ph = 0;
  uint32_t p_key = 0;  // block key of this lane's slot in the phase being made
  uint32_t p_lim = 0;  // s, or 0 past the last phase: nonzeros numbered below it are real
  const uint32_t sh_col = (uint32_t)(wave * KW + lane % KW), sh_slot = (uint32_t)((lane / KW) % S);
  const uint32_t sh_j = (uint32_t)(lane / (KW * S));
  auto load_keys = [&]() {
    p_key = s_key[min(p_ph, NPH - 1) * S + sh_slot];
    p_lim = p_ph < NPH ? p.s : 0u;
  };
  load_keys();
  // byte offset of (first row of the lane's slot, the lane's K-column) in a tile, and of a pad column
  const uint32_t sh_base = sh_slot * (uint32_t)(BR * PHI_LD * 2) + sh_col * 2u;
  const uint32_t sh_padb = (uint32_t)((lane & 31) * PHI_LD + KC + ((wave * 2 + kg) & 7)) * 2u;
  uint32_t pr = 0, pstep = 0, psg = 0;  // next tile row of this lane's share, its stride, the sign bits left
  auto hash_row = [&]() {
    const RowHash rh = row_hash_pow2(p_key, p_us * KC + sh_col, (uint32_t)BR);
    pr = (rh.shift + sh_j * rh.stride) & (BR - 1);
    pstep = (uint32_t)LPR * rh.stride;
    psg = rh.signs >> sh_j;
  };
  // one nonzero: the 16-bit pattern of +-1 (`one` with the hash's sign bit at bit 15); nonzeros
  // numbered s or more go to a pad column that no MFMA reads
  auto put = [&](uint16_t* tile, uint32_t idx, uint32_t sign_at_bit0) {
    // (a select written with masks: as a conditional expression it compiles to a branch, which
    // cuts the k-step into several scheduling regions)
    const uint32_t real = idx < p_lim ? 0xFFFFFFFFu : 0u;
    const uint32_t at = __umul24(pr, (uint32_t)(PHI_LD * 2)) + sh_base;
    const uint32_t off = (at & real) | (sh_padb & ~real);
    *reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(tile) + off) =
        (uint16_t)(((sign_at_bit0 << 15) & 0x8000u) | Fmt<T>::one);
    pr = (pr + pstep) & (BR - 1);
  };
  // This wave's share of making a tile, in parts that the half-stages spread over their k-steps:
  // part 0 clears the K-slice and hashes, parts 1 to 4 write NPUT / 4 nonzeros each; part 6 (rarely
  // needed: s > 8) loops over the remaining nonzeros.
  auto fill = [&](uint16_t* tile, int part) {
#ifdef FS_ABLATE_FILL
    return;  // ablation build: Phi stays zero
#endif
    if (part == 0) {
#pragma unroll
      for (int u = 0; u < R * UPR / 64; ++u) {
        const int unit = lane + 64 * u;
        *reinterpret_cast<uint4*>(tile + (unit / UPR) * PHI_LD + wave * KW + (unit % UPR) * 8) = make_uint4(0, 0, 0, 0);
      }
      hash_row();
    } else if (part >= 1 && part <= 4) {
#pragma unroll
      for (int q = (part - 1) * (NPUT / 4); q < part * (NPUT / 4); ++q)
        put(tile, sh_j + (uint32_t)(q * LPR), psg >> (q * LPR));
    } else if (part == 6) {
      if (p.s > (uint32_t)(NPUT * LPR)) {
        for (uint32_t i0 = (uint32_t)(NPUT * LPR); i0 < p.s; i0 += LPR) put(tile, i0 + sh_j, psg >> i0);
      }
    }
  };
  auto fill_stage_end = [&]() {
    if (++p_us == spb) {
      p_us = 0;
      ++p_ph;
      load_keys();
    }
  };
  // work-group barrier that orders LDS traffic only (the loads of A in flight stay in flight)
  auto lds_barrier = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };

  uint4 pa2[2][S][MTS];  // Phi operands of the current and of the next k-step
  auto read_slot = [&](const uint16_t* tile, int ks, int i, uint4 (&dst)[S][MTS]) {
#pragma unroll
    for (int mt = 0; mt < MTS; ++mt)
      dst[i][mt] = *reinterpret_cast<const uint4*>(tile + ((i * MTS + mt) * 32 + (lane & 31)) * PHI_LD + ks * 16 + kg * 8);
  };

  // MFMA B operands of a k-step from the 8 rows x 2 columns a lane loaded: [column group][piece]
  auto make_b = [&](const V (&r)[8], uint4 (&op)[CG][NP]) {
    if constexpr (F32) {
#pragma unroll
      for (int c = 0; c < CG; ++c) {
        uint32_t xs[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) xs[j] = c == 0 ? r[j].x : r[j].y;
        split_ops(xs, op[c][0], op[c][1], op[c][2]);
      }
    } else {
#pragma unroll
      for (int c = 0; c < CG; ++c) {
        uint32_t* o = reinterpret_cast<uint32_t*>(&op[c][0]);
#pragma unroll
        for (int q = 0; q < 4; ++q) o[q] = perm(r[2 * q + 1], r[2 * q], c == 0 ? 0x05040100u : 0x07060302u);
      }
    }
  };

  // One sub-step: the MFMAs of the slots LO..HI (compile time) on the 16 rows in ring slot rs, the
  // loads PFD sub-steps ahead into that slot, and the side work handed in (parts of the next tile,
  // reads of the next Phi operands) spread between the MFMAs.
  auto sub_step = [&](auto lo_tag, auto hi_tag, int rs, const uint4 (&pa)[S][MTS], auto&& side_a, auto&& side_b) __attribute__((always_inline)) {
    constexpr int LO = decltype(lo_tag)::value, HI = decltype(hi_tag)::value;
    constexpr int NMP = CG * (HI - LO + 1) * MTS;  // MFMAs per piece: all to different accumulators
    V(&cur)[8] = ld[rs];
    auto mfma_piece = [&](auto pc_tag, const uint4 (&op)[CG][NP]) {
      constexpr int pc = decltype(pc_tag)::value;
#pragma unroll
      for (int c = 0; c < CG; ++c)
#pragma unroll
        for (int i = LO; i <= HI; ++i)
#pragma unroll
          for (int mt = 0; mt < MTS; ++mt) {
            acc[i][mt][c] = mfma<T>(pa[i][mt], op[c][pc], acc[i][mt][c]);
          }
    };
    uint4 op[CG][NP];
    if constexpr (F32) {
      // The three pieces of a value go to the same accumulator, so the pieces are taken one after
      // the other, each piece's MFMAs in a scheduling region of its own: within a region no two
      // MFMAs depend on each other and the order the compiler picks does no harm.  Region 0: the
      // split of the values and the loads between the MFMAs of the first piece.  Regions 1 and 2:
      // the side work between the MFMAs of the second and third piece.
      make_b(cur, op);
      issue(cur);
      mfma_piece(std::integral_constant<int, 0>{}, op);
#pragma unroll
      for (int m = 0; m < NMP; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x006, 96 / NMP, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, NMP >= 16 ? 1 : NMP >= 8 ? 2 : 4, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      side_a();
      mfma_piece(std::integral_constant<int, 1>{}, op);
#pragma unroll
      for (int m = 0; m < NMP; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x006, 96 / NMP, 0);
        __builtin_amdgcn_sched_group_barrier(0x080, NMP >= 16 ? 1 : NMP >= 8 ? 2 : 4, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      side_b();
      mfma_piece(std::integral_constant<int, 2>{}, op);
#pragma unroll
      for (int m = 0; m < NMP; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x006, 96 / NMP, 0);
        __builtin_amdgcn_sched_group_barrier(0x080, NMP >= 16 ? 1 : NMP >= 8 ? 2 : 4, 0);
      }
    } else {
      side_a();
      side_b();
      make_b(cur, op);
      issue(cur);
      mfma_piece(std::integral_constant<int, 0>{}, op);
      // spread the rest evenly between the MFMAs
#pragma unroll
      for (int m = 0; m < NMP; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x006, NMP >= 16 ? 5 : 10, 0);
        __builtin_amdgcn_sched_group_barrier(0x090, NMP >= 16 ? 1 : 2, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // One stage of a phase whose first block feeds M_ slots (M_ = S: its only block): 4 k-steps on
  // tile PAR, each of one sub-step (all slots) or two (slots below M_ on the first block's rows,
  // the others on the second block's), while this wave's share of the next tile is made.  The
  // work-group barrier sits one k-step before the end; behind it the last k-step reads the first
  // operands of the next stage from the new tile.
  auto stage = [&](auto par_tag, auto m_tag, int seq) __attribute__((always_inline)) {  // seq: number of the stage in its loop pass
    constexpr int PAR = decltype(par_tag)::value, M_ = decltype(m_tag)::value;
    uint16_t* cur_tile = s_phi + PAR * TILE;
    uint16_t* fill_tile = s_phi + (1 - PAR) * TILE;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      uint4(&pa)[S][MTS] = pa2[ks & 1];
      uint4(&pn)[S][MTS] = pa2[(ks + 1) & 1];
      // the first three k-steps make two parts of the next tile each
      auto part_a = [&]() { if (ks < 3) fill(fill_tile, 2 * ks); };
      auto part_b = [&]() { if (ks < 3) fill(fill_tile, 2 * ks + 1); };
      auto read_next = [&]() {  // the Phi operands of the next k-step
#pragma unroll
        for (int i = 0; i < S; ++i) {
          if (ks + 1 < KSTEPS) read_slot(cur_tile, ks + 1, i, pn);
          else read_slot(fill_tile, 0, i, pn);
        }
      };
      auto nothing = [&]() {};
      using Z = std::integral_constant<int, 0>;
      using LAST = std::integral_constant<int, S - 1>;
      if constexpr (M_ == S) {
        sub_step(Z{}, LAST{}, (seq * KSTEPS + ks) % PFD, pa, part_a, [&]() { part_b(); read_next(); });
      } else {
        sub_step(Z{}, std::integral_constant<int, M_ - 1>{}, (seq * 2 * KSTEPS + 2 * ks) % PFD, pa, part_a, nothing);
        sub_step(std::integral_constant<int, M_>{}, LAST{}, (seq * 2 * KSTEPS + 2 * ks + 1) % PFD, pa, part_b, read_next);
      }
      if (ks == 2) {
        // Every wave has by now issued its last reads of cur_tile (the operands of k-step 3) and
        // its writes to fill_tile: behind this barrier cur_tile may be cleared (next stage) and
        // fill_tile read (next k-step).
        fill(fill_tile, 6);
        lds_barrier();
      }
      __builtin_amdgcn_sched_barrier(0);
      fetch_phase_check();
    }
    fill_stage_end();
  };

  // ---- prologue ---------------------------------------------------------------------------------
#pragma unroll
  for (int i = 0; i < PFD; ++i) {
    issue(ld[i]);
    if (!f_second) fetch_phase_check();
  }
  for (int part = 0; part < 7; ++part) fill(s_phi, part);
  fill_stage_end();
  lds_barrier();
#ifdef FS_ABLATE_LOADS
  loads_on = false;
#endif
#pragma unroll
  for (int i = 0; i < S; ++i) read_slot(s_phi, 0, i, pa2[0]);

  // ---- the walk over the phases and stages ------------------------------------------------------------
  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;
  // With S | kappa a group of kind t (first position t S modulo kappa) has phases of one block
  // except the phases t + i KS, i = 1 .. S-1, which have two with i slots on the first.  So the
  // walk is a fixed sequence of loops.  (Straight-line code, one loop per shape and no choice
  // inside a loop: with a choice the register allocator gives the accumulators different homes in
  // the branches and moves them at every join.)
  auto run = [&](auto m_tag, uint32_t phases) __attribute__((always_inline)) {
    // (a pass of the loop covers a whole number of turns of the load ring)
    constexpr int PASS = PFS > 2 ? 4 : 2;
    for (uint32_t c = phases * spb; c > 0; c -= PASS) {
      stage(P0{}, m_tag, 0);
      stage(P1{}, m_tag, 1);
      if constexpr (PASS == 4) {
        stage(P0{}, m_tag, 2);
        stage(P1{}, m_tag, 3);
      }
    }
  };
  const uint32_t kind = (pos0 / (uint32_t)S) % KS;
  run(std::integral_constant<int, S>{}, KS + kind);
  run(std::integral_constant<int, 1>{}, 1);
  if constexpr (S >= 4) {
    run(std::integral_constant<int, S>{}, KS - 1);
    run(std::integral_constant<int, 2>{}, 1);
    run(std::integral_constant<int, S>{}, KS - 1);
    run(std::integral_constant<int, 3>{}, 1);
  }
  run(std::integral_constant<int, S>{}, KS - 1 - kind);

  // ---- epilogue: scale, convert, store the S blocks ---------------------------------------------------
  // accumulator register r of tile (i, mt, c) holds row mt*32 + 8*(r/4) + 4*kg + r%4 of the block
  // in slot i, column col0 + c
  if (col0 >= a.n) return;
#pragma unroll
  for (int i = 0; i < S; ++i) {
    const uint32_t g = a.pos2blk[pos0 + i];
#pragma unroll
    for (int mt = 0; mt < MTS; ++mt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = (uint32_t)(mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3));
        const float v0 = acc[i][mt][0][r] * p.scale, v1 = acc[i][mt][1][r] * p.scale;
        T* dst = reinterpret_cast<T*>(a.out) + ((int64_t)g * BR + row) * a.ldo + col0;
        if (!a.out_vec) {
          Elt<T>::store(dst, v0);
          Elt<T>::store(dst + 1, v1);
        } else if constexpr (F32) {
          *reinterpret_cast<float2*>(dst) = make_float2(v0, v1);
        } else {
          T e0, e1;
          Elt<T>::store(&e0, v0);
          Elt<T>::store(&e1, v1);
          *reinterpret_cast<uint32_t*>(dst) = (uint32_t)__builtin_bit_cast(uint16_t, e0) |
                                              ((uint32_t)__builtin_bit_cast(uint16_t, e1) << 16);
        }
      }
    }
  }
}

template <auto kernel>
hipError_t go(dim3 grid, unsigned threads, size_t lds, hipStream_t st, const StackedArgs& a) {
  static bool raised = false;
  if (lds > 64 * 1024 && !raised) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    raised = true;
  }
  hipLaunchKernelGGL(kernel, grid, dim3(threads), lds, st, a);
  return hipGetLastError();
}

// the slot count for a shape: 4 blocks of 64 rows, 2 blocks of 128 rows
int slots_for(uint32_t Br) { return Br == 64 ? 4 : Br == 128 ? 2 : 0; }

}  // namespace

bool stacked_supported(const SketchParams& p, const void* A, int64_t lda, int64_t n, fs_dtype dt, bool have_orbit) {
  const int S = slots_for(p.Br);
  const size_t esz = dt == FS_F32 ? 4 : 2;
  // (with fewer permutations than slots a phase could hold three input blocks)
  if (!have_orbit || S == 0 || p.M % S || p.kappa > (uint32_t)MAX_KAPPA || p.kappa < (uint32_t)S) return false;
  // the phases of two blocks must come in one run, in every group: S | kappa
  if (p.kappa % (uint32_t)S) return false;
  // 16-bit types, 128-row blocks: the kernel with one block per work-group is faster (measured on
  // the "wide" workload: 0.445 against 0.475 ms)
  if (dt != FS_F32 && p.Br == 128) return false;
  if (n < 256 || n % 2) return false;
  // two columns per lane: loads of 2 elements
  if ((uintptr_t)A % (2 * esz) || (lda * esz) % (2 * esz)) return false;
  const int64_t spb = ((int64_t)p.Bc + KC - 1) / KC;
  if (spb < 2 || spb % 2) return false;
  if ((16 * lda + n) * (int64_t)esz >= ((int64_t)1 << 31)) return false;
  if (spb * KC * lda * (int64_t)esz >= ((int64_t)1 << 31)) return false;
  const int64_t col_tiles = (n + 255) / 256;
  if (col_tiles > 65535) return false;
  // enough work-groups (they hold a CU each: 4 SIMDs with one wave each) to beat the kernels that
  // split rows instead; measured cross-over on the mid shape: half the CUs
  return (int64_t)(p.M / S) * col_tiles >= 128;
}

hipError_t launch_stacked(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out, int64_t ldo,
                          fs_dtype dt, const uint32_t* orbit, hipStream_t st, EventPair ev, char* desc,
                          size_t desc_cap) {
  StackedArgs a;
  a.p = p; a.A = A; a.out = out; a.pos2blk = orbit;
  a.lda = lda; a.ldo = ldo; a.n = (int)n;
  a.spb = (int)(((int64_t)p.Bc + KC - 1) / KC);
  const size_t esz = dt == FS_F32 ? 4 : 2;
  a.out_vec = ((uintptr_t)out % (2 * esz) == 0 && (ldo * esz) % (2 * esz) == 0) ? 1 : 0;
  const int S = slots_for(p.Br);
  constexpr int NW = 4;
  const unsigned col_tiles = (unsigned)((n + 64 * NW - 1) / (64 * NW));
  const size_t lds = (size_t)MAX_PHASES * (S + 3) * 4 + 2 * (size_t)(S * p.Br) * PHI_LD * 2;
  dim3 grid(p.M / S, col_tiles, 1);
  if (desc && desc_cap)
    snprintf(desc, desc_cap, "stacked_kernel<%s,%d,%d,%d>", dt == FS_F32 ? "f32" : dt == FS_BF16 ? "bf16" : "f16",
             (int)p.Br / 32, S, NW);
  if (ev.start) (void)hipEventRecord(ev.start, st);
  hipError_t e;
  if (p.Br == 64) {
    if (dt == FS_F32) e = go<stacked_kernel<float, 2, 4, NW>>(grid, 64 * NW, lds, st, a);
    else if (dt == FS_BF16) e = go<stacked_kernel<uint16_t, 2, 4, NW>>(grid, 64 * NW, lds, st, a);
    else e = go<stacked_kernel<f16, 2, 4, NW>>(grid, 64 * NW, lds, st, a);
  } else {
    if (dt != FS_F32) return hipErrorInvalidValue;
    e = go<stacked_kernel<float, 4, 2, NW>>(grid, 64 * NW, lds, st, a);
  }
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  return e;
}

}  // namespace fs
