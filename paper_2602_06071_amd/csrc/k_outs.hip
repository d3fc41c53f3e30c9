// BlockPerm-SJLT apply, output-stationary with SHARED Phi tiles, for 16-bit inputs whose blocks are
// exactly one matrix-core tile high (Br = 32, 64 or 128) -- the bf16 "wide" shape.
//
// Work decomposition as in Alg. 1: a work-group owns (output block g, a tile of columns) and walks
// the kappa input blocks f^l(g) (Appendix E).  What differs from mfma_kernel's output-stationary
// mode is how the work-group makes the +-1 operand Phi and how lean the inner loop is:
//
//  * ONE pair of Phi tiles per work-group.  Wave w hashes (Appendix E, "Within-block hashing") only
//    the KC/NW input rows [w*KW, w*KW + KW) of a stage, LPR lanes per row, each lane writing its
//    share of the row's s nonzeros, and clears only that K-slice of the tile.  Per wave the cost of
//    making Phi falls by the number of waves.  One work-group barrier per stage orders the tiles:
//    it sits at the end of the stage's third k-step, when every wave has issued its last reads of
//    the tile being consumed and finished its writes to the tile being made, so it is rarely waited
//    for; it orders LDS traffic only (the loads of A in flight stay in flight).
//  * With one wave per SIMD (128-row tiles keep 256 accumulator registers) a wave issues in order,
//    one instruction per issue slot, and a 32x32x16 MFMA occupies the matrix pipe for 8 slots: every
//    non-MFMA instruction beyond 7 per MFMA is time the matrix pipe idles.  So the loop carries no
//    address arithmetic: the 8 rows a lane loads per k-step use 8 loop-invariant scalar offsets,
//    the k-step advances one VGPR offset, and the three cursors (loads PFS stages ahead, Phi one
//    stage ahead, MFMAs) are counters stepped once per stage.
//
//  * Too few (output block, column tile) pairs for the chip: grid.z splits the kappa*spb stages of
//    an output block, work-group z takes the stages [z*stages, (z+1)*stages) and stores unscaled
//    fp32 sums to plane z; the fixed-order reduction kernel scales, converts and stores.
//
// A goes HBM -> registers -> v_perm transpose -> MFMA B operand exactly as in mfma_kernel.
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

struct OutsArgs {
  SketchParams p;
  const void* A;
  void* out;
  const uint32_t* pos2blk;  // orbit order of the blocks, or NULL
  int64_t lda, ldo;
  int n;
  int spb;      // stages per input block: ceil(Bc / KC)
  int out_vec;  // out rows allow 4-column vector stores
  // row split: work-group z (grid.z) takes the stages [z*stages, (z+1)*stages) of the kappa*spb
  // stages of its output block and, when there is more than one, stores its unscaled fp32 sums to
  // plane z of ws (k x ldw floats each) for the fixed-order reduction kernel
  int zsplit, stages;
  float* ws;
  int64_t ldw;
};

template <typename T, int MT, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(MT > 2 ? 1 : 2)))
void outs_kernel(OutsArgs a) {
  static_assert(sizeof(T) == 2, "16-bit element types");
  using V = uint2;                              // 4 consecutive columns of one row
  constexpr int RWV = 32 * MT;                  // rows of the output block = of the Phi tile
  constexpr int TILE = RWV * PHI_LD;            // 16-bit elements of one Phi tile
  constexpr int PFS = MT > 2 ? 2 : 1;           // stages the loads of A run ahead
  constexpr int PFD = PFS * KSTEPS;             // ... in k-steps = depth of the register ring
  constexpr int KW = KC / NW, LPR = 64 / KW;    // fill: K-columns per wave, lanes per input row
  constexpr int UPR = KW / 8;                   // 16-byte units per tile row of a wave's K-slice
  constexpr int NT = 64 * NW;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint32_t* s_key = reinterpret_cast<uint32_t*>(smem);  // block key of (g, f^l(g)) per phase
  uint32_t* s_hblk = s_key + MAX_KAPPA;                 // input block per phase
  uint16_t* s_phi = reinterpret_cast<uint16_t*>(smem + 2 * MAX_KAPPA * 4);  // two tiles

  const SketchParams& p = a.p;
  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6, kg = lane >> 5;

  // Which (output block, column tile) this work-group takes.  With the orbit table, work-groups
  // are renumbered so that the ones an XCD runs side by side (linear ids are dealt round-robin
  // over the 8 XCDs) are consecutive orbit positions of one column tile, and each visits its kappa
  // neighbours in the order of their orbit position modulo kappa: the kappa readers of an input
  // block then read it at about the same time and the re-reads hit that XCD's L2.
  uint32_t jt = blockIdx.y, opos = 0, blk = blockIdx.x;
  const bool remap = a.pos2blk != nullptr;
  if (remap) {
    const uint32_t total = gridDim.x * gridDim.y;
    uint32_t id = blockIdx.y * gridDim.x + blockIdx.x;
    if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
    opos = id % gridDim.x;
    jt = id / gridDim.x;
    blk = __builtin_amdgcn_readfirstlane(a.pos2blk[opos]);
  }
  for (int sl = tid; sl < (int)p.kappa; sl += NT) {
    uint32_t x = blk;
    if (remap) {
      const uint32_t l = (sl + p.kappa - (opos + 1) % p.kappa) % p.kappa;
      x = a.pos2blk[(opos + 1 + l) % p.M];
    } else {
      for (int l = 0; l <= sl; ++l) x = wire_next(x, p.a, p.b, p.M);
    }
    s_hblk[sl] = x;
    s_key[sl] = block_key(p.key1, blk, x, p.M);
  }
  for (int i = tid; i < 2 * TILE / 8; i += NT) reinterpret_cast<uint4*>(s_phi)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();

  // ---- addressing of A ------------------------------------------------------------------
  const int col0 = (int)jt * (WCOLS * NW) + wave * WCOLS + 4 * (lane & 31);
  const char* Abase = reinterpret_cast<const char*>(a.A);
  const int64_t row_bytes = a.lda * (int64_t)sizeof(T);
  // a lane whose columns all lie at or beyond n gets an offset outside every descriptor range:
  // its loads return 0 and move no data
  const uint32_t voff0 = col0 < a.n ? (uint32_t)(((int64_t)(kg * 8) * a.lda + col0) * (int64_t)sizeof(T))
                                    : 0x80000000u;
  uint32_t soff[8];  // loop-invariant scalar offsets of the 8 rows of a k-step
#pragma unroll
  for (int j = 0; j < 8; ++j) soff[j] = (uint32_t)j * (uint32_t)row_bytes;
  const uint32_t kstep_bytes = 16u * (uint32_t)row_bytes;
  // Descriptor over the rows of one input block; rows at or beyond d (zero padding of a partly
  // filled last block) and rows of a block's last stage at or beyond Bc lie outside its range and
  // read as 0.  The range ends with the last valid row's columns rounded up to the 4-column vector.
  auto make_rsrc = [&](uint32_t hb) {
    const int64_t first_row = (int64_t)hb * p.Bc;
    const int64_t valid = min((int64_t)p.Bc, p.d - first_row);
    const int64_t ncols = ((int64_t)a.n + 3) & ~(int64_t)3;
    const int64_t bytes = valid > 0 ? (valid - 1) * row_bytes + ncols * (int64_t)sizeof(T) : 0;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(Abase + first_row * row_bytes), 0, (int)bytes,
                                             0x00020000);
  };

  f32x16 acc[MT][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][c][i] = 0.f;

  // ---- the three cursors -------------------------------------------------------------------
  // loads (PFS stages ahead of the MFMAs): descriptor of the block, lane offset, stage in block
  const uint32_t spb = (uint32_t)a.spb;
  const uint32_t t0 = blockIdx.z * (uint32_t)a.stages;  // first stage of this work-group
  uint32_t f_us = t0 % spb, f_l = t0 / spb;
  uint32_t f_voff = voff0 + f_us * (uint32_t)KSTEPS * kstep_bytes;
  __amdgpu_buffer_rsrc_t f_rs = make_rsrc(__builtin_amdgcn_readfirstlane(s_hblk[f_l]));
  V ld[PFD][8];
#ifdef FS_ABLATE_LOADS
  bool loads_on = true;  // ablation build: only the prologue loads A, the ring keeps that data
#endif
  auto issue = [&](V (&dst)[8]) {
#ifdef FS_ABLATE_LOADS
    if (loads_on)
#endif
#pragma unroll
    for (int j = 0; j < 8; ++j)
      dst[j] = __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b64(f_rs, f_voff, soff[j], 0));
    f_voff += kstep_bytes;
  };
  auto fetch_stage_end = [&]() {
    if (++f_us == spb) {
      f_us = 0;
      f_voff = voff0;
      if (++f_l < p.kappa) f_rs = make_rsrc(__builtin_amdgcn_readfirstlane(s_hblk[f_l]));
    }
  };
  // Phi (one stage ahead): key of the block, stage in block
  uint32_t p_us = t0 % spb, p_l = t0 / spb, p_key = __builtin_amdgcn_readfirstlane(s_key[p_l]);
  const uint32_t sh_col = (uint32_t)(wave * KW + lane % KW), sh_j = (uint32_t)(lane / KW);
  // byte offsets inside a tile: this lane's K-column, and a pad column that no MFMA reads
  const uint32_t sh_colb = sh_col * 2u;
  const uint32_t sh_padb = (uint32_t)((lane & 31) * PHI_LD + KC + ((wave * 2 + kg) & 7)) * 2u;
  uint32_t pr = 0, pstep = 0, psg = 0;  // next tile row of this lane's share, its stride, its sign bits
  // This wave's share of making a tile.  Part 0 clears its K-slice and hashes its input rows;
  // part 1 scatters the first two nonzeros of each lane's share (lane share j writes nonzeros
  // j, j + LPR, ...: all of them when s <= 2 LPR); part 2, the rest (a loop, rarely entered).
  // A nonzero is the 16-bit pattern of +-1: `one` with the hash's sign bit moved to bit 15.
  auto put = [&](uint16_t* tile, uint32_t i, uint32_t sign_at_bit0) {
    const uint32_t off = i < p.s ? __umul24(pr, (uint32_t)(PHI_LD * 2)) + sh_colb : sh_padb;
    *reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(tile) + off) =
        (uint16_t)(((sign_at_bit0 << 15) & 0x8000u) | Fmt<T>::one);
    pr = (pr + pstep) & (p.Br - 1);
  };
  auto fill = [&](uint16_t* tile, int part) {
#ifdef FS_ABLATE_FILL
    return;  // ablation build: Phi stays zero
#endif
    if (part == 0) {
#pragma unroll
      for (int i = 0; i < RWV * UPR / 64; ++i) {
        const int unit = lane + 64 * i;
        *reinterpret_cast<uint4*>(tile + (unit / UPR) * PHI_LD + wave * KW + (unit % UPR) * 8) = make_uint4(0, 0, 0, 0);
      }
      const RowHash rh = row_hash_pow2(p_key, p_us * KC + sh_col, p.Br);
      pr = (rh.shift + sh_j * rh.stride) & (p.Br - 1);
      pstep = (uint32_t)LPR * rh.stride;
      psg = rh.signs >> sh_j;
    } else if (part == 1) {
      put(tile, sh_j, psg);
      put(tile, sh_j + LPR, psg >> LPR);
    } else if (part == 2) {
      if (p.s > 2u * LPR)
        for (uint32_t i0 = 2u * LPR; i0 < p.s; i0 += LPR) put(tile, i0 + sh_j, psg >> i0);
    }
  };
  auto fill_stage_end = [&]() {
    if (++p_us == spb) {
      p_us = 0;
      p_l = min(p_l + 1u, p.kappa - 1u);
      p_key = __builtin_amdgcn_readfirstlane(s_key[p_l]);
    }
  };
  // work-group barrier that orders LDS traffic only
  auto lds_barrier = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };

  // Ragged last column tile: a lane's 4-column vector may straddle column n.  What it then loads
  // beyond n is the row's own padding (lda is a multiple of 4, so the memory is the caller's), and
  // it needs no masking: column c of the lane feeds only the accumulators of column col0 + c (a
  // column of a matrix product depends on that column of the right operand alone), and columns at
  // or beyond n are never stored.

  uint4 pa2[2][MT];  // Phi operands of the current and of the next k-step
  auto read_pa = [&](const uint16_t* tile, int ks, uint4 (&dst)[MT]) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      dst[mt] = *reinterpret_cast<const uint4*>(tile + (mt * 32 + (lane & 31)) * PHI_LD + ks * 16 + kg * 8);
  };

  // One stage: 4 k-steps of 4 MT MFMAs on tile PAR while the loads PFS stages ahead are issued into
  // the ring slots just consumed and this wave's share of the next tile is made.
  auto stage = [&](auto par_tag, auto fetch_tag, auto fill_tag) {
    constexpr int PAR = decltype(par_tag)::value;
    constexpr bool FETCH = decltype(fetch_tag)::value;
    constexpr bool FILL = decltype(fill_tag)::value;
    uint16_t* cur_tile = s_phi + PAR * TILE;
    uint16_t* fill_tile = s_phi + (1 - PAR) * TILE;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      V(&cur)[8] = ld[(PFS > 1 ? PAR * KSTEPS : 0) + ks];
      uint4(&pa)[MT] = pa2[ks & 1];
      uint4(&pn)[MT] = pa2[(ks + 1) & 1];
      if constexpr (FILL) {
        if (ks < 2) fill(fill_tile, ks);
      }
      if (ks + 1 < KSTEPS) read_pa(cur_tile, ks + 1, pn);
      else if constexpr (FILL) read_pa(fill_tile, 0, pn);
      uint4 op[4];
      make_ops(cur, op);
      if constexpr (FETCH) issue(cur);
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc[mt][c] = mfma<T>(pa[mt], op[c], acc[mt][c]);
        }
      // spread the rest evenly between the MFMAs
#pragma unroll
      for (int i = 0; i < 4 * MT; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, MT > 2 ? 3 : 5, 0);
        __builtin_amdgcn_sched_group_barrier(0x090, MT > 2 ? 1 : 2, 0);
      }
      if constexpr (FILL) {
        if (ks == 1) fill(fill_tile, 2);
      }
      // Every wave has by now issued its last reads of cur_tile (k-step KSTEPS-1's operands) and its
      // writes to fill_tile (k-steps 0 and 1): behind this barrier cur_tile may be cleared (next
      // stage) and fill_tile read (next k-step).
      if constexpr (FILL) {
        if (ks == KSTEPS - 2) lds_barrier();
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (FETCH) fetch_stage_end();
    if constexpr (FILL) fill_stage_end();
  };

  // ---- prologue, main loop ----------------------------------------------------------------------
#pragma unroll
  for (int i = 0; i < PFD; ++i) {
    issue(ld[i]);
    if (i % KSTEPS == KSTEPS - 1) fetch_stage_end();
  }
  fill(s_phi, 0);
  fill(s_phi, 1);
  fill(s_phi, 2);
  fill_stage_end();
  lds_barrier();
#ifdef FS_ABLATE_LOADS
  loads_on = false;
#endif
  read_pa(s_phi, 0, pa2[0]);
  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;
  const int n_stages = a.stages;  // even, >= 2 (checked on the host)
  for (int t = 0; t + 2 < n_stages; t += 2) {
    stage(P0{}, std::true_type{}, std::true_type{});
    stage(P1{}, std::true_type{}, std::true_type{});
  }
  if constexpr (PFS > 1) {
    stage(P0{}, std::false_type{}, std::true_type{});
  } else {
    stage(P0{}, std::true_type{}, std::true_type{});
  }
  stage(P1{}, std::false_type{}, std::false_type{});

  // ---- epilogue: scale, convert, store ------------------------------------------------------------
  // accumulator register i of tile (mt, c) holds block row mt*32 + 8*(i/4) + 4*kg + i%4 of column
  // col0 + c
  if (col0 >= a.n) return;
  if (a.zsplit > 1) {  // a partial sum: plane blockIdx.z (ldw is a multiple of 4 and col0 + 3 < ldw)
    float* plane = a.ws + (int64_t)blockIdx.z * p.k * a.ldw;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const uint32_t row = (uint32_t)(mt * 32 + 8 * (i >> 2) + 4 * kg + (i & 3));
        *reinterpret_cast<float4*>(plane + ((int64_t)blk * p.Br + row) * a.ldw + col0) =
            make_float4(acc[mt][0][i], acc[mt][1][i], acc[mt][2][i], acc[mt][3][i]);
      }
    }
    return;
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t row = (uint32_t)(mt * 32 + 8 * (i >> 2) + 4 * kg + (i & 3));
      float v[4] = {acc[mt][0][i] * p.scale, acc[mt][1][i] * p.scale, acc[mt][2][i] * p.scale,
                    acc[mt][3][i] * p.scale};
      T* dst = reinterpret_cast<T*>(a.out) + ((int64_t)blk * p.Br + row) * a.ldo + col0;
      if (a.out_vec && col0 + 3 < a.n) {
        *reinterpret_cast<uint2*>(dst) = pack4<T>(v);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (col0 + c < a.n) Elt<T>::store(dst + c, v[c]);
      }
    }
  }
}

template <auto kernel>
hipError_t go(dim3 grid, unsigned threads, size_t lds, hipStream_t st, const OutsArgs& a) {
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

template <typename T, int MT>
hipError_t launch_t(int nw, dim3 grid, size_t lds, hipStream_t st, const OutsArgs& a) {
  if (nw == 4) return go<outs_kernel<T, MT, 4>>(grid, 256, lds, st, a);
  return go<outs_kernel<T, MT, 2>>(grid, 128, lds, st, a);
}

}  // namespace

// Shapes this kernel takes (the caller has already chosen the output-stationary decomposition
// without slices, and the row split): 16-bit type, Br = 32, 64 or 128, vector-aligned A, an even
// number >= 4 of stages, more than one wave of columns, offsets that fit 32 bits.
bool outs_supported(const SketchParams& p, const void* A, int64_t lda, int64_t n, fs_dtype dt, int zsplit) {
  if (dt == FS_F32) return false;
  if (p.Br != 32 && p.Br != 64 && p.Br != 128) return false;
  if (p.kappa > (uint32_t)MAX_KAPPA || n <= WCOLS) return false;
  if ((uintptr_t)A % 8 || (lda * 2) % 8) return false;
  const int64_t spb = ((int64_t)p.Bc + KC - 1) / KC;
  const int64_t T = spb * p.kappa;
  if (T < 4 || T % 2) return false;
  if (zsplit < 1 || T % zsplit || (T / zsplit) % 2) return false;  // an even number of stages per work-group
  if ((16 * lda + n) * 2 >= ((int64_t)1 << 31)) return false;
  if (spb * KC * lda * 2 >= ((int64_t)1 << 31)) return false;
  const int nw = n > 2 * WCOLS ? 4 : 2;
  if ((n + WCOLS * nw - 1) / (WCOLS * nw) > 65535) return false;
  return true;
}

hipError_t launch_outs(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out, int64_t ldo,
                       fs_dtype dt, const uint32_t* orbit, int zsplit, float* ws, int64_t ldw, hipStream_t st,
                       EventPair ev, char* desc, size_t desc_cap) {
  OutsArgs a;
  a.p = p; a.A = A; a.out = out; a.pos2blk = orbit;
  a.lda = lda; a.ldo = ldo; a.n = (int)n;
  a.spb = (int)(((int64_t)p.Bc + KC - 1) / KC);
  a.out_vec = ((uintptr_t)out % 8 == 0 && (ldo * 2) % 8 == 0) ? 1 : 0;
  a.zsplit = zsplit; a.stages = (int)((int64_t)a.spb * p.kappa / zsplit); a.ws = ws; a.ldw = ldw;
  if (zsplit > 1 && (!ws || ldw % 4 || ldw < n)) return hipErrorInvalidValue;
  const int nw = n > 2 * WCOLS ? 4 : 2;
  const int mt = (int)p.Br / 32;
  const int tnw = WCOLS * nw;
  const unsigned col_tiles = (unsigned)((n + tnw - 1) / tnw);
  const size_t lds = 2 * MAX_KAPPA * 4 + 2 * (size_t)(32 * mt) * PHI_LD * 2;
  dim3 grid(p.M, col_tiles, zsplit);
  if (desc && desc_cap)
    snprintf(desc, desc_cap, "outs_kernel<%s,%d,%d>%s", dt == FS_BF16 ? "bf16" : "f16", mt, nw,
             zsplit > 1 ? "+reduce_planes" : "");
  if (ev.start) (void)hipEventRecord(ev.start, st);
  hipError_t e;
#define FS_T(T)                                                           \
  (mt == 4 ? launch_t<T, 4>(nw, grid, lds, st, a)                         \
   : mt == 2 ? launch_t<T, 2>(nw, grid, lds, st, a)                       \
             : launch_t<T, 1>(nw, grid, lds, st, a))
  if (dt == FS_BF16) e = FS_T(uint16_t); else e = FS_T(f16);
#undef FS_T
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  return e;
}

}  // namespace fs
