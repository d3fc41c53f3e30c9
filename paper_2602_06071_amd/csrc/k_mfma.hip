// BlockPerm-SJLT apply on the matrix cores (gfx950 MFMA).
//
// The s signed additions per input element of Alg. 1 cost kappa*s fp32 adds per
// element of A, which for 2-byte inputs exceeds what the vector ALUs can do at
// HBM speed.  Here a Br x Bc block Phi_{g,h} (entries 0, +1, -1) is instead
// treated as a dense bf16 matrix and Phi * A_tile is computed with
// v_mfma_f32_32x32x16_bf16 into fp32 accumulators: products with 0/+-1 are
// exact, so the result is the same sum in a different order.
//
//  * Phi is never stored in HBM: per 64-row stage of A, every wave hashes the
//    (block, row) pairs it needs (one lane per pair, Appendix E "Within-block
//    hashing"), scatters the s nonzeros of each into its own zeroed LDS tile
//    [stacked row][64 + 8 pad] and reads its MFMA operands from there with 128-bit
//    LDS reads.  Two tiles per wave alternate (consume / clear and refill); nothing is
//    shared between waves, so the steady state has no barrier.
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
//      IN-stationary, orbit runs (RUN = 4)  all kappa permutations are powers of one
//                      full-cycle map f (Appendix E), so in the order of f's orbit the
//                      input block at position q feeds the outputs at positions
//                      q-1..q-kappa.  A work-group takes RUN consecutive orbit
//                      positions (one pair of waves each), and before anything leaves
//                      the CU adds up, in LDS, the tiles that go to the same output:
//                      kappa+RUN-1 tiles leave instead of kappa*RUN, which cuts the
//                      partial-plane traffic by kappa*RUN/(kappa+RUN-1).
//
// Inputs must be finite: a dense product multiplies every element by the zeros of
// Phi as well, so an Inf/NaN in A spreads to all rows of the blocks that read it.
#include <stdio.h>

#include "k_mfma_kernel.h"

namespace fs {

// one per element type, each in a translation unit of its own
hipError_t launch_mfma_f32(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st);
hipError_t launch_mfma_bf16(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st);
hipError_t launch_mfma_f16(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st);
hipError_t launch_mfma_f32_unal(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st);
hipError_t launch_mfma_bf16_unal(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st);
hipError_t launch_mfma_f16_unal(const mm::Plan& pl, const mm::MfmaArgs& a, dim3 grid, hipStream_t st);

namespace {

using namespace mm;

// ---- host-side planning ----------------------------------------------------

constexpr size_t kLdsBudget = 160 * 1024;

bool tile_shape(uint32_t rw, int* mt, int* nrg) {
  if (rw == 32) { *mt = 1; *nrg = 1; return true; }
  if (rw == 64) { *mt = 2; *nrg = 1; return true; }
  if (rw == 128) { *mt = 4; *nrg = 1; return true; }
  return false;
}

// tables, then the larger of (two Phi tiles per wave) and (the orbit-run merge buffer)
size_t lds_bytes(int mt, int nrg, int ncg, int run, size_t merge) {
  const size_t tables = (size_t)run * 2 * MAX_KAPPA * 4;
  const size_t tiles = (size_t)run * nrg * ncg * 2 * (size_t)(32 * mt) * PHI_LD * 2;
  return tables + (tiles > merge ? tiles : merge);
}

Plan make_plan(const SketchParams& p, const void* A, int64_t lda, int64_t n, fs_dtype dt,
               bool have_orbit) {
  Plan pl;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  if (n < 1) return pl;
  // Br not a power of two: input-stationary only, a slot padded to the next power of two rows
  uint32_t brp = 1;
  while (brp < p.Br) brp <<= 1;
  if (!p.br_pow2 && brp > 128) return pl;
  const int64_t blk_stages = ((int64_t)p.Bc + KC - 1) / KC;  // the last one may be partly filled
  if ((uintptr_t)A % esz) return pl;
  pl.unal = (uintptr_t)A % (4 * esz) || (lda * esz) % (4 * esz);  // no 4-column vector loads
  if ((16 * lda + n) * (int64_t)esz >= ((int64_t)1 << 31)) return pl;     // 32-bit lane offsets
  if (blk_stages * KC * lda * (int64_t)esz >= ((int64_t)1 << 31)) return pl;  // 32-bit row offsets in a block
  pl.ncg = n > WCOLS ? 2 : 1;
  const int64_t col_tiles = (n + WCOLS * pl.ncg - 1) / (WCOLS * pl.ncg);
  if (col_tiles > 65535) return pl;

  int mt_i = 0, nrg_i = 0, mt_o = 0, nrg_o = 0;
  // IN: the kappa*Br stacked rows sit in the smallest tile that holds them (rows above them idle)
  const uint64_t rw = (uint64_t)p.kappa * brp;
  // OUT: blocks of 32, 64 or 128 rows, or 128-row slices of a higher (power-of-two) block
  const int nsub = p.Br > 128 ? (int)(p.Br / 128) : 1;
  // (its slot tables hold all kappa neighbours: at most MAX_KAPPA; the IN modes table one group)
  const bool can_out = p.br_pow2 && p.kappa <= (uint32_t)MAX_KAPPA &&
                       tile_shape(p.Br > 128 ? 128 : p.Br, &mt_o, &nrg_o);
  // More stacked rows than the highest tile and blocks too small for OUT (or not a power of two):
  // groups of 128/Br slots, each a work-group of its own that reads the input block again.
  const bool grouped = rw > 128 && !can_out && brp <= 64;
  const bool can_in = (rw <= 128 || grouped) && tile_shape(rw <= 32 ? 32 : rw <= 64 ? 64 : 128, &mt_i, &nrg_i);
  if (!can_in && !can_out) return pl;
  const int group_slots = grouped ? (int)(128 / brp) : (int)p.kappa;
  const int groups = (int)((p.kappa + group_slots - 1) / group_slots);

  // IN-stationary row split: more work-groups fill the chip better, but every split adds kappa
  // partial planes.  Pick the split with the smallest modelled time: A streamed at ~6 TB/s once
  // there is a wave per SIMD (1024 of them), planes written at ~3.4 TB/s and read back at ~6 TB/s
  // (rates measured on this kernel pair).
  int zs = 1;
  {
    const double a_bytes = (double)p.d * (double)n * esz * groups;
    const double waves_per_wg = pl.ncg * (can_in ? nrg_i : 1);
    double best = 0;
    for (int zc = 1; zc <= 16; zc *= 2) {
      if (zc > 1 && p.Bc % (uint32_t)(zc * KC) != 0) break;  // splits are whole stages
      const double waves = (double)p.M * col_tiles * zc * waves_per_wg * groups;
      const double plane_bytes = (double)zc * p.kappa * (double)p.k * (double)n * 4.0;
      const double t = a_bytes / (6e12 * (waves < 1024 ? waves / 1024 : 1.0)) + plane_bytes / 3.4e12 +
                       plane_bytes / 6e12;
      if (zc == 1 || t < best) { best = t; zs = zc; }
    }
  }
  // workspace traffic (write + read of the partial planes) relative to reading A once
  const double rho = 2.0 * zs * p.kappa * (double)p.k * 4.0 / ((double)p.d * esz);
  const bool out_starved = (int64_t)p.M * col_tiles < 256;  // fewer output tiles than CUs
  // IN pays for its partial planes (rho, written at about half the read rate), OUT for kappa-1
  // re-reads of A that mostly hit L2 (about 0.3 of an HBM read each): measured cross-over
  // rho ~ 0.23 (kappa - 1).  With kappa = 1 there is nothing to re-read and OUT stores directly.
  pl.in_stat = can_in && (!can_out || (p.kappa > 1 && (out_starved || rho <= 0.23 * (p.kappa - 1))));
  if (pl.in_stat) {
    pl.mt = mt_i; pl.nrg = nrg_i; pl.zsplit = zs;
    pl.stages = (int)(blk_stages / zs);
    pl.ldw = (n + 3) & ~(int64_t)3;
    pl.planes = zs * (int)p.kappa;
    pl.groups = groups; pl.group_slots = group_slots;
    if (zs * groups > 65535) return pl;
    // orbit runs of 4: the 64-row / 256-column shape, enough blocks for one work-group
    // per CU, and a merge buffer that fits beside nothing else in LDS
    constexpr int R = 4;
    const size_t merge = (size_t)(p.kappa + R - 1) * p.Br * (WCOLS * 2) * 4;
    if (have_orbit && p.br_pow2 && !pl.unal && zs == 1 && rw == 64 && pl.nrg == 1 && pl.ncg == 2 && p.kappa > 1 &&
        p.M % R == 0 && (int64_t)(p.M / R) * col_tiles >= 256 && merge <= 100 * 1024) {
      pl.run = R;
      pl.planes = (int)((p.kappa + R - 2) / R) + 1;
    }
  } else {
    // split the kappa*Bc rows of a work-group over grid.z when there are too few output tiles to
    // fill the chip (small n), as long as the extra plane traffic stays below that of reading A
    const int total_stages = (int)((int64_t)p.kappa * blk_stages);
    int zo = 1;
    // 16-bit shapes of the kernel with work-group-shared Phi tiles: its work-groups cover 512
    // columns and hold a CU each, so it wants a row split that brings their number to between
    // five eighths of the CUs and all of them (measured on wide: n = 2560 and 3072 whole, 0.20 ms
    // against 0.25 and 0.26 ms split; n = 1536 in 2 splits, n = 1024 in 4)
    const int64_t shared_wgs = (int64_t)p.M * ((n + 511) / 512);
    const bool shared_phi = nsub == 1 && !pl.unal && outs_supported(p, A, lda, n, dt, 1);
    auto enough = [&](int z) {
      return shared_phi ? shared_wgs * z >= 160 : (int64_t)p.M * col_tiles * nsub * z >= 512;
    };
    // (the split must divide the stages; the shared-Phi kernel wants an even number per work-group)
    while (!enough(zo) && zo < 8 && total_stages % (zo * 2 * (shared_phi ? 2 : 1)) == 0 &&
           2.0 * (zo * 2) * (double)p.k * 4.0 / ((double)p.d * esz) <= 1.0)
      zo *= 2;
    pl.mt = mt_o; pl.nrg = nrg_o; pl.zsplit = zo; pl.nsub = nsub;
    if (col_tiles * nsub > 65535) return pl;
    pl.stages = total_stages / zo;
    if (zo > 1) { pl.ldw = (n + 3) & ~(int64_t)3; pl.planes = zo; }
  }
  // bf16 with one wave per SIMD (128-row tiles) has the registers for a ring twice as deep, and
  // with a single wave nothing else hides the latency of A; the two-stage ring needs an even
  // stage count.  (For fp32 the deeper ring measured no gain.)
  if (pl.mt == 4 && dt != FS_F32 && pl.stages % 2 == 0 && !pl.unal) pl.pfx = 2;
  // 16-bit output-stationary shapes without row splits or slices go to the kernel whose work-group
  // shares its Phi tiles (measured on the "wide" workload: 0.445 against 0.52 ms)
  pl.outs = !pl.in_stat && pl.nsub == 1 && !pl.unal && outs_supported(p, A, lda, n, dt, pl.zsplit);
  // Shapes the kernel with several output blocks per wave takes go there (it loads A from L2
  // (kappa+S-1)/S times per output block, not kappa times; measured on "mid": kappa = 4, 0.365
  // against 0.395 ms, kappa = 8, 0.63 against 0.74 ms).  It stores the result itself.
  if (stacked_supported(p, A, lda, n, dt, have_orbit)) {
    pl.stacked = true; pl.unal = false; pl.outs = false; pl.in_stat = false; pl.run = 1; pl.planes = 0;
    pl.zsplit = 1; pl.nsub = 1; pl.groups = 1;
  }
  pl.lds = lds_bytes(pl.mt, pl.nrg, pl.ncg, pl.run,
                     pl.run > 1 ? (size_t)(p.kappa + pl.run - 1) * p.Br * 256 * 4 : 0);
  pl.ok = pl.stacked || pl.lds <= kLdsBudget;
  return pl;
}

}  // namespace

bool mfma_supported(const SketchParams& p, const void* A, int64_t lda, int64_t n, const void* out,
                    int64_t ldo, fs_dtype dt) {
  (void)out; (void)ldo;
  return make_plan(p, A, lda, n, dt, false).ok;
}

bool mfma_describe(const SketchParams& p, const void* A, int64_t lda, int64_t n, fs_dtype dt,
                   bool have_orbit, int* mode, int* flags, size_t* workspace) {
  const Plan pl = make_plan(p, A, lda, n, dt, have_orbit);
  if (!pl.ok) return false;
  *mode = !pl.in_stat ? 1 : pl.run > 1 ? 3 : 2;
  *flags = (pl.unal ? FS_PLAN_ELEMENT_LOADS : 0) | (pl.nsub > 1 ? FS_PLAN_ROW_SLICES : 0) |
           (pl.groups > 1 ? FS_PLAN_SLOT_GROUPS : 0) | (pl.zsplit > 1 ? FS_PLAN_SPLIT : 0) |
           (pl.stacked ? FS_PLAN_STACKED : 0);
  *workspace = (size_t)pl.planes * (size_t)p.k * (size_t)pl.ldw * sizeof(float);
  return true;
}

bool mfma_wants_orbit(const SketchParams& p) {
  return p.M >= 4 && p.M <= (1u << 20);
}

size_t mfma_workspace_bytes(const SketchParams& p, int64_t n, fs_dtype dt) {
  // sized without the orbit-run saving, so it holds for either mode
  const int64_t ld = (n + 7) & ~(int64_t)7;
  const Plan pl = make_plan(p, (const void*)(uintptr_t)256, ld, n, dt, false);
  if (!pl.ok || pl.planes == 0) return 0;
  return (size_t)pl.planes * (size_t)p.k * (size_t)pl.ldw * sizeof(float);
}

// The fixed-order sum of the partial planes into the output, scaled and converted.
static hipError_t launch_reduce(const SketchParams& p, const Plan& pl, int64_t n, void* out, int64_t ldo,
                                fs_dtype dt, float* ws, const uint32_t* orbit, hipStream_t st) {
  const size_t esz = dt == FS_F32 ? 4 : 2;
  const int out_vec = ((uintptr_t)out % (4 * esz) == 0 && (ldo * esz) % (4 * esz) == 0) ? 1 : 0;
  const int64_t work = p.k * (pl.ldw / 4);
  const unsigned blocks = (unsigned)((work + 255) / 256);
  const uint32_t* blk2pos = orbit ? orbit + p.M : nullptr;
  if (dt == FS_BF16)
    hipLaunchKernelGGL(reduce_planes_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, ws, pl.planes,
                       p.k, pl.ldw, (int)n, (uint16_t*)out, ldo, p.scale, out_vec, pl.run, blk2pos,
                       p.Br, p.kappa);
  else if (dt == FS_F16)
    hipLaunchKernelGGL(reduce_planes_kernel<f16>, dim3(blocks), dim3(256), 0, st, ws, pl.planes,
                       p.k, pl.ldw, (int)n, (f16*)out, ldo, p.scale, out_vec, pl.run, blk2pos,
                       p.Br, p.kappa);
  else
    hipLaunchKernelGGL(reduce_planes_kernel<float>, dim3(blocks), dim3(256), 0, st, ws, pl.planes,
                       p.k, pl.ldw, (int)n, (float*)out, ldo, p.scale, out_vec, pl.run, blk2pos,
                       p.Br, p.kappa);
  return hipGetLastError();
}

hipError_t launch_mfma(const SketchParams& p, const void* A, int64_t lda, int64_t n, void* out,
                       int64_t ldo, fs_dtype dt, void* ws, const uint32_t* orbit, hipStream_t st,
                       EventPair ev, int* mode, char* desc, size_t desc_cap) {
  const Plan pl = make_plan(p, A, lda, n, dt, orbit != nullptr);
  if (!pl.ok) return hipErrorInvalidValue;
  *mode = !pl.in_stat ? 1 : pl.run > 1 ? 3 : 2;
  if (pl.stacked) return launch_stacked(p, A, lda, n, out, ldo, dt, orbit, st, ev, desc, desc_cap);
  hipError_t e;
  if (pl.outs) {
    e = launch_outs(p, A, lda, n, out, ldo, dt, orbit, pl.zsplit, (float*)ws, pl.ldw, st, ev, desc, desc_cap);
    if (e != hipSuccess || pl.planes == 0) return e;
    return launch_reduce(p, pl, n, out, ldo, dt, (float*)ws, orbit, st);
  }
  if (desc && desc_cap)  // the template arguments of the instantiation launched below, in order
    snprintf(desc, desc_cap, "mfma_kernel<%s,%d,%d,%d,%s,%d,%d,%d,%s,%s>%s",
             dt == FS_F32 ? "f32" : dt == FS_BF16 ? "bf16" : "f16", pl.mt, pl.nrg, pl.ncg,
             pl.in_stat ? "in" : "out", pl.run, pl.cpl, pl.unal ? 1 : pl.pfx, pl.nsub > 1 ? "sub" : "-",
             pl.unal ? "unal" : "-", pl.planes ? "+reduce_planes" : "");
  const size_t esz = dt == FS_F32 ? 4 : 2;
  MfmaArgs a;
  a.p = p; a.A = A; a.out = out; a.ws = (float*)ws;
  a.pos2blk = orbit;
  a.lda = lda; a.ldo = ldo; a.ldw = pl.ldw; a.n = (int)n;
  a.zsplit = pl.zsplit; a.stages = pl.stages;
  a.group_slots = pl.in_stat ? pl.group_slots : (int)p.kappa;
  a.nsub = pl.nsub;
  a.out_vec = ((uintptr_t)out % (4 * esz) == 0 && (ldo * esz) % (4 * esz) == 0) ? 1 : 0;
  a.log2_br = 0;
  while ((1u << a.log2_br) < p.Br) ++a.log2_br;
  const int tnw = 32 * pl.cpl * pl.ncg;
  const unsigned col_tiles = (unsigned)((n + tnw - 1) / tnw);
  dim3 grid(p.M / pl.run, col_tiles * pl.nsub, pl.zsplit * pl.groups);

  if (ev.start) (void)hipEventRecord(ev.start, st);
  if (dt == FS_BF16) e = pl.unal ? launch_mfma_bf16_unal(pl, a, grid, st) : launch_mfma_bf16(pl, a, grid, st);
  else if (dt == FS_F16) e = pl.unal ? launch_mfma_f16_unal(pl, a, grid, st) : launch_mfma_f16(pl, a, grid, st);
  else e = pl.unal ? launch_mfma_f32_unal(pl, a, grid, st) : launch_mfma_f32(pl, a, grid, st);
  if (ev.stop) (void)hipEventRecord(ev.stop, st);
  if (e != hipSuccess || pl.planes == 0) return e;

  return launch_reduce(p, pl, n, out, ldo, dt, a.ws, orbit, st);
}

}  // namespace fs
