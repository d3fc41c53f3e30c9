// C ABI of the library: argument checks, seed -> wiring derivation, variant
// dispatch and workspace management.  No arithmetic of the sketch apply itself
// lives here; it is all in the k_*.hip kernels.
#include <math.h>
#include <stdio.h>
#include <string.h>
#include <new>

#include "handle.h"
#include "spec.h"

fs_status fs::hip_fail(fs_sketch_t h, hipError_t e) {
  if (h) h->last_hip_error = (int)e;
  (void)hipGetLastError();  // clear the sticky launch error
  return FS_ERR_HIP;
}

namespace {

using fs::hip_fail;

uint32_t radical(uint32_t m) {
  uint32_t r = 1;
  for (uint32_t p = 2; (uint64_t)p * p <= m; ++p) {
    if (m % p == 0) {
      r *= p;
      while (m % p == 0) m /= p;
    }
  }
  if (m > 1) r *= m;
  return r;
}

uint32_t lcm_u32(uint32_t x, uint32_t y) { return x / fs::gcd_u32(x, y) * y; }

// inverse of a modulo M by the extended Euclidean algorithm (gcd(a, M) = 1)
uint32_t mod_inverse(uint32_t a, uint32_t M) {
  int64_t t = 0, nt = 1, r = M, nr = a % M;
  while (nr != 0) {
    int64_t q = r / nr;
    int64_t tmp = t - q * nt; t = nt; nt = tmp;
    tmp = r - q * nr; r = nr; nr = tmp;
  }
  if (t < 0) t += M;
  return (uint32_t)t;
}

// Appendix E, "Full-cycle affine construction": b coprime to M, a - 1 divisible by
// every prime of M and by 4 when 4 | M.  (a, b) are drawn from the seed keys.
void derive_wiring(uint32_t M, uint32_t key1, uint32_t* a, uint32_t* b, uint32_t* a_inv) {
  if (M == 1) { *a = 0; *b = 0; *a_inv = 0; return; }
  const uint32_t L = lcm_u32(radical(M), (M % 4 == 0) ? 4u : 1u);
  const uint32_t ha = fs::mix32(key1 ^ 1u), hb = fs::mix32(key1 ^ 2u);
  *a = (uint32_t)((1u + (uint64_t)L * (ha % (M / L))) % M);
  uint32_t bb = hb % M;
  while (fs::gcd_u32(bb, M) != 1u) bb = (bb + 1u) % M;
  *b = bb;
  *a_inv = mod_inverse(*a, M);
}

bool is_pow2(uint32_t x) { return x && !(x & (x - 1)); }

bool valid_dtype(fs_dtype dt) { return dt == FS_F32 || dt == FS_BF16 || dt == FS_F16; }

// Bytes of workspace the variant that would run needs.  exact_orbit < 0: an upper bound that
// holds whether or not the orbit table will be there; 0 / 1: the size of exactly this call,
// without / with the table.
fs_status needed_workspace(fs_sketch_t h, const void* A, int64_t lda, int64_t n, const void* out,
                           int64_t ldo, fs_dtype dt, int* variant_out, size_t* bytes, int exact_orbit = -1) {
  *bytes = 0;
  *variant_out = FS_VARIANT_GENERIC;
  if (h->kind == FS_KIND_SJLT_SCATTER) {
    *bytes = fs::scatter_workspace_bytes(h->p, n, dt);
    return FS_OK;
  }
  if (h->kind == FS_KIND_GAUSS_DENSE)
    return fs::gauss_supported(h->p.k, h->p.d, A, lda, n, dt) ? FS_OK : FS_ERR_UNSUPPORTED;
  if (h->kind == FS_KIND_BLOCKROW) return FS_OK;
  const bool can = fs::mfma_supported(h->p, A, lda, n, out, ldo, dt);
  int v = h->variant;
  if (v == FS_VARIANT_AUTO) v = can ? FS_VARIANT_MFMA : FS_VARIANT_GENERIC;
  if (v == FS_VARIANT_MFMA) {
    if (!can) return FS_ERR_UNSUPPORTED;
    *bytes = fs::mfma_workspace_bytes(h->p, n, dt);
    if (exact_orbit >= 0) {
      int mode = 0, flags = 0;
      if (!fs::mfma_describe(h->p, A, lda, n, dt, exact_orbit != 0, &mode, &flags, bytes)) return FS_ERR_UNSUPPORTED;
    }
  }
  *variant_out = v;
  return FS_OK;
}

fs_status ensure_workspace(fs_sketch_t h, size_t need) {
  if (need <= h->ws_bytes) return FS_OK;
  if (h->ws && !h->ws_owned) return FS_ERR_ALLOC;  // caller-owned and too small
  if (h->ws) {
    hipError_t e = hipFree(h->ws);  // waits for work that may still use it
    h->ws = nullptr; h->ws_bytes = 0;
    if (e != hipSuccess) return hip_fail(h, e);
  }
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, need);
  if (e != hipSuccess) { hip_fail(h, e); return FS_ERR_ALLOC; }
  h->ws = p; h->ws_bytes = need; h->ws_owned = true;
  return FS_OK;
}

// pos2blk[q] = f^q(0), blk2pos = its inverse: allocated once per handle and filled by a small
// kernel enqueued on `st` (no copy, no synchronisation).
fs_status ensure_orbit(fs_sketch_t h, hipStream_t st) {
  if (h->orbit || !fs::mfma_wants_orbit(h->p)) return FS_OK;
  void* dev = nullptr;
  hipError_t e = hipMalloc(&dev, 2 * (size_t)h->p.M * sizeof(uint32_t));
  if (e != hipSuccess) { hip_fail(h, e); return FS_ERR_ALLOC; }
  e = fs::launch_orbit(h->p, (uint32_t*)dev, st);
  if (e != hipSuccess) { (void)hipFree(dev); return hip_fail(h, e); }
  h->orbit = (uint32_t*)dev;
  return FS_OK;
}

// The next unused set of profiling events (all null when not profiling).  `begin` is recorded
// here, before anything the apply enqueues; the caller records `end` after its last launch.
struct ProfSet {
  fs::EventPair kernel;
  hipEvent_t end = nullptr;
};
ProfSet next_events(fs_sketch_t h, hipStream_t st) {
  ProfSet ps;
  if (h->profiling && h->prof_used < (int)h->prof_begin.size()) {
    const int i = h->prof_used++;
    if (h->prof_scope & FS_PROFILE_KERNEL) {
      ps.kernel.start = h->prof_start[i];
      ps.kernel.stop = h->prof_stop[i];
    }
    if (h->prof_scope & FS_PROFILE_APPLY) {
      ps.end = h->prof_end[i];
      (void)hipEventRecord(h->prof_begin[i], st);
    }
  }
  return ps;
}

}  // namespace

extern "C" {

const char* fs_status_string(fs_status st) {
  switch (st) {
    case FS_OK: return "ok";
    case FS_ERR_INVALID_ARG: return "invalid argument";
    case FS_ERR_UNSUPPORTED: return "unsupported shape or variant";
    case FS_ERR_ALLOC: return "allocation failed or workspace too small";
    case FS_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

fs_status fs_sketch_create_kind(fs_sketch_t* out, fs_kind kind, int64_t d, int64_t k, int32_t Bc,
                                int32_t Br, int32_t kappa, int32_t s, uint64_t seed) {
  if (!out) return FS_ERR_INVALID_ARG;
  *out = nullptr;
  if (kind != FS_KIND_BLOCKPERM && kind != FS_KIND_SJLT_SCATTER && kind != FS_KIND_GAUSS_DENSE &&
      kind != FS_KIND_BLOCKROW)
    return FS_ERR_INVALID_ARG;
  if (d < 1 || k < 1 || d > ((int64_t)1 << 40) || k > ((int64_t)1 << 31)) return FS_ERR_INVALID_ARG;
  if (kind == FS_KIND_GAUSS_DENSE) { Bc = (int32_t)(d > 0x7fffffff ? 0x7fffffff : d); Br = 1; kappa = 1; s = 1; }
  if (kind != FS_KIND_GAUSS_DENSE) {
    if (Bc < 1 || Br < 1 || kappa < 1 || s < 1) return FS_ERR_INVALID_ARG;
    // the block grid is square: M = k/Br = ceil(d/Bc); a last input block that is only partly
    // filled is treated as zero-padded (Section 4, "general cases ... by padding")
    if (k % Br || (d + Bc - 1) / Bc != k / Br) return FS_ERR_INVALID_ARG;
    const int64_t M = k / Br;
    if (M > (1 << 24) || kappa > M) return FS_ERR_INVALID_ARG;
    if (s > Br || s > 32 || Br > 65536) return FS_ERR_INVALID_ARG;
    // (the scatter kernel walks exactly Bc rows of A: a padded block, Bc > d, is not accepted)
    if (kind == FS_KIND_SJLT_SCATTER && (M != 1 || kappa != 1 || Bc != d)) return FS_ERR_INVALID_ARG;
  }
  fs_sketch_s* h = new (std::nothrow) fs_sketch_s();
  if (!h) return FS_ERR_ALLOC;
  SketchParams& p = h->p;
  p.d = d; p.k = k;
  p.Bc = (uint32_t)Bc; p.Br = (uint32_t)Br; p.kappa = (uint32_t)kappa; p.s = (uint32_t)s;
  p.M = kind == FS_KIND_GAUSS_DENSE ? 1u : (uint32_t)(k / Br);
  h->key0 = fs::mix32((uint32_t)(seed & 0xFFFFFFFFu) ^ fs::kC1);
  p.key1 = fs::mix32((uint32_t)(seed >> 32) ^ h->key0 ^ fs::kC2);
  derive_wiring(p.M, p.key1, &p.a, &p.b, &p.a_inv);
  p.br_pow2 = is_pow2(p.Br) ? 1u : 0u;
  p.scale = kind == FS_KIND_GAUSS_DENSE ? (float)(1.0 / sqrt((double)k))
            : kind == FS_KIND_BLOCKROW  ? (float)(sqrt((double)d / (double)k) / sqrt((double)kappa * (double)s))
                                        : (float)(1.0 / sqrt((double)kappa * (double)s));
  h->kind = (int)kind;
  h->variant = FS_VARIANT_AUTO;
  h->last_variant = 0;
  h->last_mode = 0;
  h->last_hip_error = 0;
  h->last_kernel[0] = 0;
  h->device = -1;
  h->ws = nullptr; h->ws_bytes = 0; h->ws_owned = true;
  h->dense = nullptr;
  h->profiling = false; h->prof_used = 0; h->prof_scope = 0;
  h->orbit = nullptr;

  if (kind == FS_KIND_GAUSS_DENSE) {
    if ((double)k * (double)d > 2.0e9) { delete h; return FS_ERR_UNSUPPORTED; }
    hipError_t e = hipMalloc(&h->dense, fs::gauss_bytes(k, d));
    if (e == hipSuccess) e = fs::gauss_fill(h->dense, k, d, p.key1, nullptr);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (h->dense) (void)hipFree(h->dense);
      const bool oom = (e == hipErrorOutOfMemory);
      delete h;
      return oom ? FS_ERR_ALLOC : FS_ERR_HIP;
    }
  }
  *out = h;
  return FS_OK;
}

fs_status fs_sketch_create(fs_sketch_t* out, int64_t d, int64_t k, int32_t Bc, int32_t Br,
                           int32_t kappa, int32_t s, uint64_t seed) {
  return fs_sketch_create_kind(out, FS_KIND_BLOCKPERM, d, k, Bc, Br, kappa, s, seed);
}

static void release_events(fs_sketch_t h) {
  for (auto* v : {&h->prof_begin, &h->prof_start, &h->prof_stop, &h->prof_end}) {
    for (hipEvent_t e : *v) (void)hipEventDestroy(e);
    v->clear();
  }
  h->profiling = false; h->prof_used = 0;
}

fs_status fs_sketch_profile_begin(fs_sketch_t h, int32_t max_launches, int32_t scope) {
  if (!h || max_launches < 1 || max_launches > (1 << 20) || h->profiling) return FS_ERR_INVALID_ARG;
  if (scope < 1 || scope > (FS_PROFILE_KERNEL | FS_PROFILE_APPLY)) return FS_ERR_INVALID_ARG;
  h->prof_scope = scope;
  for (int i = 0; i < max_launches; ++i) {
    for (auto* v : {&h->prof_begin, &h->prof_start, &h->prof_stop, &h->prof_end}) {
      hipEvent_t ev = nullptr;
      const hipError_t e = hipEventCreate(&ev);
      if (e != hipSuccess) {
        release_events(h);
        return hip_fail(h, e);
      }
      v->push_back(ev);
    }
  }
  h->profiling = true; h->prof_used = 0;
  return FS_OK;
}

fs_status fs_sketch_profile_end(fs_sketch_t h, float* ms, float* ms_apply, int32_t* count) {
  if (!h || !ms || !count || !h->profiling) return FS_ERR_INVALID_ARG;
  fs_status rc = FS_OK;
  *count = h->prof_used;
  const bool k = h->prof_scope & FS_PROFILE_KERNEL, a = h->prof_scope & FS_PROFILE_APPLY;
  for (int i = 0; i < h->prof_used; ++i) {
    hipError_t e = hipEventSynchronize(a ? h->prof_end[i] : h->prof_stop[i]);
    ms[i] = 0.f;
    if (ms_apply) ms_apply[i] = 0.f;
    if (e == hipSuccess && k) e = hipEventElapsedTime(&ms[i], h->prof_start[i], h->prof_stop[i]);
    if (e == hipSuccess && a && ms_apply) e = hipEventElapsedTime(&ms_apply[i], h->prof_begin[i], h->prof_end[i]);
    if (e != hipSuccess) { rc = hip_fail(h, e); *count = i; break; }
  }
  release_events(h);
  return rc;
}

fs_status fs_sketch_destroy(fs_sketch_t h) {
  if (!h) return FS_ERR_INVALID_ARG;
  fs_status st = FS_OK;
  release_events(h);
  if (h->ws && h->ws_owned && hipFree(h->ws) != hipSuccess) st = FS_ERR_HIP;
  if (h->orbit && hipFree(h->orbit) != hipSuccess) st = FS_ERR_HIP;
  if (h->dense && hipFree(h->dense) != hipSuccess) st = FS_ERR_HIP;
  if (st != FS_OK) (void)hipGetLastError();
  delete h;
  return st;
}

fs_status fs_sketch_info(fs_sketch_t h, fs_info* o) {
  if (!h || !o) return FS_ERR_INVALID_ARG;
  const SketchParams& p = h->p;
  o->d = p.d; o->k = p.k;
  o->Bc = (int32_t)p.Bc; o->Br = (int32_t)p.Br; o->kappa = (int32_t)p.kappa; o->s = (int32_t)p.s;
  o->M = (int32_t)p.M; o->a = (int32_t)p.a; o->b = (int32_t)p.b; o->a_inv = (int32_t)p.a_inv;
  o->key0 = h->key0; o->key1 = p.key1;
  o->scale = p.scale;
  o->kind = h->kind; o->variant = h->variant; o->last_variant = h->last_variant; o->last_mode = h->last_mode;
  o->last_hip_error = h->last_hip_error;
  o->workspace_bytes = h->ws_bytes;
  memcpy(o->last_kernel, h->last_kernel, sizeof(o->last_kernel));
  return FS_OK;
}

fs_status fs_sketch_set_variant(fs_sketch_t h, fs_variant v) {
  if (!h) return FS_ERR_INVALID_ARG;
  if (v != FS_VARIANT_AUTO && v != FS_VARIANT_GENERIC && v != FS_VARIANT_MFMA)
    return FS_ERR_INVALID_ARG;
  h->variant = (int)v;
  return FS_OK;
}

fs_status fs_sketch_workspace_bytes(fs_sketch_t h, int64_t n, fs_dtype dt, size_t* bytes) {
  if (!h || !bytes || n < 0 || !valid_dtype(dt)) return FS_ERR_INVALID_ARG;
  *bytes = 0;
  if (n == 0) return FS_OK;
  // Size for the best case of a well-aligned call: an aligned dummy pointer
  // and packed leading dimensions rounded up to 16 bytes.
  const int64_t ld = (n + 7) & ~(int64_t)7;
  int v;
  const void* aligned = (const void*)(uintptr_t)256;
  fs_status st = needed_workspace(h, aligned, ld, n, aligned, ld, dt, &v, bytes);
  if (st == FS_ERR_UNSUPPORTED) { *bytes = 0; return FS_OK; }
  return st;
}

fs_status fs_sketch_set_workspace(fs_sketch_t h, void* dev_ptr, size_t bytes) {
  if (!h) return FS_ERR_INVALID_ARG;
  if ((dev_ptr == nullptr) != (bytes == 0)) return FS_ERR_INVALID_ARG;
  if ((uintptr_t)dev_ptr % 256) return FS_ERR_INVALID_ARG;
  if (h->ws && h->ws_owned) {
    hipError_t e = hipFree(h->ws);
    h->ws = nullptr; h->ws_bytes = 0;
    if (e != hipSuccess) return hip_fail(h, e);
  }
  h->ws = dev_ptr; h->ws_bytes = bytes; h->ws_owned = (dev_ptr == nullptr);
  return FS_OK;
}

}  // extern "C"

// The apply of the column layout (declared in handle.h).
fs_status fs::apply_cols(fs_sketch_t h, const void* A, int64_t lda, int64_t n, void* out, int64_t ldo,
                         fs_dtype dt, void* stream, const fs::ScratchSource& src) {
  if (!h || n < 0 || !valid_dtype(dt)) return FS_ERR_INVALID_ARG;
  if (n == 0) return FS_OK;
  if (!A || !out || lda < n || ldo < n) return FS_ERR_INVALID_ARG;
  if (n > 0x7fffffff || lda > ((int64_t)1 << 40) || ldo > ((int64_t)1 << 40)) return FS_ERR_INVALID_ARG;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  if ((uintptr_t)A % esz || (uintptr_t)out % esz) return FS_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;

  // whether the kernels will get the orbit table of the wiring (it shapes their plan)
  const bool with_orbit = h->kind == FS_KIND_BLOCKPERM && fs::mfma_wants_orbit(h->p) &&
                          (!src.external || 2 * (size_t)h->p.M * sizeof(uint32_t) <= src.orbit_bytes);
  int variant;
  size_t need;
  fs_status rc = needed_workspace(h, A, lda, n, out, ldo, dt, &variant, &need, with_orbit ? 1 : 0);
  if (rc != FS_OK) return rc;
  void* ws = nullptr;
  const uint32_t* orbit = nullptr;
  if (src.external && need > src.plane_bytes) return FS_ERR_ALLOC;  // beyond the supplied memory: nothing is launched
  if (!src.external) {
    rc = ensure_workspace(h, need);
    if (rc != FS_OK) return rc;
  }
  const ProfSet prof = next_events(h, st);
  const fs::EventPair ev = prof.kernel;
  if (src.external) {
    ws = src.planes;
    // such memory is shared between handles: the table of this handle's wiring is rebuilt on every
    // call (a wiring too long for the table's room runs without one: the kernels then skip the
    // orbit-ordered modes)
    if (variant == FS_VARIANT_MFMA && with_orbit) {
      const hipError_t e = fs::launch_orbit(h->p, src.orbit, st);
      if (e != hipSuccess) return hip_fail(h, e);
      orbit = src.orbit;
    }
  } else {
    if (variant == FS_VARIANT_MFMA) {
      rc = ensure_orbit(h, st);
      if (rc != FS_OK) return rc;
    }
    ws = h->ws;
    orbit = h->orbit;
  }

  hipError_t e;
  int mode = 0;
  const char* what = "";
  if (h->kind == FS_KIND_SJLT_SCATTER) {
    e = fs::launch_scatter(h->p, A, lda, n, out, ldo, dt, ws, st, ev);
    what = "scatter_kernel";
  } else if (h->kind == FS_KIND_GAUSS_DENSE) {
    e = fs::launch_gauss(h->dense, h->p.k, h->p.d, A, lda, n, out, ldo, dt, st, ev);
    what = "gauss_kernel";
  } else if (h->kind == FS_KIND_BLOCKROW) {
    e = fs::launch_blockrow(h->p, A, lda, n, out, ldo, dt, st, ev);
    what = "blockrow_kernel";
  } else if (variant == FS_VARIANT_MFMA) {
    e = fs::launch_mfma(h->p, A, lda, n, out, ldo, dt, ws, orbit, st, ev, &mode, h->last_kernel,
                        sizeof(h->last_kernel));
  } else {
    e = fs::launch_generic(h->p, A, lda, n, out, ldo, dt, st, ev);
    what = "generic_kernel";
  }
  if (what[0]) snprintf(h->last_kernel, sizeof(h->last_kernel), "%s", what);
  if (prof.end) (void)hipEventRecord(prof.end, st);
  h->last_variant = variant;
  h->last_mode = mode;
  if (e != hipSuccess) return hip_fail(h, e);
  return FS_OK;
}

extern "C" {

fs_status fs_sketch_apply_ld(fs_sketch_t h, const void* A, int64_t lda, int64_t n, void* out,
                             int64_t ldo, fs_dtype dt, void* stream) {
  return fs::apply_cols(h, A, lda, n, out, ldo, dt, stream, fs::ScratchSource{});
}

fs_status fs_sketch_prepare(fs_sketch_t h, void* stream) {
  if (!h) return FS_ERR_INVALID_ARG;
  if (h->kind != FS_KIND_BLOCKPERM) return FS_OK;
  return ensure_orbit(h, (hipStream_t)stream);
}

fs_status fs_sketch_apply_rows(fs_sketch_t h, const void* G, int64_t ldg, int64_t n, void* out,
                               int64_t ldo, fs_dtype dt, void* stream) {
  if (!h || n < 0 || !valid_dtype(dt)) return FS_ERR_INVALID_ARG;
  if (n == 0) return FS_OK;
  if (!G || !out || ldg < h->p.d || ldo < h->p.k) return FS_ERR_INVALID_ARG;
  if (n > 0x7fffffff || ldg > ((int64_t)1 << 40) || ldo > ((int64_t)1 << 40)) return FS_ERR_INVALID_ARG;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  if ((uintptr_t)G % esz || (uintptr_t)out % esz) return FS_ERR_INVALID_ARG;
  if (h->kind != FS_KIND_BLOCKPERM) return FS_ERR_UNSUPPORTED;
  const bool can = fs::rows_supported(h->p, G, ldg, n, dt);
  if (h->variant == FS_VARIANT_MFMA && !can) return FS_ERR_UNSUPPORTED;
  const bool use_mfma = can && h->variant != FS_VARIANT_GENERIC;
  hipStream_t st = (hipStream_t)stream;
  fs_status rc = use_mfma ? ensure_workspace(h, fs::rows_workspace_bytes(h->p, G, ldg, n, dt)) : FS_OK;
  if (rc != FS_OK) return rc;
  const ProfSet prof = next_events(h, st);
  const fs::EventPair ev = prof.kernel;
  if (!use_mfma) {
    const hipError_t e = fs::launch_generic_rows(h->p, G, ldg, n, out, ldo, dt, st, ev);
    if (prof.end) (void)hipEventRecord(prof.end, st);
    snprintf(h->last_kernel, sizeof(h->last_kernel), "generic_rows_kernel");
    h->last_variant = FS_VARIANT_GENERIC;
    h->last_mode = 0;
    if (e != hipSuccess) return hip_fail(h, e);
    return FS_OK;
  }
  rc = ensure_orbit(h, st);  // the gather-reduction walks the wiring through this table
  if (rc != FS_OK) return rc;
  const hipError_t e = fs::launch_rows(h->p, G, ldg, n, out, ldo, dt, h->ws, h->orbit, st, ev);
  if (prof.end) (void)hipEventRecord(prof.end, st);
  snprintf(h->last_kernel, sizeof(h->last_kernel), "rows_kernel");
  h->last_variant = FS_VARIANT_MFMA;
  h->last_mode = 2;
  if (e != hipSuccess) return hip_fail(h, e);
  return FS_OK;
}

fs_status fs_sketch_rows_workspace_bytes(fs_sketch_t h, int64_t n, fs_dtype dt, size_t* bytes) {
  if (!h || !bytes || n < 0 || !valid_dtype(dt)) return FS_ERR_INVALID_ARG;
  *bytes = 0;
  if (n == 0 || h->kind != FS_KIND_BLOCKPERM) return FS_OK;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  const int64_t ld = (h->p.d + 7) & ~(int64_t)7;  // a well-aligned call: packed rows rounded to 16 bytes
  if (34 * ld * (int64_t)esz >= ((int64_t)1 << 31)) return FS_OK;
  *bytes = fs::rows_workspace_bytes(h->p, (const void*)(uintptr_t)256, ld, n, dt);
  return FS_OK;
}

fs_status fs_sketch_plan(fs_sketch_t h, const void* A, int64_t ld, int64_t n, fs_dtype dt, int32_t rows,
                         int32_t* variant, int32_t* mode, int32_t* flags, size_t* workspace_bytes) {
  if (!h || n < 0 || !valid_dtype(dt) || (rows != 0 && rows != 1)) return FS_ERR_INVALID_ARG;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  if (!A || (uintptr_t)A % esz || ld < (rows ? h->p.d : n) || n > 0x7fffffff || ld > ((int64_t)1 << 40))
    return FS_ERR_INVALID_ARG;
  if (rows && h->kind != FS_KIND_BLOCKPERM) return FS_ERR_UNSUPPORTED;
  int v = FS_VARIANT_GENERIC, m = 0, f = 0;
  size_t ws = 0;
  if (n > 0 && h->kind == FS_KIND_BLOCKPERM) {
    int mm = 0, ff = 0;
    size_t w = 0;
    const bool can = rows ? fs::rows_describe(h->p, A, ld, n, dt, &mm, &ff, &w)
                          : fs::mfma_describe(h->p, A, ld, n, dt, fs::mfma_wants_orbit(h->p), &mm, &ff, &w);
    if (h->variant == FS_VARIANT_MFMA && !can) return FS_ERR_UNSUPPORTED;
    if (can && h->variant != FS_VARIANT_GENERIC) { v = FS_VARIANT_MFMA; m = mm; f = ff; ws = w; }
  } else if (n > 0) {
    int vv;
    const fs_status rc = needed_workspace(h, A, ld, n, A, n, dt, &vv, &ws);
    if (rc != FS_OK) return rc;
  }
  if (variant) *variant = v;
  if (mode) *mode = m;
  if (flags) *flags = f;
  if (workspace_bytes) *workspace_bytes = ws;
  return FS_OK;
}

fs_status fs_sketch_apply(fs_sketch_t h, const void* A, int64_t lda, int64_t n, void* out,
                          fs_dtype dt, void* stream) {
  return fs_sketch_apply_ld(h, A, lda, n, out, n, dt, stream);
}

fs_status fs_sketch_export(fs_sketch_t h, int32_t* rows, int8_t* signs, void* stream) {
  if (!h || !rows || !signs) return FS_ERR_INVALID_ARG;
  if (h->kind == FS_KIND_GAUSS_DENSE) return FS_ERR_UNSUPPORTED;
  hipError_t e = h->kind == FS_KIND_BLOCKROW
                     ? fs::launch_blockrow_export(h->p, rows, signs, (hipStream_t)stream)
                     : fs::launch_export(h->p, rows, signs, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(h, e);
  return FS_OK;
}

fs_status fs_sketch_export_dense(fs_sketch_t h, float* S_dense, void* stream) {
  if (!h || !S_dense) return FS_ERR_INVALID_ARG;
  if (h->kind != FS_KIND_GAUSS_DENSE) return FS_ERR_UNSUPPORTED;
  hipError_t e = hipMemcpyAsync(S_dense, h->dense, (size_t)h->p.k * h->p.d * sizeof(float),
                                hipMemcpyDeviceToDevice, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(h, e);
  return FS_OK;
}

}  // extern "C"
