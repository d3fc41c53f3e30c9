// C ABI of the library: argument checks, seed -> wiring derivation, variant
// dispatch and workspace management.  No arithmetic of the sketch apply itself
// lives here; it is all in the k_*.hip kernels.
#include <math.h>
#include <new>

#include "handle.h"
#include "spec.h"

namespace {

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

fs_status hip_fail(fs_sketch_t h, hipError_t e) {
  if (h) h->last_hip_error = (int)e;
  (void)hipGetLastError();  // clear the sticky launch error
  return FS_ERR_HIP;
}

// Bytes of workspace the variant that would run needs.
fs_status needed_workspace(fs_sketch_t h, const void* A, int64_t lda, int64_t n, const void* out,
                           int64_t ldo, fs_dtype dt, int* variant_out, size_t* bytes) {
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

// pos2blk[q] = f^q(0), blk2pos = its inverse; uploaded once per handle.
fs_status ensure_orbit(fs_sketch_t h) {
  if (h->orbit || !fs::mfma_wants_orbit(h->p)) return FS_OK;
  const uint32_t M = h->p.M;
  std::vector<uint32_t> tab(2 * (size_t)M);
  uint32_t x = 0;
  for (uint32_t q = 0; q < M; ++q) {
    tab[q] = x;
    tab[M + x] = q;
    x = fs::wire_next(x, h->p.a, h->p.b, M);
  }
  void* dev = nullptr;
  hipError_t e = hipMalloc(&dev, tab.size() * sizeof(uint32_t));
  if (e != hipSuccess) { hip_fail(h, e); return FS_ERR_ALLOC; }
  e = hipMemcpy(dev, tab.data(), tab.size() * sizeof(uint32_t), hipMemcpyHostToDevice);
  if (e != hipSuccess) { (void)hipFree(dev); return hip_fail(h, e); }
  h->orbit = (uint32_t*)dev;
  return FS_OK;
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
    if (kind == FS_KIND_SJLT_SCATTER && (M != 1 || kappa != 1)) return FS_ERR_INVALID_ARG;
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
  h->device = -1;
  h->ws = nullptr; h->ws_bytes = 0; h->ws_owned = true;
  h->dense = nullptr;
  h->profiling = false; h->prof_used = 0;
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
  for (hipEvent_t e : h->prof_start) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->prof_stop) (void)hipEventDestroy(e);
  h->prof_start.clear(); h->prof_stop.clear();
  h->profiling = false; h->prof_used = 0;
}

fs_status fs_sketch_profile_begin(fs_sketch_t h, int32_t max_launches) {
  if (!h || max_launches < 1 || max_launches > (1 << 20) || h->profiling) return FS_ERR_INVALID_ARG;
  for (int i = 0; i < max_launches; ++i) {
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t e = hipEventCreate(&a);
    if (e == hipSuccess) e = hipEventCreate(&b);
    if (e != hipSuccess) {
      if (a) (void)hipEventDestroy(a);
      release_events(h);
      return hip_fail(h, e);
    }
    h->prof_start.push_back(a); h->prof_stop.push_back(b);
  }
  h->profiling = true; h->prof_used = 0;
  return FS_OK;
}

fs_status fs_sketch_profile_end(fs_sketch_t h, float* ms, int32_t* count) {
  if (!h || !ms || !count || !h->profiling) return FS_ERR_INVALID_ARG;
  fs_status rc = FS_OK;
  *count = h->prof_used;
  for (int i = 0; i < h->prof_used; ++i) {
    hipError_t e = hipEventSynchronize(h->prof_stop[i]);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms[i], h->prof_start[i], h->prof_stop[i]);
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

fs_status fs_sketch_apply_ld(fs_sketch_t h, const void* A, int64_t lda, int64_t n, void* out,
                             int64_t ldo, fs_dtype dt, void* stream) {
  if (!h || n < 0 || !valid_dtype(dt)) return FS_ERR_INVALID_ARG;
  if (n == 0) return FS_OK;
  if (!A || !out || lda < n || ldo < n) return FS_ERR_INVALID_ARG;
  if (n > 0x7fffffff || lda > ((int64_t)1 << 40) || ldo > ((int64_t)1 << 40)) return FS_ERR_INVALID_ARG;
  const size_t esz = dt == FS_F32 ? 4 : 2;
  if ((uintptr_t)A % esz || (uintptr_t)out % esz) return FS_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;

  int variant;
  size_t need;
  fs_status rc = needed_workspace(h, A, lda, n, out, ldo, dt, &variant, &need);
  if (rc != FS_OK) return rc;
  rc = ensure_workspace(h, need);
  if (rc != FS_OK) return rc;
  if (variant == FS_VARIANT_MFMA) {
    rc = ensure_orbit(h);
    if (rc != FS_OK) return rc;
  }

  fs::EventPair ev;
  if (h->profiling && h->prof_used < (int)h->prof_start.size()) {
    ev.start = h->prof_start[h->prof_used];
    ev.stop = h->prof_stop[h->prof_used];
    ++h->prof_used;
  }
  hipError_t e;
  int mode = 0;
  if (h->kind == FS_KIND_SJLT_SCATTER) {
    e = fs::launch_scatter(h->p, A, lda, n, out, ldo, dt, h->ws, st, ev);
  } else if (h->kind == FS_KIND_GAUSS_DENSE) {
    e = fs::launch_gauss(h->dense, h->p.k, h->p.d, A, lda, n, out, ldo, dt, st, ev);
  } else if (h->kind == FS_KIND_BLOCKROW) {
    e = fs::launch_blockrow(h->p, A, lda, n, out, ldo, dt, st, ev);
  } else if (variant == FS_VARIANT_MFMA) {
    e = fs::launch_mfma(h->p, A, lda, n, out, ldo, dt, h->ws, h->orbit, st, ev, &mode);
  } else {
    e = fs::launch_generic(h->p, A, lda, n, out, ldo, dt, st, ev);
  }
  h->last_variant = variant;
  h->last_mode = mode;
  if (e != hipSuccess) return hip_fail(h, e);
  return FS_OK;
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
  fs::EventPair ev;
  if (h->profiling && h->prof_used < (int)h->prof_start.size()) {
    ev.start = h->prof_start[h->prof_used];
    ev.stop = h->prof_stop[h->prof_used];
    ++h->prof_used;
  }
  if (!use_mfma) {
    const hipError_t e = fs::launch_generic_rows(h->p, G, ldg, n, out, ldo, dt, st, ev);
    h->last_variant = FS_VARIANT_GENERIC;
    h->last_mode = 0;
    if (e != hipSuccess) return hip_fail(h, e);
    return FS_OK;
  }
  rc = ensure_orbit(h);  // the gather-reduction walks the wiring through this table
  if (rc != FS_OK) return rc;
  const hipError_t e = fs::launch_rows(h->p, G, ldg, n, out, ldo, dt, h->ws, h->orbit, st, ev);
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
