/*
 * flashsketch.h -- C ABI of the MI355X (gfx950) BlockPerm-SJLT sketch library.
 *
 * The library applies a sparse sketch S (k x d) to a dense A (d x n) and
 * returns Y = S A (k x n)  (paper Section 3 "Notation": A in R^{d x n},
 * S in R^{k x d}, Y := S A).
 *
 * S is never stored.  It is a pure function of (d, k, Bc, Br, kappa, s, seed):
 *   - an M x M grid of Br x Bc blocks, M = k/Br = ceil(d/Bc) (Section 4, "Block model"); when
 *     Bc does not divide d the input is treated as zero-padded to M*Bc rows (the paper's
 *     "padding"), i.e. S is the first d columns of the padded sketch;
 *   - block (g, h) is nonzero iff h = f^l(g) for some l in 1..kappa, where
 *     f(x) = (a x + b) mod M is a full-period affine map whose (a, b) are
 *     derived from the seed (Section 4, "Block-level wiring"; Appendix E,
 *     "Full-cycle affine construction");
 *   - every column of a nonzero block has exactly s entries +-1 at distinct
 *     rows given by a 32-bit hash of (seed, g, h, local row) (Section 4,
 *     "Intra-block SJLT mixing"; Appendix E, "Within-block hashing");
 *   - all entries are scaled by 1/sqrt(kappa*s) (Alg. 1, scaling step).
 *
 * Conventions
 *   Layout     A is row-major d x n: element (u, t) at A[u*lda + t]; lda >= n,
 *              counted in ELEMENTS.  out is row-major k x n with leading
 *              dimension ldo >= n (fs_sketch_apply: ldo = n).  The n columns
 *              are the vectors being sketched.
 *   Pointers   A, out, rows, signs, S_dense and workspaces are DEVICE pointers
 *              owned by the caller.  Handles and fs_info are HOST objects.
 *   Alignment  A and out must be aligned to their element size.  The matrix-core
 *              kernels load 4 columns per lane as one vector when A and lda are
 *              aligned to 4 elements; otherwise they load element by element,
 *              about half as fast (never an error).  With vector loads and n not
 *              a multiple of 4, up to 3 elements of a row's own padding (columns
 *              n .. lda-1, inside the aligned 4-element group of the row's last
 *              valid element) are loaded and discarded; their values, NaN
 *              included, never reach the result.  Element loads read nothing
 *              beyond column n-1.  Stores to out are vectors when out and ldo are
 *              aligned to 4 elements, else element by element.
 *   Streams    `stream` is a hipStream_t passed as void* (NULL = default
 *              stream).  Calls enqueue work and return; they never synchronise.
 *              A handle must not be used from two streams at the same time
 *              (its workspace is shared).
 *   Precision  accumulation is always fp32; one fp32 multiply by
 *              (float)(1/sqrt(kappa*s)) follows; bf16 and half outputs are rounded to
 *              nearest-even.
 *   Errors     every call returns fs_status; nothing throws, aborts or prints.
 *              Argument errors are detected before any HIP call is made.
 *   Determinism FS_KIND_BLOCKPERM uses no atomics on data: the same inputs give
 *              bit-identical outputs.  FS_KIND_SJLT_SCATTER sums with global
 *              float atomics and is order-nondeterministic by construction.
 */
#ifndef FLASHSKETCH_H
#define FLASHSKETCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fs_sketch_s* fs_sketch_t; /* opaque host handle */

typedef enum {
  FS_OK = 0,
  FS_ERR_INVALID_ARG = 1, /* bad pointer, size, divisibility, range        */
  FS_ERR_UNSUPPORTED = 2, /* valid request this build has no kernel for    */
  FS_ERR_ALLOC = 3,       /* host or device allocation failed              */
  FS_ERR_HIP = 4          /* a HIP runtime call failed (see fs_info)       */
} fs_status;

/* dtype of A and of out.  The paper's kernels are fp32 only (Section 6 names other precisions
 * as future work); the 16-bit types here accumulate in fp32 and round the result once, to
 * nearest even.  FS_F16 is IEEE binary16: subnormal inputs count with their value, results
 * beyond +-65504 become infinities. */
typedef enum { FS_F32 = 0, FS_BF16 = 1, FS_F16 = 2 } fs_dtype;

typedef enum {
  FS_KIND_BLOCKPERM = 0,    /* the paper's sketch (Section 4)                              */
  FS_KIND_SJLT_SCATTER = 1, /* prior-art baseline: plain SJLT, global scatter-add
                               (Section 3 "GPU bottlenecks for Sparse Sketching").
                               Same S as BLOCKPERM with M = 1: needs Bc = d, Br = k,
                               kappa = 1.                                                  */
  FS_KIND_GAUSS_DENSE = 2,  /* dense Gaussian sketch S_ij ~ N(0, 1/k) (Section 1) applied
                               by an MFMA GEMM; Bc, Br, kappa, s are ignored.  Reference
                               point only: needs 64 | d, 128 | k, 4 | lda, a 16-byte (fp32)
                               or 8-byte (bf16, half) aligned A and d*lda*sizeof(elt) < 2^31,
                               else apply returns FS_ERR_UNSUPPORTED.                      */
  FS_KIND_BLOCKROW = 3      /* FlashBlockRow (Appendix D, Alg. 2): gather-only block-row
                               sampling.  Same parameters as BLOCKPERM; output row (g, r)
                               adds s signed rows of A from each of the kappa blocks f^l(g)
                               and scales by sqrt(d/k)/sqrt(kappa*s).  Reads k*kappa*s rows
                               of A; input coordinates that no row samples are ignored.   */
} fs_kind;

/* Kernel variants of the BLOCKPERM apply (fs_sketch_set_variant). */
typedef enum {
  FS_VARIANT_AUTO = 0,    /* pick by shape/dtype/alignment                          */
  FS_VARIANT_GENERIC = 1, /* one lane per column, LDS-private output tile, any Br   */
  FS_VARIANT_MFMA = 2     /* +-1 operand on the matrix cores: any power-of-two Br
                             (other Br while its kappa slots, each padded to the next
                             power of two rows, fit 128 tile rows, or padded Br <= 64),
                             any Bc, kappa <= 128 (more when Br <= 64),
                             64*ceil(Bc/64)*lda*sizeof(elt) < 2^31; about twice as fast
                             when A and lda are aligned to 4 columns (vector loads)  */
} fs_variant;

typedef struct {
  int64_t d, k;
  int32_t Bc, Br, kappa, s;
  int32_t M;           /* blocks per side                                   */
  int32_t a, b;        /* wiring f(x) = (a x + b) mod M                     */
  int32_t a_inv;       /* inverse of a modulo M (0 when M = 1)              */
  uint32_t key0, key1; /* seed-derived hash keys                            */
  float scale;         /* (float)(1/sqrt(kappa*s)); 1/sqrt(k) for GAUSS     */
  int32_t kind;        /* fs_kind                                           */
  int32_t variant;     /* fs_variant requested                              */
  int32_t last_variant;/* variant the most recent apply actually launched   */
  int32_t last_mode;   /* its work decomposition: 0 one tile per work-group (generic),
                          1 MFMA output-stationary, 2 MFMA input-stationary with
                          partial planes, 3 the same with orbit runs merged in LDS */
  int32_t last_hip_error; /* hipError_t of the last failed HIP call, else 0 */
  uint64_t workspace_bytes; /* size of the workspace currently attached     */
  char last_kernel[64];     /* NUL-terminated name of the kernel the most recent apply launched,
                               with its compile-time variant (matrix-core kernels: the template
                               arguments in order), so that a stored profile can be matched to
                               what ran; "" before the first apply                  */
} fs_info;

/* Create a BLOCKPERM handle.  Pure host work (no HIP call, usable without a GPU).
 * Errors (FS_ERR_INVALID_ARG): out == NULL; d, k, Bc, Br, kappa, s < 1;
 * Br does not divide k, ceil(d/Bc) != k/Br; kappa > M
 * (Appendix E: the kappa neighbours are distinct only for kappa <= M);
 * s > Br (rows must be distinct, Alg. 1) or s > 32; Br > 65536; M > 2^24. */
fs_status fs_sketch_create(fs_sketch_t* out, int64_t d, int64_t k, int32_t Bc, int32_t Br,
                           int32_t kappa, int32_t s, uint64_t seed);

/* As above for any kind.  SJLT_SCATTER requires Bc == d, Br == k, kappa == 1.
 * GAUSS_DENSE allocates and fills the k x d matrix on the current device
 * (FS_ERR_HIP / FS_ERR_ALLOC without a device); it ignores Bc, Br, kappa, s. */
fs_status fs_sketch_create_kind(fs_sketch_t* out, fs_kind kind, int64_t d, int64_t k, int32_t Bc,
                                int32_t Br, int32_t kappa, int32_t s, uint64_t seed);

/* Y = S A of the paper's problem statement (Section 3, "Notation"), computed as Alg. 1 defines
 * it block by block (Section 5.1): out (k x n, ld = n) = S * A (d x n, ld = lda), both of type
 * `dtype`.
 * n == 0 is FS_OK and launches nothing.  Errors: NULL handle/A/out, n < 0,
 * lda < n, unknown dtype.  May grow the handle's workspace with hipMalloc on
 * first use unless one was attached with fs_sketch_set_workspace.  The first
 * matrix-core apply of a handle also allocates a table of 8*M bytes (the orbit
 * of the wiring map) and enqueues the small kernel that fills it, unless fs_sketch_prepare
 * has done so; no call ever copies from the host or synchronises.  Later applies only enqueue
 * kernels (call prepare, or apply once, before capturing applies into a HIP graph). */
fs_status fs_sketch_apply(fs_sketch_t h, const void* A, int64_t lda, int64_t n, void* out,
                          fs_dtype dtype, void* stream);

/* Same with an explicit output leading dimension (column-chunk views: the 256-column
 * chunks a gradient-compression pipeline hands over, Appendix F). */
fs_status fs_sketch_apply_ld(fs_sketch_t h, const void* A, int64_t lda, int64_t n, void* out,
                             int64_t ldo, fs_dtype dtype, void* stream);

/* fs_sketch_apply_ld for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results; but the kernels' scratch memory (partial planes of the
 * cross-block accumulation, the scatter baseline's fp32 accumulator, the orbit table of the
 * wiring, rebuilt by a small kernel on every call) is a fixed device array inside the library,
 * FS_STATIC_SCRATCH_BYTES for the planes plus 1 MiB for the table, which every GPU that runs
 * the library holds until the process ends (the runtime places it there when the first call on
 * that GPU looks up its address: make that call before a graph capture starts).  The call
 * allocates and frees nothing, copies nothing from the host and never synchronises; the
 * handle's own workspace is not touched.
 * A call whose planes need more than FS_STATIC_SCRATCH_BYTES (see fs_sketch_plan) returns
 * FS_ERR_ALLOC and launches nothing; a wiring with M > 2^17 runs without the orbit table
 * (slower modes, same result up to summation order).  FS_KIND_GAUSS_DENSE works (its matrix was
 * allocated by create).  All calls on one GPU share the one array, which keeps the last call's
 * contents: calls that overlap in time on one GPU (two streams, two threads, two handles)
 * race; order them on one stream or with events. */
#define FS_STATIC_SCRATCH_BYTES (32u << 20)
fs_status fs_sketch_apply_static(fs_sketch_t h, const void* A, int64_t lda, int64_t n, void* out,
                                 int64_t ldo, fs_dtype dtype, void* stream);

/* The same sketch for inputs held examples-as-rows: G is n x d row-major (ld = ldg >= d,
 * every row one vector to sketch, as a pipeline that compresses per-example gradients holds
 * them: Section 7, "End-to-end ML: GraSS for Data Attribution", and Appendix F) and
 * out (n x k, ld = ldo >= k) = G S^T, i.e. out[i, :] = S G[i, :] -- the transpose of what
 * fs_sketch_apply_ld computes on G^T.  FS_KIND_BLOCKPERM only.  Two kernels, chosen as for
 * fs_sketch_apply (fs_sketch_set_variant applies here too):
 *  - matrix cores: Br a power of two (else see FS_VARIANT_MFMA).  kappa*Br <= 128 is
 *    input-stationary (G is read once; fastest when kappa*Br is exactly 32, 64 or 128, the
 *    heights of its tiles); beyond
 *    that Br >= 32 is output-stationary (G is read kappa times, mostly from L2; blocks higher
 *    than 128 rows in 128-row slices) and smaller Br input-stationary in groups of 128/Br
 *    wiring slots (G is read once per group).  Also needs 130*ldg*sizeof(elt) < 2^31 (input-stationary: 34*ldg*sizeof(elt));
 *    any Bc, and d need not be a multiple of it.
 *    Fastest when G, ldg*sizeof(elt) and Bc*sizeof(elt) are multiples of 16
 *    bytes (128-bit loads; otherwise four dword loads or, for an odd ldg of a 16-bit type,
 *    eight element loads per piece).  A row stride that is a large power of two maps the
 *    rows of a tile to one HBM channel: prefer ldg = d + 64 elements.
 *  - general: every other valid sketch (more than 128 padded rows of blocks whose padded
 *    height is 128 or more, with Br not a power of two or kappa > 128);
 *    tiles are turned through LDS and accumulated without atomics, G is read kappa times.
 * Forcing FS_VARIANT_MFMA on a call the matrix-core kernel cannot take returns
 * FS_ERR_UNSUPPORTED (nothing is launched).
 * n == 0 is FS_OK.  Errors: NULL handle/G/out, n < 0, ldg < d, ldo < k, unknown dtype.
 * Workspace (matrix cores, input-stationary shapes only): kappa (times a row split) sets of
 * n x k floats, grown or attached as for fs_sketch_apply; fs_sketch_rows_workspace_bytes gives its size for
 * a well-aligned call.  The first call of a handle also uploads the 8*M-byte orbit table. */
fs_status fs_sketch_apply_rows(fs_sketch_t h, const void* G, int64_t ldg, int64_t n, void* out,
                               int64_t ldo, fs_dtype dtype, void* stream);
fs_status fs_sketch_rows_workspace_bytes(fs_sketch_t h, int64_t n, fs_dtype dtype, size_t* bytes);

/* Which kernel an apply with these arguments would launch, without launching anything (pure
 * host work, usable without a GPU): for tuning block sizes and for checking that a call stays
 * on the fast path.  `rows` = 0 describes fs_sketch_apply_ld(h, A, ld, n, ...), 1 describes
 * fs_sketch_apply_rows(h, A, ld, n, ...); only the alignment of the address A is used, the
 * memory is not touched.  Results: *variant (fs_variant that would run; for kinds other than
 * FS_KIND_BLOCKPERM FS_VARIANT_GENERIC), *mode (as fs_info.last_mode), *flags (fs_plan_flags),
 * *workspace_bytes (what the call needs attached or would allocate).  The handle's
 * fs_sketch_set_variant choice is honoured.  Errors as for the apply it describes
 * (FS_ERR_INVALID_ARG, FS_ERR_UNSUPPORTED); any result pointer may be NULL. */
typedef enum {
  FS_PLAN_ELEMENT_LOADS = 1, /* A / G not aligned for vector loads: narrower loads, slower    */
  FS_PLAN_ROW_SLICES = 2,    /* output blocks higher than 128 rows, served in 128-row slices   */
  FS_PLAN_SLOT_GROUPS = 4,   /* more than 128 stacked rows of small blocks: input read once
                                per group of wiring slots                                      */
  FS_PLAN_SPLIT = 8,         /* the rows of a work-group's input are split over grid.z         */
  FS_PLAN_STACKED = 16       /* output-stationary with several output blocks, consecutive on
                                the orbit of the wiring, per wave (mode 1, no workspace)       */
} fs_plan_flags;
fs_status fs_sketch_plan(fs_sketch_t h, const void* A, int64_t ld, int64_t n, fs_dtype dtype,
                         int32_t rows, int32_t* variant, int32_t* mode, int32_t* flags,
                         size_t* workspace_bytes);

/* Materialise the nonzeros of S on the device (BLOCKPERM / SJLT_SCATTER):
 * rows[c*kappa*s + (l-1)*s + i] = global output row, signs[...] = +1/-1, for
 * column c of S, wiring slot l (the l with f^l(g) = c / Bc) and update i.
 * Both buffers hold d*kappa*s entries.
 * BLOCKROW: the sketch is stored by rows instead: rows[i*kappa*s + (l-1)*s + t] = global
 * COLUMN index read by output row i (it may lie in the zero padding, >= d), signs likewise;
 * both buffers hold k*kappa*s entries. */
fs_status fs_sketch_export(fs_sketch_t h, int32_t* rows, int8_t* signs, void* stream);

/* GAUSS_DENSE only: copy the k x d fp32 matrix (row-major, ld = d) to S_dense. */
fs_status fs_sketch_export_dense(fs_sketch_t h, float* S_dense, void* stream);

/* Allocates the handle's device tables (today: the orbit of the wiring map f of Appendix E,
 * 8*M bytes, for 4 <= M <= 2^20) on the current device and enqueues on `stream` the kernel that
 * fills them.  Optional: the first apply does the same.  After it, applies of a handle with an
 * attached workspace neither allocate nor synchronise.  Later applies must be ordered after
 * this call's work (same stream, or an event).  FS_OK and nothing done for other kinds. */
fs_status fs_sketch_prepare(fs_sketch_t h, void* stream);

/* The integers that define S for this handle (Section 3 "Notation" for d, k; Section 4 for
 * M, Bc, Br, kappa, s; Appendix E for the wiring a, b), the scale of Alg. 1's last step, and
 * what the most recent apply launched. */
fs_status fs_sketch_info(fs_sketch_t h, fs_info* out);

/* Bytes of device workspace an apply of n columns of `dtype` needs at most with the
 * handle's current variant setting (0 if none).  The workspace holds the fp32 partial results
 * of the cross-block accumulation (Section 5.3: each output tile is owned by one work-group and
 * summed without global atomics) when the work is split by INPUT block: kappa (times a row
 * split) planes of k x n floats, fewer when consecutive blocks of the wiring's orbit are merged
 * on chip.  For FS_KIND_SJLT_SCATTER with 16-bit types: the k x n fp32 accumulator. */
fs_status fs_sketch_workspace_bytes(fs_sketch_t h, int64_t n, fs_dtype dtype, size_t* bytes);

/* Attach a caller-owned device workspace (256-byte aligned); applies then never grow a
 * workspace and fail with FS_ERR_ALLOC if it is too small (after fs_sketch_prepare they
 * allocate nothing at all).  Its contents need not be kept between calls.
 * (NULL, 0) detaches it and returns to the internal, lazily grown one. */
fs_status fs_sketch_set_workspace(fs_sketch_t h, void* dev_ptr, size_t bytes);

/* Force a kernel variant for BLOCKPERM applies (tests, benchmarks).
 * FS_ERR_UNSUPPORTED at apply time if the forced variant cannot run the shape. */
fs_status fs_sketch_set_variant(fs_sketch_t h, fs_variant v);

/* Kernel timing for benchmarks.  After profile_begin, each apply records HIP events on its
 * stream, up to max_launches applies: with FS_PROFILE_KERNEL in `scope` one pair around its
 * dominant kernel (the one that streams A), with FS_PROFILE_APPLY one pair around everything
 * the apply enqueues (zero-fills, table builds, the dominant kernel, plane reductions,
 * conversions).  Every recorded event costs a few microseconds on the stream, so with both
 * scopes the inner pair lengthens what the outer pair measures: ask for one scope at a time
 * when that matters.  profile_end synchronises the events and writes, per bracketed apply, the
 * elapsed milliseconds of the dominant kernel to the HOST array ms and of the whole apply to
 * the HOST array ms_apply (each of capacity max_launches; ms_apply may be NULL; a scope that was
 * not asked for reads 0), the number of applies to *count, and releases the events.  Errors:
 * NULL handle, ms or count, max_launches < 1, unknown scope, begin while already profiling, end
 * without begin. */
typedef enum { FS_PROFILE_KERNEL = 1, FS_PROFILE_APPLY = 2 } fs_profile_scope;
fs_status fs_sketch_profile_begin(fs_sketch_t h, int32_t max_launches, int32_t scope);
fs_status fs_sketch_profile_end(fs_sketch_t h, float* ms, float* ms_apply, int32_t* count);

/* Frees the handle and any device memory it owns (not caller workspaces).  Like every call
 * that frees device memory it must not run while a stream is being captured into a HIP graph
 * (HIP invalidates the capture). */
fs_status fs_sketch_destroy(fs_sketch_t h);

const char* fs_status_string(fs_status st);

#ifdef __cplusplus
}
#endif
#endif /* FLASHSKETCH_H */
