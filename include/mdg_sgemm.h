/*
 * mdg_sgemm -- model-driven adaptive SGEMM for AMD MI355X (gfx950).  C ABI.
 *
 * The operation is the general matrix multiplication of Eq. 1, Section 2.2 of
 * "A model-driven approach for a new generation of adaptive libraries":
 *
 *     C = alpha * op(A) * op(B) + beta * C,   op(X) = X or X^T,
 *     op(A) is M x K, op(B) is K x N, C is M x N, all real fp32,
 *
 * stated with the BLAS xGEMM argument list.  Each call is served by one member
 * of a small family of parametric kernels ("variants"): a "direct" kernel that
 * covers every use-case and a specialised tiled kernel (Section 2.3 describes
 * that split for the library the paper studies).  Which variant runs is
 * decided by a decision tree over (M, N, K, transA, transB), trained off-line
 * on measured runtimes and compiled into this library as nested if-then-else
 * (Section 3, 'Model and code generation').
 *
 * Conventions common to all entry points
 *   - Pointers A, B, C and the workspace are DEVICE pointers owned by the
 *     caller.  The library allocates no device memory and frees none.  A and B
 *     are only read; C is read iff beta != 0 and written.  C must not overlap A or B.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it; no call synchronises unless its comment says so.
 *   - alpha and beta are host values.
 *   - Layout: MDG_COL_MAJOR stores element (r, c) of a matrix at r + c*ld,
 *     MDG_ROW_MAJOR at r*ld + c.  Stored A is M x K (K x M if transA), stored B
 *     is K x N (N x K if transB).  Leading dimensions must be >= max(1, extent
 *     of the contiguous index of the stored matrix).  Elements between that
 *     extent and ld are never read and never written.
 *   - Degenerate sizes: M == 0 or N == 0 -> success, nothing touched.
 *     K == 0 or alpha == 0 -> C = beta*C, A and B not read.  beta == 0 -> C is
 *     not read (NaN/Inf in C do not propagate).
 *   - Return value: MDG_OK (0), or for an invalid argument minus its 1-based
 *     position in the mdg_sgemm argument list (layout -1, transA -2, transB -3,
 *     M -4, N -5, K -6, A -8, lda -9, B -10, ldb -11, C -13, ldc -14), or one
 *     of the MDG_ERR_* codes below.  Nothing is printed and nothing aborts.
 *   - Soundness (Section 3, requirement 1): mdg_sgemm accepts every input the
 *     argument list admits -- any sizes, leading dimensions and alignments --
 *     because one variant (id 0) is legal for all of them.
 */
#ifndef MDG_SGEMM_H
#define MDG_SGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Largest M, N or K accepted (larger values are an invalid argument).  The kernels index rows, columns and k with
   32-bit integers and add at most a tile or a K slice to a dimension: the limit keeps those sums below 2^31. */
#define MDG_MAX_DIM 2147418111 /* 2^31 - 1 - 65536 */

typedef enum { MDG_ROW_MAJOR = 101, MDG_COL_MAJOR = 102 } mdg_layout;
typedef enum { MDG_NO_TRANS = 111, MDG_TRANS = 112, MDG_CONJ_TRANS = 113 /* same as MDG_TRANS for real data */ } mdg_op;

enum {
  MDG_OK = 0,
  MDG_ERR_WORKSPACE = -101,       /* variant needs more workspace than is registered */
  MDG_ERR_ILLEGAL_VARIANT = -102, /* forced variant cannot run on this input */
  MDG_ERR_LAUNCH = -103,          /* the HIP runtime rejected a launch or an event call */
  MDG_ERR_BAD_VARIANT = -104,     /* variant id out of range */
  MDG_ERR_NULL = -105,            /* a required output pointer is NULL */
  MDG_ERR_ALIGNMENT = -106,       /* a workspace pointer is not 256-byte aligned */
  MDG_ERR_SCRATCH_LIMIT = -107    /* mdg_sgemm_static_scratch: the variant needs more than MDG_STATIC_SCRATCH_BYTES */
};

/* Kernel families (Section 2.3: one generic kernel plus one specialised kernel; the vector-shaped
   family serves products with a very thin N). */
typedef enum {
  MDG_FAMILY_DIRECT = 0, /* register-blocked, bounds-checked, vector ALUs; any shape */
  MDG_FAMILY_TILED = 1,  /* LDS-staged, double-buffered, fp32 matrix-core (MFMA) tiles */
  MDG_FAMILY_SKINNY = 2, /* N <= a few columns: streams A once, bandwidth-bound */
  MDG_FAMILY_INDIRECT = 3 /* Section 2.3's indirect path: pad / transpose helper passes copy op(A), op(B) into the
                             workspace in the tiled kernel's preferred layout, then the tiled kernel runs on the
                             copies with every tile whole; the variant's time includes the helpers */
} mdg_family;

/* One point of the tuning space (Section 2.3 lists the kind of parameters: work-group tile, per-thread
   or per-wave tile, vector widths, K step, use of local memory). */
typedef struct {
  int32_t id;
  int32_t family;      /* mdg_family */
  int32_t tile_m;      /* work-group tile of C, rows */
  int32_t tile_n;      /* work-group tile of C, columns */
  int32_t tile_k;      /* K step per main-loop iteration */
  int32_t threads;     /* work-group size */
  int32_t sub_m;       /* direct: rows per thread; tiled: rows per wave; skinny: rows per thread */
  int32_t sub_n;       /* direct: columns per thread; tiled: columns per wave; skinny: columns held per thread */
  int32_t vec;         /* widest global access in fp32 elements */
  int32_t lds;         /* 1 if operands are staged through LDS; 2 if row-contiguous operands are moved from global
                          memory straight into LDS (needs those operands 16-byte aligned) */
  int32_t split_k;     /* number of K slices (1 = none); > 1 needs workspace and a reduce pass */
  int32_t fallback;    /* variant tried next when this one is not legal for an input (chains end at a variant that is) */
  char name[48];
} mdg_variant_desc;

/*
 * The GEMM call (Eq. 1, Section 2.2).  Validates, maps a row-major problem to
 * the equivalent column-major one (C^T = op(B)^T op(A)^T), asks the compiled
 * decision tree for a variant, and if that is not legal for this input
 * (Section 4.1: every class must be a valid configuration for the input)
 * follows the variant's fallback chain -- fewer K slices of the same tile, a
 * wider skinny kernel, finally variant 0 -- to the first legal one, and
 * enqueues the kernel(s) on `stream`.
 */
int mdg_sgemm(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha, const float* A,
              int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc, void* stream);

/*
 * Same operation with the variant forced (tuning run and tests; Section 4.1:
 * the dataset is built by running every configuration on every input).
 * Returns MDG_ERR_ILLEGAL_VARIANT / MDG_ERR_WORKSPACE instead of falling back.
 */
int mdg_sgemm_variant(int variant, int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                      const float* A, int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc,
                      void* stream);

/*
 * mdg_sgemm for callers that cannot allocate device memory and have registered no workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result.  The
 * partial sums of split-K variants (and the packed operand copies of indirect variants) go to a device array
 * of MDG_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the library is used on holds its own copy until the process ends) instead
 * of the registered workspace, which this call neither reads nor needs.  The call allocates and frees nothing.
 *
 * The variant is the one mdg_sgemm would run with a workspace that is never too small.  If that variant needs
 * more than MDG_STATIC_SCRATCH_BYTES (mdg_workspace_bytes: split_k * M * N * 4 bytes for a split-K variant), the
 * call returns MDG_ERR_SCRATCH_LIMIT and
 * enqueues nothing; C is untouched.  Variants that do not split K need no scratch and always run.
 *
 * All calls on one GPU share that GPU's array: calls on different streams (or from different threads) that may
 * execute at the same time race on it, exactly as calls sharing a registered workspace do; calls on one stream
 * are ordered and safe.  Nothing in the array has to be cleared between calls (every element a call reads, it
 * has written first).  The device address of the array is looked up on the first call on each device, with
 * that device current.
 */
#define MDG_STATIC_SCRATCH_BYTES (32 << 20)
int mdg_sgemm_static_scratch(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                             const float* A, int64_t lda, const float* B, int64_t ldb, float beta, float* C,
                             int64_t ldc, void* stream);

/*
 * The compiled decision tree (Section 3, 'Model and code generation'): pure
 * host integer code, no GPU needed.  transA / transB are 0 or 1 and refer to
 * the column-major problem.  Returns a variant id in [0, mdg_variant_count()).
 */
int mdg_select(int transA, int transB, int64_t M, int64_t N, int64_t K);

/*
 * What mdg_sgemm itself asks: the same model behind a memo of the shapes this thread asked about recently
 * (1024 entries in 512 two-way sets, thread-local).  Returns exactly what mdg_select returns; a repeated shape costs a
 * few nanoseconds instead of a model evaluation (the end of Section 5.4 discusses the overhead of the model at run time).
 */
int mdg_select_memo(int transA, int transB, int64_t M, int64_t N, int64_t K);

/* The traditional dispatch the paper compares against (Section 5, "default"): one tiled and one direct
   configuration switched by a size threshold. */
int mdg_select_default(int transA, int transB, int64_t M, int64_t N, int64_t K);

/* Name of the model compiled into mdg_select (e.g. "hMax-L1/logratio"), static storage. */
const char* mdg_selector_name(void);

int mdg_variant_count(void);

/* Fills *out; MDG_ERR_BAD_VARIANT / MDG_ERR_NULL on misuse. */
int mdg_variant_info(int variant, mdg_variant_desc* out);

/*
 * 1 if `variant` may run on this column-major problem, 0 if not, < 0 on a bad
 * variant id.  Depends on sizes, transposes, leading dimensions, pointer
 * alignment and the registered workspace.  Pointers are only inspected, never
 * dereferenced (host code).
 */
int mdg_variant_legal(int variant, int transA, int transB, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb,
                      int64_t ldc, const void* A, const void* B, const void* C);

/* Bytes of workspace `variant` needs for a problem of this size (0 for most variants): split_k slices of the
   M x N result for split-K variants; for indirect variants the padded operand copies, taken over the transpose
   combination that needs most. */
size_t mdg_workspace_bytes(int variant, int64_t M, int64_t N, int64_t K);

/*
 * Registers a caller-owned device buffer used by split-K variants for partial
 * sums and by indirect variants for their packed operand copies.  The library keeps the pointer until it is replaced (NULL, 0 clears
 * it) and never frees it.  dev_ptr must be 256-byte aligned (MDG_ERR_ALIGNMENT
 * otherwise).  Calls that use the workspace must not overlap on different
 * streams.  Process-wide; may be called from any thread (a call that runs at
 * the same time sees either the old or the new registration, never a mix),
 * but replacing the workspace while GEMM calls that use it are still being
 * issued or executed is the caller's race.
 */
int mdg_set_workspace(void* dev_ptr, size_t bytes);

/* Static, human-readable text for a status code. */
const char* mdg_status_string(int status);

/*
 * Timing core of the tuning run (Section 4.1, dataset creation) and of the
 * benchmark: measures whole calls -- the kernel plus any pass the variant
 * needs before or after it -- with HIP events recorded on `stream`.
 *
 * `variant` >= 0 forces that variant; -1 times mdg_sgemm (selector included);
 * -2 times mdg_sgemm with the default dispatch in place of the tree.
 * The problem is always column-major.  A, B, C point to `n_sets` operand sets
 * laid out `a_set_stride`, `b_set_stride`, `c_set_stride` ELEMENTS apart;
 * successive calls rotate through the sets so that no operand is still in
 * cache from the previous call (n_sets = 1 gives warm-cache numbers).
 * Does `warmup` untimed calls, then `spans` spans of `reps` back-to-back
 * calls, and writes the average milliseconds per call of each span to the
 * HOST array ms_per_call[spans].  SYNCHRONISES the stream.  C is overwritten.
 */
int mdg_time_calls(int variant, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha, const float* A,
                   int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc, int n_sets,
                   int64_t a_set_stride, int64_t b_set_stride, int64_t c_set_stride, int warmup, int reps, int spans,
                   float* ms_per_call, void* stream);

/*
 * Host nanoseconds per call of mdg_select averaged over `iters` passes through
 * the n given problems (the end of Section 5.4 reports the tree-traversal overhead).
 */
double mdg_time_select_ns(const int32_t* transA, const int32_t* transB, const int64_t* M, const int64_t* N,
                          const int64_t* K, int64_t n, int iters);

/* The same measurement through mdg_select_memo: what a caller pays when its shapes repeat. */
double mdg_time_select_memo_ns(const int32_t* transA, const int32_t* transB, const int64_t* M, const int64_t* N,
                               const int64_t* K, int64_t n, int iters);

#ifdef __cplusplus
}
#endif
#endif /* MDG_SGEMM_H */
