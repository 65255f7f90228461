/*
 * GEMM oracle -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A slow, plain CPU statement of the general matrix multiplication of the
 * paper's Eq. 1 (Section 2.2):  C = alpha * op(A) * op(B) + beta * C, with
 * op(A) of size M x K, op(B) of size K x N, C of size M x N, and A, B each
 * optionally stored transposed.  Inputs and output are fp32; every element is
 * the sum over ascending k of exact fp64 products, accumulated in fp64,
 * scaled in fp64 and rounded to fp32 once.  (The product of two fp32 values
 * is exact in fp64, so whether the compiler fuses the multiply-add or not
 * changes nothing.)
 *
 * Two entry points compute the same thing:
 *   oracle_sgemm_ijk   the three nested loops of Section 2.2, one element at a time;
 *   oracle_sgemm       the same per-element sums with the loops over output
 *                      elements interchanged and OpenMP over columns, so that
 *                      large cases finish; tests assert it is bit-identical
 *                      to oracle_sgemm_ijk.
 *   oracle_sgemm_elements  the same sum for a caller-given list of (i, j)
 *                      positions, for sampled checks of very large cases.
 *
 * Readings where the paper is silent (BLAS conventions):
 *   - real fp32 only; a conjugate transpose equals a transpose;
 *   - layout 101 = row-major, 102 = column-major; trans 111 = none, 112/113 = transposed;
 *   - beta == 0: C is not read (NaN/Inf in C do not propagate);
 *   - alpha == 0 or K == 0: A and B are not read, C = beta * C;
 *   - M == 0 or N == 0: nothing is touched;
 *   - padding between the stored rows and the leading dimension is never read
 *     for the result and never written.
 * Pins (tests, CPU only): identity and permutation operands, all-ones operands,
 * rank-1 products, transpose and layout identities, exact power-of-two scaling,
 * the special cases above, small-integer inputs against integer arithmetic,
 * numpy's fp64 matmul, and brute force over all tiny shapes.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * this file.  It shares no code with the GPU library.
 */
#include <stdint.h>
#include <stdlib.h>

#define ORACLE_ROW_MAJOR 101
#define ORACLE_COL_MAJOR 102
#define ORACLE_NO_TRANS 111
#define ORACLE_TRANS 112
#define ORACLE_CONJ_TRANS 113

/* Address of stored element (r, c) of a matrix with leading dimension ld. */
static inline int64_t at(int layout, int64_t r, int64_t c, int64_t ld) {
  return layout == ORACLE_COL_MAJOR ? r + c * ld : r * ld + c;
}

static inline int is_trans(int t) { return t == ORACLE_TRANS || t == ORACLE_CONJ_TRANS; }

static inline int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }

/* BLAS-style argument check: 0 if fine, else minus the 1-based position of the first bad argument. */
static int check_args(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K,
                      int64_t lda, int64_t ldb, int64_t ldc) {
  if (layout != ORACLE_ROW_MAJOR && layout != ORACLE_COL_MAJOR) return -1;
  if (transA != ORACLE_NO_TRANS && !is_trans(transA)) return -2;
  if (transB != ORACLE_NO_TRANS && !is_trans(transB)) return -3;
  if (M < 0) return -4;
  if (N < 0) return -5;
  if (K < 0) return -6;
  /* stored A is M x K (or K x M when transposed); the leading dimension spans
     the contiguous index: rows for column-major, columns for row-major. */
  int64_t a_rows = is_trans(transA) ? K : M, a_cols = is_trans(transA) ? M : K;
  int64_t b_rows = is_trans(transB) ? N : K, b_cols = is_trans(transB) ? K : N;
  int64_t a_min = layout == ORACLE_COL_MAJOR ? a_rows : a_cols;
  int64_t b_min = layout == ORACLE_COL_MAJOR ? b_rows : b_cols;
  int64_t c_min = layout == ORACLE_COL_MAJOR ? M : N;
  if (lda < max64(1, a_min)) return -9;
  if (ldb < max64(1, b_min)) return -11;
  if (ldc < max64(1, c_min)) return -14;
  return 0;
}

/* op(A)(i,k) and op(B)(k,j) as fp64 */
static inline double opA(int layout, int tA, const float* A, int64_t lda, int64_t i, int64_t k) {
  return (double)(tA ? A[at(layout, k, i, lda)] : A[at(layout, i, k, lda)]);
}
static inline double opB(int layout, int tB, const float* B, int64_t ldb, int64_t k, int64_t j) {
  return (double)(tB ? B[at(layout, j, k, ldb)] : B[at(layout, k, j, ldb)]);
}

/* One output element: the definition. */
static inline float element(int layout, int tA, int tB, int64_t K, float alpha, const float* A, int64_t lda,
                            const float* B, int64_t ldb, float beta, const float* C, int64_t ldc, int64_t i,
                            int64_t j) {
  double acc = 0.0;
  if (alpha != 0.0f)
    for (int64_t k = 0; k < K; ++k) acc += opA(layout, tA, A, lda, i, k) * opB(layout, tB, B, ldb, k, j);
  double r = (alpha != 0.0f) ? (double)alpha * acc : 0.0;
  if (beta != 0.0f) r += (double)beta * (double)C[at(layout, i, j, ldc)];
  return (float)r;
}

/* Section 2.2: three nested loops, each element of C in turn. */
int oracle_sgemm_ijk(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                     const float* A, int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc) {
  int info = check_args(layout, transA, transB, M, N, K, lda, ldb, ldc);
  if (info) return info;
  int tA = is_trans(transA), tB = is_trans(transB);
  for (int64_t i = 0; i < M; ++i)
    for (int64_t j = 0; j < N; ++j)
      C[at(layout, i, j, ldc)] = element(layout, tA, tB, K, alpha, A, lda, B, ldb, beta, C, ldc, i, j);
  return 0;
}

/*
 * Same sums, loops over output elements interchanged: for one column j of C
 * keep M fp64 accumulators and run k outermost over them (unit stride through
 * op(A) when it is stored with i contiguous); when op(A) is stored with k
 * contiguous, run the dot product innermost instead.  Either way element
 * (i, j) adds its products in ascending k, so the result equals
 * oracle_sgemm_ijk bit for bit.
 */
int oracle_sgemm(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha, const float* A,
                 int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc) {
  int info = check_args(layout, transA, transB, M, N, K, lda, ldb, ldc);
  if (info) return info;
  if (M == 0 || N == 0) return 0;
  int tA = is_trans(transA), tB = is_trans(transB);
  /* is op(A)(i,k) contiguous in i? */
  int a_i_contig = (layout == ORACLE_COL_MAJOR) ? !tA : tA;
  int failed = 0;
#pragma omp parallel
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)M);
    if (!acc) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    if (!failed) {
#pragma omp for schedule(dynamic, 1)
      for (int64_t j = 0; j < N; ++j) {
        for (int64_t i = 0; i < M; ++i) acc[i] = 0.0;
        if (alpha != 0.0f) {
          if (a_i_contig) {
            for (int64_t k = 0; k < K; ++k) {
              double b = opB(layout, tB, B, ldb, k, j);
              for (int64_t i = 0; i < M; ++i) acc[i] += opA(layout, tA, A, lda, i, k) * b;
            }
          } else {
            for (int64_t i = 0; i < M; ++i) {
              double s = 0.0;
              for (int64_t k = 0; k < K; ++k) s += opA(layout, tA, A, lda, i, k) * opB(layout, tB, B, ldb, k, j);
              acc[i] = s;
            }
          }
        }
        for (int64_t i = 0; i < M; ++i) {
          double r = (alpha != 0.0f) ? (double)alpha * acc[i] : 0.0;
          if (beta != 0.0f) r += (double)beta * (double)C[at(layout, i, j, ldc)];
          C[at(layout, i, j, ldc)] = (float)r;
        }
      }
    }
    free(acc);
  }
  return failed ? -1000 : 0;
}

/*
 * The definition evaluated at n listed positions (ii[t], jj[t]) only;
 * out[t] receives the element, C is left untouched.
 */
int oracle_sgemm_elements(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                          const float* A, int64_t lda, const float* B, int64_t ldb, float beta, const float* C,
                          int64_t ldc, int64_t n, const int64_t* ii, const int64_t* jj, float* out) {
  int info = check_args(layout, transA, transB, M, N, K, lda, ldb, ldc);
  if (info) return info;
  int tA = is_trans(transA), tB = is_trans(transB);
  for (int64_t t = 0; t < n; ++t)
    if (ii[t] < 0 || ii[t] >= M || jj[t] < 0 || jj[t] >= N) return -17;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t t = 0; t < n; ++t)
    out[t] = element(layout, tA, tB, K, alpha, A, lda, B, ldb, beta, C, ldc, ii[t], jj[t]);
  return 0;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
