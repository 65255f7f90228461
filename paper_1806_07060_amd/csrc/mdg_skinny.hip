// Skinny-N kernel: products whose N is a handful of columns (fully-connected
// layers at small batch; the "mostly rectangular" shapes Section 4.1 of the
// paper points at).  Such calls move M*K floats of A for only 2*N flops per
// float: they are bound by HBM bandwidth, so the kernel streams A exactly once
// with coalesced loads and keeps NB columns of C per thread in registers.
// No matrix cores: the arithmetic intensity is far below their ridge.
//
//   A not transposed (m contiguous): one thread per row m; a wave reads 64
//     consecutive rows per k (256 contiguous bytes), B(k, j) is wave-uniform.
//   A transposed (k contiguous): one wave per R = 4 rows; lanes run along k,
//     partial dot products are combined with a cross-lane butterfly.
// K may be cut into split_k slices (more work-groups in flight for small M);
// partial sums then go to the workspace and a reduce pass finishes C.
// Columns beyond NB are covered by blockIdx.z.
#include "mdg_internal.h"
#include "mdg_variant_list.h"

namespace mdg {

struct SkinnyParams {
  const float* A;
  const float* B;
  float* C;
  float* ws;
  int64_t lda, ldb, ldc;
  int M, N, K;
  int split_k, k_per_split;
  float alpha, beta;
};

template <bool TB>
__device__ __forceinline__ float ld_b(const float* __restrict__ B, int64_t ldb, int k, int j) {
  return TB ? B[(int64_t)j + (int64_t)k * ldb] : B[(int64_t)k + (int64_t)j * ldb];
}

__device__ __forceinline__ void skinny_store(const SkinnyParams& p, int split, int m, int n, float v) {
  if (p.split_k > 1) {
    p.ws[(int64_t)split * p.M * p.N + (int64_t)m + (int64_t)n * p.M] = v;
  } else {
    float* c = p.C + (int64_t)m + (int64_t)n * p.ldc;
    float r = p.alpha * v;
    if (p.beta != 0.f) r = fmaf(p.beta, *c, r);
    *c = r;
  }
}

// ---- A not transposed: thread per row ------------------------------------------------------
template <int NB, bool TB>
__global__ __launch_bounds__(256) void skinny_n_kernel(SkinnyParams p) {
  const int m = blockIdx.x * 256 + threadIdx.x;
  const int split = blockIdx.y;
  const int n0 = blockIdx.z * NB;
  const int k_begin = split * p.k_per_split;
  const int k_end = min(p.K, k_begin + p.k_per_split);
  const int mc = min(m, p.M - 1);
  const float* __restrict__ a = p.A + mc;
  float acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) acc[j] = 0.f;
  int jc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) jc[j] = min(n0 + j, p.N - 1);

  int k = k_begin;
  for (; k + 16 <= k_end; k += 16) {  // 16 independent loads in flight per lane
    float av[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) av[u] = a[(int64_t)(k + u) * p.lda];
#pragma unroll
    for (int u = 0; u < 16; ++u)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[j] = fmaf(av[u], ld_b<TB>(p.B, p.ldb, k + u, jc[j]), acc[j]);
  }
  for (; k < k_end; ++k) {
    float av = a[(int64_t)k * p.lda];
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[j] = fmaf(av, ld_b<TB>(p.B, p.ldb, k, jc[j]), acc[j]);
  }
  if (m >= p.M) return;
#pragma unroll
  for (int j = 0; j < NB; ++j)
    if (n0 + j < p.N) skinny_store(p, split, m, n0 + j, acc[j]);
}

// ---- A transposed: wave per R rows, lanes along k ------------------------------------------
template <int NB, bool TB>
__global__ __launch_bounds__(256) void skinny_t_kernel(SkinnyParams p) {
  constexpr int R = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m0 = (blockIdx.x * 4 + wave) * R;
  const int split = blockIdx.y;
  const int n0 = blockIdx.z * NB;
  if (m0 >= p.M) return;  // whole wave leaves; no barriers in this kernel
  const int k_begin = split * p.k_per_split;
  const int k_end = min(p.K, k_begin + p.k_per_split);
  const float* __restrict__ arow[R];
#pragma unroll
  for (int r = 0; r < R; ++r) arow[r] = p.A + (int64_t)min(m0 + r, p.M - 1) * p.lda;
  int jc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) jc[j] = min(n0 + j, p.N - 1);
  float acc[R][NB];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[r][j] = 0.f;

  int k = k_begin + lane;
  for (; k + 64 < k_end; k += 128) {  // two k per lane per trip
    float a0[R], a1[R], b0[NB], b1[NB];
#pragma unroll
    for (int r = 0; r < R; ++r) a0[r] = arow[r][k], a1[r] = arow[r][k + 64];
#pragma unroll
    for (int j = 0; j < NB; ++j) b0[j] = ld_b<TB>(p.B, p.ldb, k, jc[j]), b1[j] = ld_b<TB>(p.B, p.ldb, k + 64, jc[j]);
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[r][j] = fmaf(a1[r], b1[j], fmaf(a0[r], b0[j], acc[r][j]));
  }
  for (; k < k_end; k += 64) {
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      float b = ld_b<TB>(p.B, p.ldb, k, jc[j]);
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r][j] = fmaf(arow[r][k], b, acc[r][j]);
    }
  }
  // butterfly over the 64 lanes; every lane ends with the full sums
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      float v = acc[r][j];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
      acc[r][j] = v;
    }
  // lane (r, j) writes element (m0 + r, n0 + j)
  if (lane < R * NB) {
    const int r = lane / NB, j = lane % NB;
    float v = 0.f;
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
      for (int jj = 0; jj < NB; ++jj)
        if (rr == r && jj == j) v = acc[rr][jj];
    if (m0 + r < p.M && n0 + j < p.N) skinny_store(p, split, m0 + r, n0 + j, v);
  }
}

template <int NB>
static int launch_cfg(int split_k, const GemmArgs& g) {
  SkinnyParams p;
  p.A = g.A, p.B = g.B, p.C = g.C, p.ws = g.ws;
  p.lda = g.lda, p.ldb = g.ldb, p.ldc = g.ldc;
  p.M = (int)g.M, p.N = (int)g.N, p.K = (int)g.K;
  p.split_k = split_k;
  p.k_per_split = (int)((g.K + split_k - 1) / split_k);
  p.alpha = g.alpha, p.beta = g.beta;
  const int64_t col_groups = (g.N + NB - 1) / NB;
  if (col_groups > 65535 || split_k > 65535) return MDG_ERR_LAUNCH;
  if (!g.tA) {
    dim3 grid((unsigned)((g.M + 255) / 256), (unsigned)split_k, (unsigned)col_groups);
    if (g.tB) skinny_n_kernel<NB, true><<<grid, dim3(256), 0, g.stream>>>(p);
    else skinny_n_kernel<NB, false><<<grid, dim3(256), 0, g.stream>>>(p);
  } else {
    dim3 grid((unsigned)((g.M + 15) / 16), (unsigned)split_k, (unsigned)col_groups);
    if (g.tB) skinny_t_kernel<NB, true><<<grid, dim3(256), 0, g.stream>>>(p);
    else skinny_t_kernel<NB, false><<<grid, dim3(256), 0, g.stream>>>(p);
  }
  int st = check_launch();
  if (st != MDG_OK || split_k == 1) return st;
  return launch_splitk_reduce(split_k, g);
}

int launch_skinny(int cfg, int split_k, const GemmArgs& g) {
  switch (cfg) {
#define X(c, NB) \
  case c:        \
    return launch_cfg<NB>(split_k, g);
    MDG_SKINNY_CONFIGS(X)
#undef X
  }
  return MDG_ERR_BAD_VARIANT;
}

}  // namespace mdg
