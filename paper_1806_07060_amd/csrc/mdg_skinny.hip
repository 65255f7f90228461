// Skinny-N kernel: products whose N is a handful of columns (fully-connected
// layers at small batch; the "mostly rectangular" shapes Section 4.1 of the
// paper points at).  Such calls move M*K floats of A for only 2*N flops per
// float: they are bound by HBM bandwidth, so the kernels stream A exactly once
// with coalesced loads, keep NB columns of C per thread in registers and are
// built around the number of bytes a CU has in flight (about 40 KB per CU are
// needed to cover the memory latency at 8 TB/s).  Up to a few columns the
// arithmetic is vector FMAs; from about a dozen columns on the FMAs themselves
// would cap the streaming rate, and a matrix-core member (thin_mfma_kernel,
// further down) takes over.
//
//   A not transposed (m contiguous): a work-group owns a strip of 64 rows; its W
//     waves (16 for NB <= 4, else 4) each take a contiguous part of the K range,
//     so that one row strip alone keeps 16 x 16 loads of 256 contiguous bytes in
//     flight; lane = row, B(k, j) is wave-uniform and read with scalar loads; the
//     W partial sums meet in LDS and are added in wave order.
//   A transposed (k contiguous): one wave per R = 4 rows; lanes run along k with
//     16-byte loads (two per row in flight; any 4-byte-aligned address will do),
//     scalar loads for the tail and for a transposed B; partial dot products are
//     combined with a cross-lane butterfly.
// K may additionally be cut into split_k slices (grid.y): partial sums then go to
// the workspace and the reduce pass finishes C.  Columns beyond NB are covered by
// blockIdx.z.  Every sum is formed in a fixed order: results are deterministic.
#include "mdg_internal.h"
#include "mdg_variant_list.h"

namespace mdg {

typedef float floatx4 __attribute__((ext_vector_type(4)));
// four consecutive floats at any 4-byte-aligned address: one 16-byte load all the same (global memory takes any
// dword-aligned address), so the vector paths below need their elements in range, not aligned
typedef floatx4 floatx4u __attribute__((aligned(4)));

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

// ---- A not transposed: 64-row strip per work-group, waves interleaved along k -----------------
template <int NB, bool TB>
__global__ __launch_bounds__(64 * (NB <= 4 ? 16 : 4)) void skinny_n_kernel(SkinnyParams p) {
  constexpr int W = NB <= 4 ? 16 : 4;  // waves per work-group
  constexpr int U = 16;                // loads in flight per lane
  __shared__ float red[W][NB][64];
  const int lane = threadIdx.x & 63;
  // the wave index and everything derived from it (k, the addresses of B) are wave-uniform: saying so
  // lets B(k, j) be fetched with scalar loads instead of 64 identical vector loads
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = blockIdx.x * 64 + lane;
  const int split = blockIdx.y;
  const int n0 = blockIdx.z * NB;
  const int k_begin = split * p.k_per_split;
  const int k_end = min(p.K, k_begin + p.k_per_split);
  const float* __restrict__ a = p.A + min(m, p.M - 1);
  float acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) acc[j] = 0.f;
  int jc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) jc[j] = __builtin_amdgcn_readfirstlane(min(n0 + j, p.N - 1));

  // wave w owns the contiguous k range [kw_begin, kw_end): consecutive k keep the scalar loads of B
  // contiguous too (they merge into wide scalar loads)
  const int kc = (max(k_end - k_begin, 0) + W - 1) / W;
  const int kw_begin = k_begin + wave * kc, kw_end = min(k_end, kw_begin + kc);
  int k = kw_begin;
  for (; k + U <= kw_end; k += U) {
    float av[U];
#pragma unroll
    for (int u = 0; u < U; ++u) av[u] = a[(int64_t)(k + u) * p.lda];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[j] = fmaf(av[u], ld_b<TB>(p.B, p.ldb, k + u, jc[j]), acc[j]);
  }
  for (; k < kw_end; ++k) {
    const float av = a[(int64_t)k * p.lda];
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[j] = fmaf(av, ld_b<TB>(p.B, p.ldb, k, jc[j]), acc[j]);
  }
#pragma unroll
  for (int j = 0; j < NB; ++j) red[wave][j][lane] = acc[j];
  __syncthreads();
  // NB x 64 outputs, summed over the waves in wave order by the first NB*64 threads
  for (int o = threadIdx.x; o < NB * 64; o += 64 * W) {
    const int j = o >> 6, l = o & 63;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) s += red[w][j][l];
    const int mm = blockIdx.x * 64 + l;
    if (mm < p.M && n0 + j < p.N) skinny_store(p, split, mm, n0 + j, s);
  }
}

// ---- A transposed: wave per R rows, lanes along k ----------------------------------------------
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

  int k = k_begin;
  if (!TB) {
    // 16-byte loads: a wave covers 256 consecutive k per row and trip, two trips in flight
    for (; k + 512 <= k_end; k += 512) {
      floatx4 a0[R], a1[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        a0[r] = *reinterpret_cast<const floatx4u*>(arow[r] + k + 4 * lane);
        a1[r] = *reinterpret_cast<const floatx4u*>(arow[r] + k + 256 + 4 * lane);
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const float* bcol = p.B + (int64_t)jc[j] * p.ldb + k + 4 * lane;
        const floatx4 b0 = *reinterpret_cast<const floatx4u*>(bcol);
        const floatx4 b1 = *reinterpret_cast<const floatx4u*>(bcol + 256);
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[r][j] = fmaf(a0[r][e], b0[e], acc[r][j]);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[r][j] = fmaf(a1[r][e], b1[e], acc[r][j]);
        }
      }
    }
    for (; k + 256 <= k_end; k += 256) {
      floatx4 a0[R];
#pragma unroll
      for (int r = 0; r < R; ++r) a0[r] = *reinterpret_cast<const floatx4u*>(arow[r] + k + 4 * lane);
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const floatx4 b0 = *reinterpret_cast<const floatx4u*>(p.B + (int64_t)jc[j] * p.ldb + k + 4 * lane);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[r][j] = fmaf(a0[r][e], b0[e], acc[r][j]);
      }
    }
  }
  // scalar loads: transposed B, and the tail of the vector path
  k += lane;
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

// ---- matrix-core kernel for 5 .. 64 columns ----------------------------------------------------
// With more than a few columns the FMA kernels above run out of vector-ALU rate before they run out
// of bandwidth (NB FMAs per loaded float).  This kernel keeps their shape -- a strip of rows per
// work-group, the K range cut into contiguous parts over the W waves, partial sums added through
// LDS in wave order -- and does the arithmetic with v_mfma_f32_16x16x4_f32, which keeps 16 columns
// at a quarter of the issue slots:
//   D(16 x 16) += SrcA(16 x 4) * SrcB(4 x 16); lane l holds SrcA[i = l % 16][kk = l / 16],
//   SrcB[kk = l / 16][j = l % 16] and D[i = 4 * (l / 16) + r][j = l % 16], r = 0 .. 3.
// SrcA is fed from op(B) (i = column n of C), SrcB from op(A) (j = row m of C): D is a piece of C^T.
//   A not transposed: lane (j, kk) loads the four rows m0 + 4 j + b of column k + kk with one 16-byte
//     load (one wave load = 64 rows x 4 k = 1 KB contiguous per k); value b feeds block b.
//   A transposed: lane (j, kk) loads k + 4 kk .. + 3 of row m0 + j with one 16-byte load (16 rows x 16 k);
//     value t feeds step t, whose SrcA holds op(B)(k + 4 kk + t, n) -- any pairing of k with (step, kk)
//     is a valid order of summation as long as both operands use the same one.
// VEC = 16-byte loads allowed: always when A is transposed; when it is not, M % 4 == 0 is needed so that a
// 4-row group is inside or outside as a whole.  Alignment is not: the loads go through floatx4u.  Rows and columns past the edge are clamped for
// loads and skipped for stores; k past the end multiplies zeros.

template <bool TA, bool TB, int NBK, bool VEC>
__global__ __launch_bounds__(64 * (NBK == 1 ? 16 : 8)) void thin_mfma_kernel(SkinnyParams p) {
  constexpr int W = NBK == 1 ? 16 : 8;  // waves per work-group
  constexpr int U = 8;                  // 16-byte loads of A in flight per lane (16 spill and run slower)
  constexpr int ROWS = TA ? 16 : 64;    // rows of C per work-group
  constexpr int MB = TA ? 1 : 4;        // 16-row blocks per wave
  constexpr int KU = TA ? 16 : 4;       // k covered by one wave load
  __shared__ float red[W][NBK * MB * 4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, kk = lane >> 4;
  const int m0 = blockIdx.x * ROWS;
  const int split = blockIdx.y;
  const int n0 = blockIdx.z * (16 * NBK);
  const int k_begin = split * p.k_per_split;
  const int k_end = min(p.K, k_begin + p.k_per_split);
  // wave w owns [kw_begin, kw_end), a multiple of 16 long (keeps 16-byte loads along k aligned)
  const int kc = ((max(k_end - k_begin, 0) + W - 1) / W + 15) / 16 * 16;
  const int kw_begin = min(k_end, k_begin + wave * kc), kw_end = min(k_end, kw_begin + kc);

  int ncol[NBK];
#pragma unroll
  for (int nb = 0; nb < NBK; ++nb) ncol[nb] = min(n0 + 16 * nb + j, p.N - 1);
  // first row this lane loads (clamped so that every load stays inside A)
  const int mrow = TA ? min(m0 + j, p.M - 1) : (VEC ? min(m0 + 4 * j, p.M - 4) : m0 + 4 * j);

  floatx4 acc[NBK][MB];
#pragma unroll
  for (int nb = 0; nb < NBK; ++nb)
#pragma unroll
    for (int b = 0; b < MB; ++b) acc[nb][b] = floatx4{0.f, 0.f, 0.f, 0.f};

  // one wave load of A and the matching values of op(B), at k offset k0 of this lane's chunk; `guard`
  // (tail only) zero-fills k >= kw_end
  auto load_a = [&](int k0, bool guard) __attribute__((always_inline)) -> floatx4 {
    floatx4 a;
    if constexpr (TA) {
      const int k = k0 + 4 * kk;
      const float* src = p.A + (int64_t)k + (int64_t)mrow * p.lda;
      if (VEC && !guard) return *reinterpret_cast<const floatx4u*>(src);
#pragma unroll
      for (int t = 0; t < 4; ++t) a[t] = (k + t < kw_end) ? src[t] : 0.f;
    } else {
      const int k = k0 + kk;
      const bool in = k < kw_end;
      const float* src = p.A + (int64_t)mrow + (int64_t)min(k, p.K - 1) * p.lda;
      if constexpr (VEC) {
        a = *reinterpret_cast<const floatx4u*>(src);
        if (guard && !in) a = floatx4{0.f, 0.f, 0.f, 0.f};
      } else {
#pragma unroll
        for (int b = 0; b < 4; ++b) a[b] = in ? src[min(mrow + b, p.M - 1) - mrow] : 0.f;
      }
    }
    return a;
  };
  // op(B)(k, n) for the lane's k values: TA -> four consecutive k (steps t), else the single k of this lane
  auto load_b = [&](int k0, int nb, bool guard) __attribute__((always_inline)) -> floatx4 {
    floatx4 b = floatx4{0.f, 0.f, 0.f, 0.f};
    if constexpr (TA) {
      const int k = k0 + 4 * kk;
      if (!TB && VEC && !guard) return *reinterpret_cast<const floatx4u*>(p.B + (int64_t)k + (int64_t)ncol[nb] * p.ldb);
#pragma unroll
      for (int t = 0; t < 4; ++t) b[t] = (k + t < kw_end) ? ld_b<TB>(p.B, p.ldb, k + t, ncol[nb]) : 0.f;
    } else {
      const int k = k0 + kk;
      b[0] = (k < kw_end) ? ld_b<TB>(p.B, p.ldb, k, ncol[nb]) : 0.f;
    }
    return b;
  };
  auto multiply = [&](const floatx4& a, const floatx4 (&b)[NBK]) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < NBK; ++nb) {
      if constexpr (TA) {
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(b[nb][t], a[t], acc[nb][0], 0, 0, 0);
      } else {
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
          acc[nb][blk] = __builtin_amdgcn_mfma_f32_16x16x4f32(b[nb][0], a[blk], acc[nb][blk], 0, 0, 0);
      }
    }
  };

  int k = kw_begin;
  for (; k + U * KU <= kw_end; k += U * KU) {
    floatx4 av[U], bv[U][NBK];
#pragma unroll
    for (int u = 0; u < U; ++u) av[u] = load_a(k + u * KU, false);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int nb = 0; nb < NBK; ++nb) bv[u][nb] = load_b(k + u * KU, nb, false);
    // keep all loads of the trip in flight: without the fence the scheduler pairs every load with its
    // multiplications to save registers, and two loads per lane cannot cover the memory latency
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) multiply(av[u], bv[u]);
    __builtin_amdgcn_sched_barrier(0);
  }
  for (; k < kw_end; k += KU) {  // remaining wave loads one at a time; only the last can be partial
    const bool partial = k + KU > kw_end;
    floatx4 bv[NBK];
    const floatx4 av = load_a(k, partial);
#pragma unroll
    for (int nb = 0; nb < NBK; ++nb) bv[nb] = load_b(k, nb, partial);
    multiply(av, bv);
  }

  // partial sums of the W waves -> LDS, added in wave order
#pragma unroll
  for (int nb = 0; nb < NBK; ++nb)
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[wave][(nb * MB + b) * 4 + r][lane] = acc[nb][b][r];
  __syncthreads();
  for (int o = threadIdx.x; o < NBK * MB * 4 * 64; o += 64 * W) {
    const int a = o >> 6, l = o & 63;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) s += red[w][a][l];
    const int r = a & 3, b = (a >> 2) % MB, nb = a / (4 * MB);
    const int n = n0 + 16 * nb + 4 * (l >> 4) + r;
    const int m = TA ? m0 + (l & 15) : m0 + 4 * (l & 15) + b;
    if (m < p.M && n < p.N) skinny_store(p, split, m, n, s);
  }
}

template <int NBK>
static int launch_mfma_cfg(int split_k, const GemmArgs& g) {
  SkinnyParams p;
  p.A = g.A, p.B = g.B, p.C = g.C, p.ws = g.ws;
  p.lda = g.lda, p.ldb = g.ldb, p.ldc = g.ldc;
  p.M = (int)g.M, p.N = (int)g.N, p.K = (int)g.K;
  p.split_k = split_k;
  p.k_per_split = (int)((((g.K + split_k - 1) / split_k) + 15) / 16 * 16);  // slices start at multiples of 16
  p.alpha = g.alpha, p.beta = g.beta;
  // 16-byte loads: along k for A transposed (always possible), along m for A not transposed (then a 4-row
  // group must not straddle the edge)
  const bool vec = g.tA ? true : ((g.M & 3) == 0 && g.M >= 4);
  const int64_t col_groups = (g.N + 16 * NBK - 1) / (16 * NBK);
  const int64_t strips = (g.M + (g.tA ? 15 : 63)) / (g.tA ? 16 : 64);
  if (col_groups > 65535 || split_k > 65535 || strips > 0x7fffffffLL) return MDG_ERR_LAUNCH;
  const dim3 grid((unsigned)strips, (unsigned)split_k, (unsigned)col_groups), block(64 * (NBK == 1 ? 16 : 8));
#define MDG_THIN(TA, TB)                                                                        \
  do {                                                                                          \
    if (vec) thin_mfma_kernel<TA, TB, NBK, true><<<grid, block, 0, stream_of(g)>>>(p);              \
    else thin_mfma_kernel<TA, TB, NBK, false><<<grid, block, 0, stream_of(g)>>>(p);                 \
  } while (0)
  if (g.tA) {
    if (g.tB) MDG_THIN(true, true);
    else MDG_THIN(true, false);
  } else {
    if (g.tB) MDG_THIN(false, true);
    else MDG_THIN(false, false);
  }
#undef MDG_THIN
  int st = check_launch();
  if (st != MDG_OK || split_k == 1) return st;
  return launch_splitk_reduce(split_k, g);
}

template <int NB>
static int launch_cfg(int split_k, const GemmArgs& g) {
  SkinnyParams p;
  p.A = g.A, p.B = g.B, p.C = g.C, p.ws = g.ws;
  p.lda = g.lda, p.ldb = g.ldb, p.ldc = g.ldc;
  p.M = (int)g.M, p.N = (int)g.N, p.K = (int)g.K;
  p.split_k = split_k;
  p.k_per_split = (int)((((g.K + split_k - 1) / split_k) + 3) / 4 * 4);
  p.alpha = g.alpha, p.beta = g.beta;
  const int64_t col_groups = (g.N + NB - 1) / NB;
  if (col_groups > 65535 || split_k > 65535) return MDG_ERR_LAUNCH;
  if (!g.tA) {
    constexpr int W = NB <= 4 ? 16 : 4;
    dim3 grid((unsigned)((g.M + 63) / 64), (unsigned)split_k, (unsigned)col_groups);
    if (g.tB) skinny_n_kernel<NB, true><<<grid, dim3(64 * W), 0, stream_of(g)>>>(p);
    else skinny_n_kernel<NB, false><<<grid, dim3(64 * W), 0, stream_of(g)>>>(p);
  } else {
    dim3 grid((unsigned)((g.M + 15) / 16), (unsigned)split_k, (unsigned)col_groups);
    if (g.tB) skinny_t_kernel<NB, true><<<grid, dim3(256), 0, stream_of(g)>>>(p);
    else skinny_t_kernel<NB, false><<<grid, dim3(256), 0, stream_of(g)>>>(p);
  }
  int st = check_launch();
  if (st != MDG_OK || split_k == 1) return st;
  return launch_splitk_reduce(split_k, g);
}

int launch_skinny(int cfg, int split_k, const GemmArgs& g) {
  switch (cfg) {
#define X(c, NB, MATRIX)                                                \
  case c:                                                               \
    return MATRIX ? launch_mfma_cfg<(MATRIX ? NB / 16 : 1)>(split_k, g) \
                  : launch_cfg<(MATRIX ? 1 : NB)>(split_k, g);
    MDG_SKINNY_CONFIGS(X)
#undef X
  }
  return MDG_ERR_BAD_VARIANT;
}

}  // namespace mdg
