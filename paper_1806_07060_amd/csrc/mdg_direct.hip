// Direct kernel: the generic member of the family, "covering all GEMM use-cases"
// (Section 2.3 of the paper) -- any sizes, any transposes, any leading
// dimensions and alignments, no helper passes.  fp32 FMAs on the vector ALUs,
// a 16 x 16 work-group whose threads each hold a TM x TN register tile of C.
//
// Thread (tx, ty) owns rows m0 + tx + 16*a and columns n0 + ty + 16*b, so that
// neighbouring lanes touch neighbouring rows: coalesced for a non-transposed A
// and for C (column-major).  Out-of-range rows/columns are clamped for loads and
// skipped for stores; the K tail is zero-filled.
#include "mdg_internal.h"
#include "mdg_variant_list.h"

namespace mdg {

struct DirectParams {
  const float* A;
  const float* B;
  float* C;
  int64_t lda, ldb, ldc;
  int M, N, K;
  int tiles_m;
  float alpha, beta;
};

template <bool T>
__device__ __forceinline__ float ld_op(const float* X, int64_t ld, int r, int k) {
  // op(X)(r, k): r is the non-contracted index.  T = stored with k contiguous.
  return T ? X[(int64_t)k + (int64_t)r * ld] : X[(int64_t)r + (int64_t)k * ld];
}

// A is "k-contiguous" when transposed; B is "k-contiguous" when NOT transposed.
template <int TM, int TN, bool LDS, bool TA, bool TB>
__global__ __launch_bounds__(256) void direct_kernel(DirectParams p) {
  constexpr int BM = 16 * TM, BN = 16 * TN, BK = 16;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  // one-dimensional grid (no 65535 limit on the tile count in N)
  const int m0 = (int)(blockIdx.x % (unsigned)p.tiles_m) * BM, n0 = (int)(blockIdx.x / (unsigned)p.tiles_m) * BN;
  float acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b) acc[a][b] = 0.f;

  if constexpr (!LDS) {
    int mrow[TM], ncol[TN];
#pragma unroll
    for (int a = 0; a < TM; ++a) mrow[a] = min(m0 + tx + 16 * a, p.M - 1);
#pragma unroll
    for (int b = 0; b < TN; ++b) ncol[b] = min(n0 + ty + 16 * b, p.N - 1);
    int k = 0;
    for (; k + 4 <= p.K; k += 4) {  // four k per trip: their loads are independent and overlap
      float av[4][TM], bv[4][TN];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int a = 0; a < TM; ++a) av[u][a] = ld_op<TA>(p.A, p.lda, mrow[a], k + u);
#pragma unroll
        for (int b = 0; b < TN; ++b) bv[u][b] = ld_op<!TB>(p.B, p.ldb, ncol[b], k + u);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b) acc[a][b] = fmaf(av[u][a], bv[u][b], acc[a][b]);
    }
    for (; k < p.K; ++k) {
      float av[TM], bv[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a) av[a] = ld_op<TA>(p.A, p.lda, mrow[a], k);
#pragma unroll
      for (int b = 0; b < TN; ++b) bv[b] = ld_op<!TB>(p.B, p.ldb, ncol[b], k);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
    }
  } else {
    __shared__ float As[BK][BM + 1];
    __shared__ float Bs[BK][BN + 1];
    const int t = threadIdx.x;
    for (int k0 = 0; k0 < p.K; k0 += BK) {
      // cooperative, coalesced along whichever index is contiguous in memory
#pragma unroll
      for (int e = t; e < BM * BK; e += 256) {
        int mi = TA ? e / BK : e % BM;
        int ki = TA ? e % BK : e / BM;
        int m = min(m0 + mi, p.M - 1), k = k0 + ki;
        As[ki][mi] = (k < p.K) ? ld_op<TA>(p.A, p.lda, m, k) : 0.f;
      }
#pragma unroll
      for (int e = t; e < BN * BK; e += 256) {
        int ni = TB ? e % BN : e / BK;
        int ki = TB ? e / BN : e % BK;
        int n = min(n0 + ni, p.N - 1), k = k0 + ki;
        Bs[ki][ni] = (k < p.K) ? ld_op<!TB>(p.B, p.ldb, n, k) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < BK; ++kk) {
        float av[TM], bv[TN];
#pragma unroll
        for (int a = 0; a < TM; ++a) av[a] = As[kk][tx + 16 * a];
#pragma unroll
        for (int b = 0; b < TN; ++b) bv[b] = Bs[kk][ty + 16 * b];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
      }
      __syncthreads();
    }
  }

  // all reads of the old C first (independent loads in flight), then scale and store
  float old[TM][TN];
  if (p.beta != 0.f) {
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int a = 0; a < TM; ++a) {
        const int m = min(m0 + tx + 16 * a, p.M - 1), n = min(n0 + ty + 16 * b, p.N - 1);
        old[a][b] = p.C[(int64_t)m + (int64_t)n * p.ldc];
      }
  }
#pragma unroll
  for (int b = 0; b < TN; ++b) {
    int n = n0 + ty + 16 * b;
    if (n >= p.N) continue;
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      int m = m0 + tx + 16 * a;
      if (m >= p.M) continue;
      float r = p.alpha * acc[a][b];
      if (p.beta != 0.f) r = fmaf(p.beta, old[a][b], r);
      p.C[(int64_t)m + (int64_t)n * p.ldc] = r;
    }
  }
}

template <int TM, int TN, bool LDS>
static int launch_cfg(const GemmArgs& g) {
  const int64_t tiles_m = (g.M + 16 * TM - 1) / (16 * TM), tiles_n = (g.N + 16 * TN - 1) / (16 * TN);
  if (tiles_m * tiles_n > 0x7fffffffLL) return MDG_ERR_LAUNCH;
  DirectParams p{g.A, g.B, g.C, g.lda, g.ldb, g.ldc, (int)g.M, (int)g.N, (int)g.K, (int)tiles_m, g.alpha, g.beta};
  dim3 grid((unsigned)(tiles_m * tiles_n));
  dim3 block(256);
  if (g.tA) {
    if (g.tB) direct_kernel<TM, TN, LDS, true, true><<<grid, block, 0, stream_of(g)>>>(p);
    else direct_kernel<TM, TN, LDS, true, false><<<grid, block, 0, stream_of(g)>>>(p);
  } else {
    if (g.tB) direct_kernel<TM, TN, LDS, false, true><<<grid, block, 0, stream_of(g)>>>(p);
    else direct_kernel<TM, TN, LDS, false, false><<<grid, block, 0, stream_of(g)>>>(p);
  }
  return check_launch();
}

int launch_direct(int cfg, const GemmArgs& g) {
  switch (cfg) {
#define X(c, TM, TN, L) \
  case c:               \
    return launch_cfg<TM, TN, (L) != 0>(g);
    MDG_DIRECT_CONFIGS(X)
#undef X
  }
  return MDG_ERR_BAD_VARIANT;
}

// ---- helper passes ---------------------------------------------------------------------------

__global__ __launch_bounds__(256) void scale_c_kernel(float* C, int64_t ldc, int M, int N, float beta) {
  int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)M * N) return;
  int m = (int)(e % M), n = (int)(e / M);
  float* c = C + (int64_t)m + (int64_t)n * ldc;
  *c = (beta == 0.f) ? 0.f : beta * *c;
}

int launch_scale_c(const GemmArgs& g) {
  if (g.beta == 1.f) return MDG_OK;
  int64_t total = g.M * g.N;
  scale_c_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream_of(g)>>>(g.C, g.ldc, (int)g.M, (int)g.N,
                                                                                   g.beta);
  return check_launch();
}

// Partial sums are added in slice order, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* ws, float* C, int64_t ldc, int M, int N,
                                                            int split_k, float alpha, float beta) {
  int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int64_t total = (int64_t)M * N;
  if (e >= total) return;
  int m = (int)(e % M), n = (int)(e / M);
  float* c = C + (int64_t)m + (int64_t)n * ldc;
  const float c0 = (beta != 0.f) ? *c : 0.f;  // issued first, needed last
  float s = 0.f;
  for (int i0 = 0; i0 < split_k; i0 += 8) {  // eight independent loads in flight, added in slice order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (i0 + u < split_k) ? ws[(int64_t)(i0 + u) * total + e] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  float r = alpha * s;
  if (beta != 0.f) r = fmaf(beta, c0, r);
  *c = r;
}

int launch_splitk_reduce(int split_k, const GemmArgs& g) {
  int64_t total = g.M * g.N;
  splitk_reduce_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream_of(g)>>>(
      g.ws, g.C, g.ldc, (int)g.M, (int)g.N, split_k, g.alpha, g.beta);
  return check_launch();
}

}  // namespace mdg
