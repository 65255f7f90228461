// Indirect path (Section 2.3 of the paper): O(n^2) helper passes bring op(A) and op(B) into the form the tiled
// kernel handles best, then the O(n^3) kernel runs under assumptions the helpers have established -- no ragged
// tiles, no K tail, no transposed operand.  The paper's library pays that price to keep its tiled kernel simple;
// here the tiled kernel copes with everything by itself, so the indirect variants exist to *measure* the
// trade-off on this chip: helpers + assumption-heavy kernel against one generic launch.
//
// Packed form (in the registered workspace, never in the caller's buffers):
//   Ap[k][m] = op(A)(m, k)   Kp rows of Mp floats   (the non-contracted index contiguous)
//   Bp[k][n] = op(B)(k, n)   Kp rows of Np floats
// with Mp, Np, Kp = M, N, K rounded up to whole tiles / K steps and zeros in the padding (a zero adds nothing to
// a sum, so results are those of the unpadded product).  That is the "A not transposed, B transposed"
// column-major case of the tiled kernel with leading dimensions Mp and Np: its interior loop loads 16-byte
// vectors straight along LDS rows, never transposes on the way into LDS and never takes the guarded path.
// C is not packed: the epilogue already writes only rows < M and columns < N.
// An operand that already has the packed form (stored with the non-contracted index contiguous, extents whole
// tiles) is used where it lies, without a copy.
#include "mdg_internal.h"
#include "mdg_variant_list.h"

namespace mdg {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Source stored with the non-contracted index contiguous: X[mn + k * ld].  One thread per four consecutive mn.
__global__ __launch_bounds__(256) void pack_rows_kernel(const float* __restrict__ X, int64_t ld, int MN, int K,
                                                        float* __restrict__ P, int MNp, int Kp) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;  // float4 slot of P
  const int per_row = MNp >> 2;
  if (q >= (int64_t)per_row * Kp) return;
  const int k = (int)(q / per_row), mn = (int)(q % per_row) * 4;
  floatx4 v = {0.f, 0.f, 0.f, 0.f};
  if (k < K) {
    const float* src = X + (int64_t)mn + (int64_t)k * ld;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (mn + e < MN) v[e] = src[e];
  }
  *reinterpret_cast<floatx4*>(P + (int64_t)mn + (int64_t)k * MNp) = v;
}

// Source stored with k contiguous: X[k + mn * ld].  A work-group transposes a 64 (mn) x 64 (k) block through LDS:
// reads run along k, writes along mn, both in whole cache lines.
__global__ __launch_bounds__(256) void pack_transpose_kernel(const float* __restrict__ X, int64_t ld, int MN, int K,
                                                             float* __restrict__ P, int MNp, int Kp) {
  __shared__ float tile[64][65];
  const int blocks_mn = MNp >> 6;
  const int mn0 = (int)(blockIdx.x % blocks_mn) * 64, k0 = (int)(blockIdx.x / blocks_mn) * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int mn = mn0 + ty + 4 * r, k = k0 + tx;
    tile[ty + 4 * r][tx] = (mn < MN && k < K) ? X[(int64_t)k + (int64_t)mn * ld] : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int k = k0 + ty + 4 * r, mn = mn0 + tx;
    if (k < Kp) P[(int64_t)mn + (int64_t)k * MNp] = tile[tx][ty + 4 * r];
  }
}

static int pack(const float* X, int64_t ld, bool k_contiguous, int64_t MN, int64_t K, float* P, int64_t MNp, int64_t Kp,
                hipStream_t s) {
  if (k_contiguous) {
    const int64_t blocks = (MNp / 64) * ((Kp + 63) / 64);
    if (blocks > 0x7fffffffLL) return MDG_ERR_LAUNCH;
    pack_transpose_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(X, ld, (int)MN, (int)K, P, (int)MNp, (int)Kp);
  } else {
    const int64_t blocks = ((MNp / 4) * Kp + 255) / 256;
    if (blocks > 0x7fffffffLL) return MDG_ERR_LAUNCH;
    pack_rows_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(X, ld, (int)MN, (int)K, P, (int)MNp, (int)Kp);
  }
  return check_launch();
}

int launch_indirect(int tiled_cfg, int tile_m, int tile_n, int tile_k, const GemmArgs& g) {
  const IndirectPlan p = plan_indirect(tile_m, tile_n, tile_k, g.tA, g.tB, g.M, g.N, g.K);
  if ((p.a_floats + p.b_floats) * sizeof(float) > g.ws_bytes) return MDG_ERR_WORKSPACE;
  GemmArgs t = g;
  float* ws = g.ws;
  if (p.pack_a) {
    int st = pack(g.A, g.lda, g.tA != 0, g.M, g.K, ws, p.Mp, p.Kp, stream_of(g));
    if (st != MDG_OK) return st;
    t.A = ws, t.lda = p.Mp, t.tA = 0;
    ws += p.a_floats;
  }
  if (p.pack_b) {
    int st = pack(g.B, g.ldb, g.tB == 0, g.N, g.K, ws, p.Np, p.Kp, stream_of(g));
    if (st != MDG_OK) return st;
    t.B = ws, t.ldb = p.Np, t.tB = 1;
  }
  t.K = p.Kp;
  t.ws = nullptr, t.ws_bytes = 0;
  // the tiled kernel on the packed operands: operand extents are the padded ones, C keeps its own
  return launch_tiled(tiled_cfg, 1, t, p.Mp, p.Np);
}

}  // namespace mdg
