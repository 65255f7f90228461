// Tiled matrix-core kernel: the specialised member of the family (Section 2.3
// of the paper: a tiled kernel that relies on data reuse in local memory).
// Unlike the "indirect" kernel described there it needs no pad/transpose helper
// passes: transposes are absorbed by the global->LDS load path and ragged
// edges by guarded loads on the border tiles only.
//
// Work decomposition (column-major C, M contiguous)
//   work-group : BM x BN tile of C, K range [k_begin, k_end) (one slice when split_k > 1)
//   wave       : WTM x WTN sub-tile, WTM = BM / WGM, WTN = BN / WGN, as FM x FN blocks of 32 x 32
//   wave group : WGK groups of WGM x WGN waves share the tile; group g multiplies rows
//                [g * BK / WGK, (g + 1) * BK / WGK) of every K step and the groups' partial
//                sums are added through LDS at the end, in group order (a split of K inside
//                the work-group: more waves per CU for small C without a second launch)
//   MFMA       : v_mfma_f32_32x32x2_f32 (true fp32 operands, fp32 accumulate).
//                The ROW operand of the instruction is fed from op(B) (index n), the
//                COLUMN operand from op(A) (index m), i.e. each block holds a 32 x 32
//                piece of C^T: the lane index then runs along m, the contiguous index
//                of C, and stores are full cache lines.
//   lane (h, p), h = lane / 32, p = lane % 32
//     operand registers: k = kk + h;  m_local = FM * p + b  (b = block),  n_local = FN * p + c
//       -> one ds_read of FM (resp. FN) consecutive floats feeds FM (FN) blocks
//     accumulator register r of block (c, b):  n_local = FN * (8 * (r / 4) + 4 * h + r % 4) + c,
//                                              m_local = FM * p + b
//       -> for fixed (c, r) the FM values of a lane are consecutive in m: one vector store.
//
// LDS: two stages of As[BK][BM + 4] and Bs[BK][BN + 4] (k-major rows, the
// non-contracted index contiguous).  Global loads are float4 along whichever
// index is contiguous in memory (also for operands that are only 4-byte
// aligned); operands stored with k contiguous are transposed on their way into
// LDS with four 4-byte writes per float4.  A half-wave holds sixteen
// neighbouring rows of two neighbouring 16-byte k pieces: with the +4 row
// padding the 64 lanes of each such write fall on 64 distinct banks, and each
// half-wave on 32 distinct banks modulo 32 (no bank conflicts, checked with the
// LDS conflict counter).  Cross-lane transposes that would
// allow 16-byte writes were built and measured slower: vector-ALU work inside
// this loop costs matrix-pipe time, LDS instructions do not.  One barrier
// per K step; global loads run two K steps ahead (two register sets), LDS stages
// alternate.
#include <type_traits>

#include "mdg_internal.h"
#include "mdg_variant_list.h"

namespace mdg {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
// Four consecutive floats at an address that is only 4-byte aligned (odd leading dimensions, offset base
// pointers).  The compiler turns a load through this type into one 16-byte load as well: global memory accepts
// any dword-aligned address for it.
typedef floatx4 floatx4u __attribute__((aligned(4)));
typedef floatx2 floatx2u __attribute__((aligned(4)));

// F consecutive floats of C (or of the split-K workspace) as one access; `aligned` says whether the address is
// a multiple of 4 * F bytes, otherwise the 4-byte-aligned vector types are used.
template <int F>
__device__ __forceinline__ void load_run(float (&dst)[F], const float* src, bool aligned) {
  if constexpr (F == 4) {
    const floatx4 v = aligned ? *reinterpret_cast<const floatx4*>(src) : floatx4(*reinterpret_cast<const floatx4u*>(src));
    dst[0] = v[0], dst[1] = v[1], dst[2] = v[2], dst[3] = v[3];
  } else if constexpr (F == 2) {
    const floatx2 v = aligned ? *reinterpret_cast<const floatx2*>(src) : floatx2(*reinterpret_cast<const floatx2u*>(src));
    dst[0] = v[0], dst[1] = v[1];
  } else {
    dst[0] = *src;
  }
}
template <int F>
__device__ __forceinline__ void store_run(float* dst, const float (&v)[F], bool aligned) {
  if constexpr (F == 4) {
    const floatx4 o = {v[0], v[1], v[2], v[3]};
    if (aligned) *reinterpret_cast<floatx4*>(dst) = o;
    else *reinterpret_cast<floatx4u*>(dst) = o;
  } else if constexpr (F == 2) {
    const floatx2 o = {v[0], v[1]};
    if (aligned) *reinterpret_cast<floatx2*>(dst) = o;
    else *reinterpret_cast<floatx2u*>(dst) = o;
  } else {
    dst[0] = v[0];
  }
}

struct TiledParams {
  const float* A;
  const float* B;
  float* C;
  float* ws;
  int64_t lda, ldb, ldc;
  int M, N, K;
  int Ma, Nb;  // rows of op(A) / columns of op(B) that may be loaded: M and N, or more when the operands are padded copies
  int tiles_m, tiles_n;
  int split_k, k_per_split;
  float alpha, beta;
  int a_vec, b_vec;  // 1 if float4 global loads of that operand are aligned
};

constexpr int kPad = 4;
constexpr int kGroupM = 8;  // tiles per group along M in the tile ordering

// Loads one BMN x BK operand tile into registers (float4 slots).
//   KMAJOR = stored with k contiguous:  X[k + mn * ld]   else   X[mn + k * ld]
// `inside` (work-group uniform) = whole tile in range: 16-byte loads, through the aligned or the 4-byte-aligned
// vector type (`aligned`, uniform too); otherwise element-wise guarded loads.
//   DIRECT = the interior loop moves this operand from global memory straight into LDS (no registers, no LDS
//            store instruction).  Such a load writes the 64 x 16 bytes of a wave to one contiguous kilobyte, so
//            the stage is laid out in pieces of 256 floats (whole rows of the tile, in slot order) kPad floats
//            apart instead of in padded rows; only for operands whose rows are contiguous in memory.
//   KMAP   = which lane of a wave loads which 16-byte piece of a k-contiguous operand (see coords)
template <int BMN, int BK, int NT, bool KMAJOR, bool DIRECT = false, int KMAP = 2>
struct OperandLoader {
  static constexpr int kSlots = BMN * BK / 4 / NT;
  static_assert(BMN * BK % (4 * NT) == 0, "tile must split evenly into float4 slots");
  static_assert(!(DIRECT && KMAJOR), "direct loads keep the memory order: rows of the non-contracted index only");
  static_assert(!DIRECT || (256 % BMN == 0 && NT % 64 == 0), "a wave load must cover whole rows");
  static constexpr int kPiece = 256 + kPad;         // floats from one wave load's kilobyte to the next
  static constexpr int kRowsPerPiece = 256 / BMN;    // (DIRECT) tile rows per piece
  // floats per LDS stage
  static constexpr int kStage = DIRECT ? (BMN * BK / 256) * kPiece : BK * (BMN + kPad);
  // float offset of row k (of a stage) in LDS; columns follow contiguously
  __host__ __device__ static constexpr int row_offset(int k) {
    return DIRECT ? (k / kRowsPerPiece) * kPiece + (k % kRowsPerPiece) * BMN : k * (BMN + kPad);
  }

  // Slot -> (non-contracted index, k) of the first of its four elements.
  //   MN-major: consecutive lanes run along mn (one k row per BMN/4 lanes).
  //   K-major : a wave covers 16 mn x 16 k, i.e. sixteen row pieces of 64 bytes, each four 16-byte pieces long;
  //             further waves / slots take the other 16-wide k chunks and mn ranges.  Which lane takes which
  //             piece decides how the wave's global load coalesces and on which banks its four transposing
  //             4-byte LDS writes per piece fall (bank = 16 * piece + 4 * e + row, modulo the bank count):
  //               KMAP 0: lanes 4 i .. 4 i + 3 the four pieces of row i (64 contiguous bytes per lane quad;
  //                       the two halves of a wave write the same banks modulo 32);
  //               KMAP 1: lanes 16 j .. 16 j + 15 piece j of the sixteen rows (every write on distinct banks);
  //               KMAP 2: lanes 2 i, 2 i + 1 of the first half-wave pieces 0, 1 of row i, of the second
  //                       half-wave pieces 2, 3 (32 contiguous bytes per lane pair; distinct banks).
  __device__ __forceinline__ static void coords(int slot, int tid, int& mn, int& k) {
    int v = tid + slot * NT;
    if (KMAJOR) {
      const int l = v & 63, chunk = v >> 6;
      const int piece = KMAP == 0 ? (l & 3) : KMAP == 1 ? (l >> 4) : (l & 1) + 2 * (l >> 5);
      const int row = KMAP == 0 ? (l >> 2) : KMAP == 1 ? (l & 15) : (l >> 1) & 15;
      k = (chunk % (BK / 16)) * 16 + piece * 4;
      mn = (chunk / (BK / 16)) * 16 + row;
    } else {
      mn = (v % (BMN / 4)) * 4;
      k = v / (BMN / 4);
    }
  }

  __device__ __forceinline__ static void load(floatx4 (&r)[kSlots], const float* __restrict__ X, int64_t ld, int mn0,
                                              int k0, int mn_lim, int k_lim, bool inside, bool aligned, int tid) {
    if (inside) {
      const float* src[kSlots];
#pragma unroll
      for (int s = 0; s < kSlots; ++s) {
        int mn, k;
        coords(s, tid, mn, k);
        mn += mn0;
        k += k0;
        src[s] = KMAJOR ? X + (int64_t)k + (int64_t)mn * ld : X + (int64_t)mn + (int64_t)k * ld;
      }
      if (aligned) {
#pragma unroll
        for (int s = 0; s < kSlots; ++s) r[s] = *reinterpret_cast<const floatx4*>(src[s]);
      } else {
#pragma unroll
        for (int s = 0; s < kSlots; ++s) r[s] = *reinterpret_cast<const floatx4u*>(src[s]);
      }
    } else {
      // border tiles and the K tail: a slot whose four elements are all in range still takes one 16-byte load
      // (most lanes of a border tile); only the slots that straddle or lie past an edge go element by element.
      // Nothing outside the logical matrix is ever read.
#pragma unroll
      for (int s = 0; s < kSlots; ++s) {
        int mn, k;
        coords(s, tid, mn, k);
        mn += mn0;
        k += k0;
        const bool whole = KMAJOR ? (mn < mn_lim && k + 3 < k_lim) : (k < k_lim && mn + 3 < mn_lim);
        floatx4 v;
        if (whole) {
          v = *reinterpret_cast<const floatx4u*>(KMAJOR ? X + (int64_t)k + (int64_t)mn * ld
                                                        : X + (int64_t)mn + (int64_t)k * ld);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            int mm = KMAJOR ? mn : mn + e;
            int kk = KMAJOR ? k + e : k;
            float x = 0.f;
            if (mm < mn_lim && kk < k_lim) x = KMAJOR ? X[(int64_t)kk + (int64_t)mm * ld] : X[(int64_t)mm + (int64_t)kk * ld];
            v[e] = x;
          }
        }
        r[s] = v;
      }
    }
  }

  // Lean path for interior tiles: one work-group-uniform base pointer that moves along K
  // (scalar registers) plus a fixed 32-bit byte offset per slot, so a K step costs no vector
  // ALU work for addressing.  Usable when every offset inside a tile fits in 31 bits.
  __device__ __forceinline__ static bool offsets_fit(int64_t ld) {
    return (KMAJOR ? (int64_t)BMN : (int64_t)BK) * ld * 4 < 0x7fffffffLL;
  }
  // `rows` < BMN: the operand ends inside the tile.  Slots past its end re-read its last row (its last four
  // rows when rows are contiguous along mn; `rows` must then be a multiple of four): what they bring in only
  // reaches elements of C that are never stored, and it is finite whenever the operand is.
  __device__ __forceinline__ static bool rows_clampable(int rows) { return KMAJOR || ((rows & 3) == 0 && rows >= 4); }
  __device__ __forceinline__ static void fast_offsets(uint32_t (&off)[kSlots], int64_t ld, int tid, int rows) {
#pragma unroll
    for (int s = 0; s < kSlots; ++s) {
      int mn, k;
      coords(s, tid, mn, k);
      mn = min(mn, rows - (KMAJOR ? 1 : 4));
      off[s] = (uint32_t)(4 * (KMAJOR ? (int64_t)k + (int64_t)mn * ld : (int64_t)mn + (int64_t)k * ld));
    }
  }
  __device__ __forceinline__ static const char* fast_base(const float* X, int64_t ld, int mn0, int k0) {
    return reinterpret_cast<const char*>(KMAJOR ? X + (int64_t)k0 + (int64_t)mn0 * ld : X + (int64_t)mn0 + (int64_t)k0 * ld);
  }
  __device__ __forceinline__ static int64_t fast_stride(int64_t ld) { return KMAJOR ? (int64_t)BK * 4 : (int64_t)BK * ld * 4; }
  template <bool ALIGNED>
  __device__ __forceinline__ static void fast_load(floatx4 (&r)[kSlots], const char* base, const uint32_t (&off)[kSlots]) {
#pragma unroll
    for (int s = 0; s < kSlots; ++s) {
      if constexpr (ALIGNED) r[s] = *reinterpret_cast<const floatx4*>(base + off[s]);
      else r[s] = *reinterpret_cast<const floatx4u*>(base + off[s]);
    }
  }

  // global memory -> LDS stage S, all slots, no registers (interior tiles, 16-byte aligned operands).  Lane i
  // of a wave writes bytes [16 i, 16 i + 16) of the piece; the piece address must be the same for all lanes.
  __device__ __forceinline__ static void direct_load(const char* base, const uint32_t (&off)[kSlots], float* S, int wave) {
#pragma unroll
    for (int s = 0; s < kSlots; ++s)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + off[s]),
                                       (__attribute__((address_space(3))) void*)(S + (wave + s * (NT / 64)) * kPiece),
                                       16, 0, 0);
  }

  // registers -> LDS stage S, one float4 slot
  __device__ __forceinline__ static void store_slot(const floatx4& r, float* S, int tid, int s) {
    constexpr int LD = BMN + kPad;
    if constexpr (DIRECT) {  // same place a direct load of this slot writes to
      const int v = tid + s * NT;
      *reinterpret_cast<floatx4*>(&S[(v >> 6) * kPiece + (v & 63) * 4]) = r;
      return;
    }
    int mn, k;
    coords(s, tid, mn, k);
    if (KMAJOR) {
#pragma unroll
      for (int e = 0; e < 4; ++e) S[(k + e) * LD + mn] = r[e];
    } else {
      *reinterpret_cast<floatx4*>(&S[k * LD + mn]) = r;
    }
  }
  __device__ __forceinline__ static void store(const floatx4 (&r)[kSlots], float* S, int tid) {
#pragma unroll
    for (int s = 0; s < kSlots; ++s) store_slot(r[s], S, tid, s);
  }
};

template <int F>
__device__ __forceinline__ void lds_read_frag(float (&dst)[F], const float* src) {
  if constexpr (F == 4) {
    floatx4 t = *reinterpret_cast<const floatx4*>(src);
    dst[0] = t[0], dst[1] = t[1], dst[2] = t[2], dst[3] = t[3];
  } else if constexpr (F == 2) {
    floatx2 t = *reinterpret_cast<const floatx2*>(src);
    dst[0] = t[0], dst[1] = t[1];
  } else {
    dst[0] = *src;
  }
}

// waves per SIMD the register allocation is held to (second __launch_bounds__ argument): two
// unless one wave's accumulators alone need more than half of the 512-register file
template <int BM, int BN, int WGM, int WGN>
constexpr int min_waves_per_simd() {
  return (BM * BN / (WGM * WGN) > 128 * 64) ? 1 : 2;
}

// DLDS: operands whose rows are contiguous in memory (A not transposed, B transposed) go from global memory
// straight into LDS in the interior loop; the others, and every border tile, take the register path.
template <int BM, int BN, int BK, int WGM, int WGN, int WGK, bool TA, bool TB, bool DLDS = false, int KMAP = 2>
__global__ __launch_bounds__(64 * WGM * WGN * WGK, (min_waves_per_simd<BM, BN, WGM, WGN>()))
void tiled_kernel(TiledParams p) {
  constexpr int NT = 64 * WGM * WGN * WGK;
  constexpr int BKW = BK / WGK;  // rows of a K step one wave group multiplies
  static_assert(BK % WGK == 0 && BKW % 2 == 0 && BKW >= 4, "each wave group needs whole pairs of k rows");
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int FM = WTM / 32, FN = WTN / 32;
  static_assert(FM == 1 || FM == 2 || FM == 4, "wave tile rows must be 32, 64 or 128");
  static_assert(FN == 1 || FN == 2 || FN == 4, "wave tile columns must be 32, 64 or 128");
  static_assert(!DLDS || WGK == 1, "direct-to-LDS loads are built for one wave group");
  constexpr bool DA = DLDS && !TA, DB = DLDS && TB;
  // A is k-contiguous when transposed; B is k-contiguous when not transposed.
  using LoadA = OperandLoader<BM, BK, NT, TA, DA, KMAP>;
  using LoadB = OperandLoader<BN, BK, NT, !TB, DB, KMAP>;
  constexpr int A_STAGE = LoadA::kStage, B_STAGE = LoadB::kStage;

  __shared__ __attribute__((aligned(16))) float lds[2 * (A_STAGE + B_STAGE)];
  static_assert((WGK - 1) * BM * BN <= 2 * (A_STAGE + B_STAGE), "the partial sums of the wave groups must fit the stages");
  float* As = lds;
  float* Bs = lds + 2 * A_STAGE;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);  // the same number, known to be wave-uniform
  const int h = lane >> 5, pl = lane & 31;
  const int kg = wave / (WGM * WGN), wq = wave % (WGM * WGN);
  const int wm = wq % WGM, wn = wq / WGM;

  // ---- which tile: undo the round-robin of work-groups over the 8 XCDs so that each
  // XCD (own L2) works on a compact block of neighbouring tiles, then walk the tiles in
  // groups of kGroupM rows.
  const int tiles = p.tiles_m * p.tiles_n;
  int bid = blockIdx.x;
  const int split = bid / tiles;
  bid -= split * tiles;
  {
    const int per = (tiles + 7) >> 3, rem = tiles & 7, xcd = bid & 7, loc = bid >> 3;
    bid = (rem == 0 || xcd < rem) ? xcd * per + loc : rem * per + (xcd - rem) * (per - 1) + loc;
  }
  const int group_sz = kGroupM * p.tiles_n;
  const int group = bid / group_sz;
  const int first_m = group * kGroupM;
  const int gm = min(p.tiles_m - first_m, kGroupM);
  const int in_group = bid - group * group_sz;
  const int tile_m = first_m + in_group % gm;
  const int tile_n = in_group / gm;
  // The tile stores rows [ms, ms + BM) and columns [ns, ns + BN) of C.  A border tile of a matrix that is at
  // least one tile tall (wide) is moved back so that it ends exactly at the edge: it then loads whole tiles like
  // an interior one (no guarded loads along the whole K range, which cost a large tile most of its speed); the
  // rows (columns) below ms (ns) it computes on the way belong to its neighbour and are not stored.
  const int ms = tile_m * BM, ns = tile_n * BN;
  const int m0 = (ms + BM > p.Ma && p.Ma >= BM) ? p.Ma - BM : ms;
  const int n0 = (ns + BN > p.Nb && p.Nb >= BN) ? p.Nb - BN : ns;

  const int k_begin = split * p.k_per_split;
  const int k_end = min(p.K, k_begin + p.k_per_split);
  const int n_steps = (k_end - k_begin + BK - 1) / BK;

  const bool a_full = (m0 + BM <= p.Ma), b_full = (n0 + BN <= p.Nb);  // tile inside the operand along m / n
  // 16-byte loads of that operand are aligned (a moved tile of a row-contiguous operand may start off the grid)
  const bool a_al = p.a_vec != 0 && (TA || (m0 & 3) == 0), b_al = p.b_vec != 0 && (!TB || (n0 & 3) == 0);

  floatx16 acc[FN][FM];
#pragma unroll
  for (int c = 0; c < FN; ++c)
#pragma unroll
    for (int b = 0; b < FM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[c][b][r] = 0.f;

  // Wave tiles with little matrix work per K step (at most 32 MFMAs, about 2000 cycles) prefetch two K steps
  // ahead through two register sets per operand: while step t runs on LDS stage t & 1, the tile of step t+1
  // sits in set (t+1) & 1 (loaded during step t-1) and the loads of step t+2 go to set t & 1.  Two steps of
  // matrix work then cover the global-memory latency, which keeps shapes with only one or two work-groups per
  // CU from being latency-bound.  Larger steps have 4000+ cycles of MFMAs to hide behind and no registers to
  // spare (a second set pushed some instantiations into spilling inside the interior loop): one set, one
  // step ahead.
  constexpr int NS = (FM * FN * (BKW / 2) <= 32 && !DLDS) ? 2 : 1;
  floatx4 ra[NS][LoadA::kSlots], rb[NS][LoadB::kSlots];

  auto load_guarded = [&](int ti, floatx4 (&qa)[LoadA::kSlots], floatx4 (&qb)[LoadB::kSlots])
                          __attribute__((always_inline)) {
    if (ti < n_steps) {
      const int k0 = k_begin + ti * BK;
      const bool kfull = (k0 + BK <= k_end);
      LoadA::load(qa, p.A, p.lda, m0, k0, p.Ma, k_end, a_full && kfull, a_al, tid);
      LoadB::load(qb, p.B, p.ldb, n0, k0, p.Nb, k_end, b_full && kfull, b_al, tid);
    }
  };

  if (n_steps > 0) {
    load_guarded(0, ra[0], rb[0]);
    LoadA::store(ra[0], As, tid);
    LoadB::store(rb[0], Bs, tid);
    if constexpr (NS == 2) load_guarded(1, ra[1], rb[1]);
  }
  __syncthreads();

  // row kk + h of a stage sits at row_offset(kk) + row_offset(h) for even kk (a piece holds an even number of
  // rows, or one); the wave group's first row kg * BKW is even as well
  const float* a_rd = As + (kg * LoadA::row_offset(BKW) + h * LoadA::row_offset(1)) + wm * WTM + FM * pl;
  const float* b_rd = Bs + (kg * LoadB::row_offset(BKW) + h * LoadB::row_offset(1)) + wn * WTN + FN * pl;
  static_assert(WGK == 1 || (!DA && !DB), "row_offset is linear only for the padded-row layout");

  // One K step on LDS stage BUF.  Schedule (pinned with scheduling barriers):
  //   - operand registers are double-buffered: the LDS reads of sub-step kk+2 are issued before
  //     the MFMAs of sub-step kk, so their latency hides behind FM*FN matrix instructions;
  //   - the global loads of the step after next are issued once the first block of MFMAs is queued;
  //   - the LDS stores of the next step (other stage, other register set) are spread over the last
  //     sub-steps, one float4 slot of each operand per sub-step, so that the LDS writes issue in the
  //     shadow of that sub-step's MFMAs instead of in one clump in front of the barrier.
  // `load_ahead(set_a, set_b)` issues the loads, `have_next` says whether there is anything to store.
  // `direct_tag`: this step's load_ahead moves the direct operands into the other stage by itself (interior
  // loop of a DLDS kernel); their register -> LDS stores are then left out and the loads are awaited before the
  // barrier, which publishes them to the other waves.
  auto k_step = [&](auto buf_tag, auto&& load_ahead, bool have_next, auto direct_tag_t) __attribute__((always_inline)) {
    constexpr int BUF = decltype(buf_tag)::value;
    constexpr bool direct_tag = decltype(direct_tag_t)::value;
    const float* a_s = a_rd + BUF * A_STAGE;
    const float* b_s = b_rd + BUF * B_STAGE;
    float af[2][FM], bf[2][FN];
    lds_read_frag<FM>(af[0], a_s);
    lds_read_frag<FN>(bf[0], b_s);
#pragma unroll
    for (int kk = 0; kk < BKW; kk += 2) {
      const int cur = (kk >> 1) & 1;
      if (kk + 2 < BKW) {
        lds_read_frag<FM>(af[cur ^ 1], a_s + LoadA::row_offset(kk + 2));
        lds_read_frag<FN>(bf[cur ^ 1], b_s + LoadB::row_offset(kk + 2));
      }
      constexpr int LS = (NS == 2) ? BUF : 0, SS = (NS == 2) ? (BUF ^ 1) : 0;  // load-target / store-source set
      if (kk == 2) load_ahead(ra[LS], rb[LS], As + (BUF ^ 1) * A_STAGE, Bs + (BUF ^ 1) * B_STAGE);
      if (have_next) {
        constexpr int NSUB = BKW / 2;
        static_assert(LoadA::kSlots <= NSUB - 1 && LoadB::kSlots <= NSUB - 1, "one slot per sub-step after the loads");
        const int sa = (kk >> 1) - (NSUB - LoadA::kSlots), sb = (kk >> 1) - (NSUB - LoadB::kSlots);
        if (sa >= 0 && !(DA && direct_tag)) LoadA::store_slot(ra[SS][sa], As + (BUF ^ 1) * A_STAGE, tid, sa);
        if (sb >= 0 && !(DB && direct_tag)) LoadB::store_slot(rb[SS][sb], Bs + (BUF ^ 1) * B_STAGE, tid, sb);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < FN; ++c)
#pragma unroll
        for (int b = 0; b < FM; ++b)
          acc[c][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(bf[cur][c], af[cur][b], acc[c][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (direct_tag && (DA || DB)) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the direct loads have landed
    __syncthreads();
  };
  using Buf0 = std::integral_constant<int, 0>;
  using Buf1 = std::integral_constant<int, 1>;

  int t = 0;
  // ---- interior tiles: K steps whose second successor is a full tile use the lean loads (one instance of the
  // loop for aligned operands, one that goes through the 4-byte-aligned vector type for everything else)
  // An operand with fewer rows than the tile takes them too when the missing rows can be stood in for.
  const int rows_a = min(BM, p.Ma - m0), rows_b = min(BN, p.Nb - n0);
  const int n_full = (LoadA::rows_clampable(rows_a) && LoadB::rows_clampable(rows_b) && LoadA::offsets_fit(p.lda) &&
                      LoadB::offsets_fit(p.ldb))
                         ? (k_end - k_begin) / BK : 0;
  if (n_full > NS + 1) {
    uint32_t offa[LoadA::kSlots], offb[LoadB::kSlots];
    LoadA::fast_offsets(offa, p.lda, tid, rows_a);
    LoadB::fast_offsets(offb, p.ldb, tid, rows_b);
    const char* pa = LoadA::fast_base(p.A, p.lda, m0, k_begin + NS * BK);
    const char* pb = LoadB::fast_base(p.B, p.ldb, n0, k_begin + NS * BK);
    const int64_t sa = LoadA::fast_stride(p.lda), sb = LoadB::fast_stride(p.ldb);
    auto interior = [&](auto aligned_tag) __attribute__((always_inline)) {
      constexpr bool AL = decltype(aligned_tag)::value;
      // operands that go straight to LDS need 16-byte aligned addresses; without them the kernel still works,
      // through the register path
      constexpr bool DIRECT_NOW = AL && (DA || DB);
      auto lean = [&](floatx4 (&qa)[LoadA::kSlots], floatx4 (&qb)[LoadB::kSlots], float* sa_next, float* sb_next)
                      __attribute__((always_inline)) {
        if constexpr (DIRECT_NOW && DA) LoadA::direct_load(pa, offa, sa_next, wave_u);
        else LoadA::template fast_load<AL>(qa, pa, offa);
        if constexpr (DIRECT_NOW && DB) LoadB::direct_load(pb, offb, sb_next, wave_u);
        else LoadB::template fast_load<AL>(qb, pb, offb);
        pa += sa;
        pb += sb;
      };
      for (; t + NS + 1 < n_full; t += 2) {  // loads tiles t+NS and t+NS+1, both full
        k_step(Buf0{}, lean, true, std::integral_constant<bool, DIRECT_NOW>{});
        k_step(Buf1{}, lean, true, std::integral_constant<bool, DIRECT_NOW>{});
      }
    };
    if (a_al && b_al) interior(std::true_type{});
    else interior(std::false_type{});
  }
  // ---- everything else (edge tiles, unaligned operands, the K tail): guarded loads
  for (; t < n_steps; ++t) {
    auto guarded = [&](floatx4 (&qa)[LoadA::kSlots], floatx4 (&qb)[LoadB::kSlots], float*, float*)
                       __attribute__((always_inline)) { load_guarded(t + NS, qa, qb); };
    if (t & 1) k_step(Buf1{}, guarded, t + 1 < n_steps, std::false_type{});
    else k_step(Buf0{}, guarded, t + 1 < n_steps, std::false_type{});
  }

  // ---- partial sums of wave groups 1 .. WGK-1 go through LDS (the stages are free after the last
  // barrier of the K loop) and are added by group 0 in group order; only group 0 writes C
  if constexpr (WGK > 1) {
    constexpr int PER_WAVE = FN * FM * 16 * 64;
    if (kg > 0) {
      float* dst = lds + ((kg - 1) * (WGM * WGN) + wq) * PER_WAVE + lane;
#pragma unroll
      for (int c = 0; c < FN; ++c)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) dst[((c * FM + b) * 16 + r) * 64] = acc[c][b][r];
    }
    __syncthreads();
    if (kg > 0) return;
#pragma unroll
    for (int g2 = 1; g2 < WGK; ++g2) {
      const float* src = lds + ((g2 - 1) * (WGM * WGN) + wq) * PER_WAVE + lane;
#pragma unroll
      for (int c = 0; c < FN; ++c)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[c][b][r] += src[((c * FM + b) * 16 + r) * 64];
    }
  }

  // ---- epilogue
  const int m_base = m0 + wm * WTM + FM * pl;
  const int n_wave = n0 + wn * WTN;
  if (p.split_k > 1) {
    // raw partial sums into slice `split` of the workspace (tight column-major M x N)
    float* W = p.ws + (int64_t)split * p.M * p.N;
    const bool vec = (FM > 1) && (m_base >= ms) && (m_base + FM <= p.M);  // the lane's FM rows are all this tile's
    const bool w_al = ((p.M | m0) & 3) == 0;             // slices are 256-byte aligned, columns M floats apart
#pragma unroll
    for (int c = 0; c < FN; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int n = n_wave + FN * (8 * (r >> 2) + 4 * h + (r & 3)) + c;
        if (n < ns || n >= p.N) continue;
        float* dst = W + (int64_t)m_base + (int64_t)n * p.M;
        if (vec) {
          float o[FM];
#pragma unroll
          for (int b = 0; b < FM; ++b) o[b] = acc[c][b][r];
          store_run<FM>(dst, o, w_al);
        } else {
#pragma unroll
          for (int b = 0; b < FM; ++b)
            if (m_base + b >= ms && m_base + b < p.M) dst[b] = acc[c][b][r];
        }
      }
    return;
  }

  const bool c_al = (((p.ldc | m0) & 3) == 0) && ((reinterpret_cast<uintptr_t>(p.C) & 15) == 0);
  const bool vec = (FM > 1) && (m_base >= ms) && (m_base + FM <= p.M);  // the lane's FM rows are all this tile's
  const float alpha = p.alpha, beta = p.beta;
  // Per block column c: first all reads of the old C (16 independent loads in flight per lane --
  // read-then-write one row at a time would pay the memory latency sixteen times), then scale and store.
#pragma unroll
  for (int c = 0; c < FN; ++c) {
    float old[16][FM];
    if (beta != 0.f) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int n = n_wave + FN * (8 * (r >> 2) + 4 * h + (r & 3)) + c;
        const float* src = p.C + (int64_t)m_base + (int64_t)min(n, p.N - 1) * p.ldc;
        if (vec) {
          load_run<FM>(old[r], src, c_al);
        } else {
#pragma unroll
          for (int b = 0; b < FM; ++b) old[r][b] = (m_base + b < p.M) ? src[b] : 0.f;
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int n = n_wave + FN * (8 * (r >> 2) + 4 * h + (r & 3)) + c;
      if (n < ns || n >= p.N) continue;
      float* dst = p.C + (int64_t)m_base + (int64_t)n * p.ldc;
      float o[FM];
#pragma unroll
      for (int b = 0; b < FM; ++b) {
        o[b] = alpha * acc[c][b][r];
        if (beta != 0.f) o[b] = fmaf(beta, old[r][b], o[b]);
      }
      if (vec) {
        store_run<FM>(dst, o, c_al);
      } else {
#pragma unroll
        for (int b = 0; b < FM; ++b)
          if (m_base + b >= ms && m_base + b < p.M) dst[b] = o[b];
      }
    }
  }
}

template <int BM, int BN, int BK, int WGM, int WGN, int WGK, bool DLDS, int KMAP>
static int launch_cfg(int split_k, const GemmArgs& g, int64_t a_rows, int64_t b_cols) {
  TiledParams p;
  p.A = g.A, p.B = g.B, p.C = g.C, p.ws = g.ws;
  p.lda = g.lda, p.ldb = g.ldb, p.ldc = g.ldc;
  p.M = (int)g.M, p.N = (int)g.N, p.K = (int)g.K;
  p.Ma = (int)(a_rows > g.M ? a_rows : g.M), p.Nb = (int)(b_cols > g.N ? b_cols : g.N);
  const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  if (tiles_m * tiles_n * split_k > 0x7fffffffLL) return MDG_ERR_LAUNCH;
  p.tiles_m = (int)tiles_m, p.tiles_n = (int)tiles_n;
  p.split_k = split_k;
  const int64_t k_steps = (g.K + BK - 1) / BK;
  p.k_per_split = (int)(((k_steps + split_k - 1) / split_k) * BK);
  p.alpha = g.alpha, p.beta = g.beta;
  p.a_vec = ((g.lda & 3) == 0) && ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0);
  p.b_vec = ((g.ldb & 3) == 0) && ((reinterpret_cast<uintptr_t>(g.B) & 15) == 0);
  dim3 grid((unsigned)(tiles_m * tiles_n * split_k)), block(64 * WGM * WGN * WGK);
  if (g.tA) {
    if (g.tB) tiled_kernel<BM, BN, BK, WGM, WGN, WGK, true, true, DLDS, KMAP><<<grid, block, 0, stream_of(g)>>>(p);
    else tiled_kernel<BM, BN, BK, WGM, WGN, WGK, true, false, DLDS, KMAP><<<grid, block, 0, stream_of(g)>>>(p);
  } else {
    if (g.tB) tiled_kernel<BM, BN, BK, WGM, WGN, WGK, false, true, DLDS, KMAP><<<grid, block, 0, stream_of(g)>>>(p);
    else tiled_kernel<BM, BN, BK, WGM, WGN, WGK, false, false, DLDS, KMAP><<<grid, block, 0, stream_of(g)>>>(p);
  }
  int st = check_launch();
  if (st != MDG_OK || split_k == 1) return st;
  return launch_splitk_reduce(split_k, g);
}

int launch_tiled(int cfg, int split_k, const GemmArgs& g, int64_t a_rows, int64_t b_cols) {
  switch (cfg) {
#define X(c, BM, BN, BK, WGM, WGN, WGK, DLDS, KMAP) \
  case c:                                           \
    return launch_cfg<BM, BN, BK, WGM, WGN, WGK, (DLDS) != 0, KMAP>(split_k, g, a_rows, b_cols);
    MDG_TILED_CONFIGS(X)
#undef X
  }
  return MDG_ERR_BAD_VARIANT;
}

}  // namespace mdg
