// Host-side declarations of libmdg_sgemm.so that need no GPU runtime: the column-major problem a call is
// canonicalised to (Eq. 1, Section 2.2 of the paper), the variant table, legality (Section 4.1) and the selectors
// (Section 3, 'Model and code generation').  mdg_dispatch.cpp implements them in plain C++, so this part of the
// library can be built and run on a machine without a GPU (host tests, sanitizer build).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "../../include/mdg_sgemm.h"

namespace mdg {

struct GemmArgs {
  int tA, tB;  // 0 / 1, column-major problem
  int64_t M, N, K;
  float alpha, beta;
  const float* A;
  const float* B;
  float* C;
  int64_t lda, ldb, ldc;
  float* ws;        // split-K workspace this call may use (may be null)
  size_t ws_bytes;  // its size
  void* stream;     // hipStream_t
};

struct VariantEntry {
  mdg_variant_desc desc;
  int cfg;  // index in the family's list
};

// The table is built once, on first use, under the C++ guarantee for function-local statics: concurrent
// first calls from several threads are safe.
const VariantEntry* variant_table(int* count);
int variant_count();

// What the indirect path (Section 2.3: pad / transpose helpers, then the tiled kernel) does to a problem: padded
// extents, which operands need a packed copy, and the floats of workspace those copies take.
struct IndirectPlan {
  int64_t Mp, Np, Kp;
  bool pack_a, pack_b;
  size_t a_floats, b_floats;
};
IndirectPlan plan_indirect(int tile_m, int tile_n, int tile_k, int tA, int tB, int64_t M, int64_t N, int64_t K);

// Bytes of workspace variant e needs for this problem: split-K slices of the M x N result, or the packed
// operand copies of an indirect variant (0 for everything else).
size_t workspace_need(const VariantEntry& e, int tA, int tB, int64_t M, int64_t N, int64_t K);

// The workspace registered with mdg_set_workspace, read as one consistent (pointer, size) pair.
void registered_workspace(float** ws, size_t* bytes);

// Checks the public argument list; on success fills the column-major problem (workspace fields and stream are
// copied from the arguments given here).  Returns MDG_OK or minus the 1-based position of the first bad argument.
int canonicalise(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha, const float* A,
                 int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc, void* stream, float* ws,
                 size_t ws_bytes, GemmArgs* out);

// Section 4.1: a class must be a valid configuration for the input.
bool legal(const VariantEntry& e, const GemmArgs& g);

enum SelectorKind { SEL_TREE = 0, SEL_DEFAULT = 1 };

// The variant a call runs: the selector's answer (the compiled model behind the per-thread memo, or the
// traditional default dispatch), then the fallback links until a variant is legal for g.
int choose_variant(const GemmArgs& g, SelectorKind sel);

inline bool is_trans(int t) { return t == MDG_TRANS || t == MDG_CONJ_TRANS; }

}  // namespace mdg
