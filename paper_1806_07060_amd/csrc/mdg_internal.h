// Internal declarations shared by the GPU translation units of libmdg_sgemm.so.
// Everything here is about the column-major problem the C ABI has already
// canonicalised to (Eq. 1, Section 2.2 of the paper).
#pragma once

#include <hip/hip_runtime.h>

#include "mdg_host.h"

namespace mdg {

// Per-family launchers.  `cfg` is the index inside the family's configuration list
// (mdg_variant_list.h), `split_k` the number of K slices.  Return MDG_OK or MDG_ERR_LAUNCH.
int launch_direct(int cfg, const GemmArgs& g);
// a_rows / b_cols: rows of op(A) / columns of op(B) that exist in memory when that is more than M / N (padded
// copies made by the indirect path); the kernel may then load whole tiles past M / N.  0 = M / N.
int launch_tiled(int cfg, int split_k, const GemmArgs& g, int64_t a_rows = 0, int64_t b_cols = 0);
// Indirect path: pad / transpose helper passes into g.ws, then tiled configuration `tiled_cfg` (its tile sizes
// are passed along) on the packed operands.
int launch_indirect(int tiled_cfg, int tile_m, int tile_n, int tile_k, const GemmArgs& g);
int launch_skinny(int cfg, int split_k, const GemmArgs& g);

// C = beta * C (beta == 0 writes zeros without reading C).
int launch_scale_c(const GemmArgs& g);

// C = alpha * sum_s ws[s] + beta * C ; ws holds split_k tight column-major M x N slices.
int launch_splitk_reduce(int split_k, const GemmArgs& g);

inline hipStream_t stream_of(const GemmArgs& g) { return static_cast<hipStream_t>(g.stream); }

inline int check_launch() { return hipGetLastError() == hipSuccess ? MDG_OK : MDG_ERR_LAUNCH; }

}  // namespace mdg
