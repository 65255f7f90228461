// The tuning space: one line per compiled kernel configuration, one table of variants.
// Single source of truth for the kernels' template instantiations, the variant
// table (mdg_variant_info), legality and the selector's class ids.
//
// The paper's library exposes thousands of parameter points per kernel
// (Section 4.1, tuning-size table); this family is deliberately small, built
// for wave64 matrix cores and 160 KB of LDS rather than for the OpenCL devices
// studied there.
#pragma once

// Direct (generic) kernel: 16 x 16 threads, each computing TM x TN elements of C.
//   X(cfg, TM, TN, LDS)     tile = 16*TM x 16*TN, K step 16 when staged through LDS
#define MDG_DIRECT_CONFIGS(X) \
  X(0, 4, 4, 1)               \
  X(1, 1, 1, 0)               \
  X(2, 2, 2, 0)               \
  X(3, 2, 2, 1)               \
  X(4, 8, 4, 1)               \
  X(5, 4, 1, 0)               \
  X(6, 1, 4, 0)

// Tiled matrix-core kernel: work-group tile BM x BN x BK, WGM x WGN waves per wave group, WGK wave
// groups that split every K step among themselves (partial sums added through LDS).  DLDS = 1: operands
// whose rows are contiguous in memory are loaded from global memory straight into LDS in the interior loop
// (legal only when those operands are 16-byte aligned).
// KMAP = lane arrangement of the global loads of k-contiguous operands (0, 1 or 2, see the kernel).
//   X(cfg, BM, BN, BK, WGM, WGN, WGK, DLDS, KMAP)
#define MDG_TILED_CONFIGS(X)       \
  X(0, 256, 256, 16, 2, 4, 1, 0, 2)      \
  X(1, 256, 128, 16, 2, 2, 1, 0, 2)      \
  X(2, 128, 256, 16, 2, 2, 1, 0, 2)      \
  X(3, 128, 128, 16, 2, 2, 1, 0, 2)      \
  X(4, 128, 128, 32, 2, 2, 1, 0, 2)      \
  X(5, 128, 64, 16, 2, 2, 1, 0, 2)       \
  X(6, 64, 128, 16, 2, 2, 1, 0, 2)       \
  X(7, 64, 64, 16, 2, 2, 1, 0, 2)        \
  X(8, 64, 64, 32, 2, 2, 1, 0, 2)        \
  X(9, 32, 32, 32, 1, 1, 1, 0, 2)        \
  X(10, 256, 256, 32, 2, 4, 1, 0, 2)     \
  X(11, 128, 32, 32, 4, 1, 1, 0, 2)      \
  X(12, 32, 128, 32, 1, 4, 1, 0, 2)      \
  X(13, 32, 32, 64, 1, 1, 4, 0, 2)       \
  X(14, 32, 32, 128, 1, 1, 8, 0, 2)      \
  X(15, 64, 64, 64, 2, 2, 4, 0, 2)       \
  X(16, 64, 64, 32, 2, 2, 2, 0, 2)       \
  X(17, 128, 128, 32, 2, 2, 2, 0, 2)     \
  X(18, 64, 32, 32, 2, 1, 1, 0, 2)       \
  X(19, 32, 64, 32, 1, 2, 1, 0, 2)       \
  X(20, 64, 32, 32, 2, 1, 2, 0, 2)       \
  X(21, 32, 64, 32, 1, 2, 2, 0, 2)       \
  X(22, 128, 64, 32, 2, 2, 1, 0, 2)      \
  X(23, 64, 128, 32, 2, 2, 1, 0, 2)        \
  X(24, 128, 128, 32, 2, 2, 1, 1, 2)       \
  X(25, 128, 256, 16, 2, 2, 1, 1, 2)       \
  X(26, 256, 128, 16, 2, 2, 1, 1, 2)    \
  X(27, 32, 32, 256, 1, 1, 4, 0, 2)     \
  X(28, 64, 64, 128, 2, 2, 4, 0, 2)

// Skinny-N kernels: stream A once; NB columns of C per pass over A.
//   X(cfg, NB, MATRIX)   MATRIX = 0: vector-ALU kernels, NB columns held per thread
//                        MATRIX = 1: 16x16x4 matrix-core kernel, NB = 16 or 32 columns per wave
#define MDG_SKINNY_CONFIGS(X) \
  X(0, 1, 0)                  \
  X(1, 4, 0)                  \
  X(2, 8, 0)                  \
  X(3, 16, 0)                 \
  X(4, 16, 1)                 \
  X(5, 32, 1)

// Indirect path (Section 2.3): helper passes write padded, untransposed copies of the operands into the
// workspace, then the tiled configuration TILED_CFG runs on them with every tile interior.
//   X(cfg, TILED_CFG)
#define MDG_INDIRECT_CONFIGS(X) \
  X(0, 4)                       \
  X(1, 2)                       \
  X(2, 0)                       \
  X(3, 8)

// The variants: (family, cfg, split_k).  Order defines the public variant ids;
// id 0 must be legal for every input (the universal fallback).
//   V(family, cfg, split_k)
#define MDG_VARIANTS(V) \
  V(DIRECT, 0, 1)       \
  V(DIRECT, 1, 1)       \
  V(DIRECT, 2, 1)       \
  V(DIRECT, 3, 1)       \
  V(DIRECT, 4, 1)       \
  V(DIRECT, 5, 1)       \
  V(DIRECT, 6, 1)       \
  V(TILED, 0, 1)        \
  V(TILED, 1, 1)        \
  V(TILED, 2, 1)        \
  V(TILED, 3, 1)        \
  V(TILED, 4, 1)        \
  V(TILED, 5, 1)        \
  V(TILED, 6, 1)        \
  V(TILED, 7, 1)        \
  V(TILED, 8, 1)        \
  V(TILED, 9, 1)       \
  V(TILED, 10, 1)       \
  V(TILED, 11, 1)       \
  V(TILED, 12, 1)       \
  V(TILED, 1, 2)        \
  V(TILED, 3, 2)        \
  V(TILED, 3, 4)        \
  V(TILED, 3, 8)        \
  V(TILED, 7, 2)        \
  V(TILED, 7, 4)        \
  V(TILED, 7, 8)        \
  V(TILED, 7, 16)       \
  V(TILED, 9, 4)       \
  V(TILED, 9, 16)      \
  V(TILED, 9, 64)      \
  V(TILED, 5, 2)        \
  V(TILED, 5, 4)        \
  V(TILED, 6, 2)        \
  V(TILED, 6, 4)        \
  V(TILED, 11, 4)       \
  V(TILED, 11, 16)      \
  V(TILED, 12, 4)       \
  V(TILED, 12, 16)      \
  V(TILED, 8, 2)        \
  V(TILED, 8, 4)        \
  V(SKINNY, 0, 1)       \
  V(SKINNY, 1, 1)       \
  V(SKINNY, 2, 1)       \
  V(SKINNY, 3, 1)       \
  V(SKINNY, 0, 8)       \
  V(SKINNY, 1, 8)       \
  V(SKINNY, 2, 8)       \
  V(SKINNY, 3, 8)       \
  V(SKINNY, 0, 32)      \
  V(SKINNY, 1, 32)      \
  V(SKINNY, 2, 32)      \
  V(TILED, 13, 1)       \
  V(TILED, 14, 1)       \
  V(TILED, 15, 1)       \
  V(TILED, 16, 1)       \
  V(TILED, 17, 1)       \
  V(TILED, 13, 4)       \
  V(TILED, 15, 4)       \
  V(TILED, 18, 1)       \
  V(TILED, 19, 1)       \
  V(SKINNY, 4, 1)       \
  V(SKINNY, 5, 1)       \
  V(SKINNY, 4, 4)       \
  V(SKINNY, 5, 4)  \
  V(INDIRECT, 0, 1)     \
  V(INDIRECT, 1, 1)     \
  V(INDIRECT, 2, 1)     \
  V(INDIRECT, 3, 1)  \
  V(TILED, 20, 1)       \
  V(TILED, 21, 1)       \
  V(TILED, 22, 1)       \
  V(TILED, 23, 1)  \
  V(TILED, 24, 1)       \
  V(TILED, 25, 1)       \
  V(TILED, 26, 1)  \
  V(TILED, 27, 1)       \
  V(TILED, 28, 1)
