// Placeholder selector used until a tuning run has produced a trained tree
// (paper_1806_07060_amd/tuning/codegen.py overwrites this file).
#pragma once
#include <stdint.h>

#define MDG_GENERATED_SELECTOR_NAME "untrained-placeholder"
#define MDG_GENERATED_DEFAULT_THRESHOLD 2097152.0 /* M*N*K at which the default dispatch switches to the tiled kernel */
#define MDG_GENERATED_DEFAULT_TILED 11
#define MDG_GENERATED_DEFAULT_DIRECT 0

static inline int mdg_generated_select(int tA, int tB, int64_t M, int64_t N, int64_t K) {
  (void)tA;
  (void)tB;
  if ((double)M * (double)N * (double)K < 2097152.0) return 0;
  if (M >= 2048 && N >= 2048) return 7;
  return 11;
}
