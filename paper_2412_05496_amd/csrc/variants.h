// Table of the (mask_mod, score_mod) pairs that the forward and backward kernels are instantiated
// for.  Each pair is compiled in its own translation unit (-DFLEXATTN_VARIANT=<index>) so that the
// build can run in parallel; the dispatchers look the pair up here.
#pragma once

#include "flex_common.h"

namespace flexattn {

struct Variant {
    uint32_t mask, score;
};

#define FLEXATTN_VARIANT_ENTRY(M, S) {M, S},
constexpr Variant kVariants[] = {FLEXATTN_FOR_EACH_VARIANT(FLEXATTN_VARIANT_ENTRY)};
#undef FLEXATTN_VARIANT_ENTRY
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
#define FLEXATTN_COUNT_ONE(i) +1
static_assert(kNumVariants == 0 FLEXATTN_VARIANT_INDICES(FLEXATTN_COUNT_ONE),
              "FLEXATTN_VARIANT_INDICES (flex_common.h) and NUM_VARIANTS (build.py) must list every variant");
#undef FLEXATTN_COUNT_ONE

inline int find_variant(uint32_t mask, uint32_t score) {
    for (int i = 0; i < kNumVariants; ++i)
        if (kVariants[i].mask == mask && kVariants[i].score == score) return i;
    return -1;
}

#define FLEXATTN_CAT_(a, b) a##b
#define FLEXATTN_CAT(a, b) FLEXATTN_CAT_(a, b)

}  // namespace flexattn
