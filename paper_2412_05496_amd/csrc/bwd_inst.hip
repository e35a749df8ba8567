// One backward-kernel variant per translation unit: compile with -DFLEXATTN_VARIANT=<index into kVariants>.
#include "bwd_kernel.h"
#include "variants.h"

#ifndef FLEXATTN_VARIANT
#error "compile with -DFLEXATTN_VARIANT=<index>"
#endif

namespace flexattn {
int FLEXATTN_CAT(bwd_launch_, FLEXATTN_VARIANT)(const BwdArgs& a, int D, uint32_t stages, hipStream_t st) {
    return launch_bwd_variant<kVariants[FLEXATTN_VARIANT].mask, kVariants[FLEXATTN_VARIANT].score>(a, D, stages, st);
}
}  // namespace flexattn
