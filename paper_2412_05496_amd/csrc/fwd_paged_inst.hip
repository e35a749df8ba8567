// One paged forward-kernel variant per translation unit: compile with -DFLEXATTN_VARIANT=<index into kVariants>.
#include "fwd_kernel.h"
#include "variants.h"

#ifndef FLEXATTN_VARIANT
#error "compile with -DFLEXATTN_VARIANT=<index>"
#endif

namespace flexattn {
int FLEXATTN_CAT(fwd_paged_launch_, FLEXATTN_VARIANT)(const FwdArgs& a, int D, int Bq, hipStream_t st) {
    return launch_fwd_variant<kVariants[FLEXATTN_VARIANT].mask, kVariants[FLEXATTN_VARIANT].score, true>(a, D, Bq, st);
}
}  // namespace flexattn
