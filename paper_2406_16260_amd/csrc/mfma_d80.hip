// Instantiations of the bf16 MFMA streaming kernel for head_dim 80 (2 head(s) per wavefront:
// 160 contiguous channels per frame row).
#include "mfma_kernel.h"

namespace dsattn {

static const MfmaVariant kVariantsD80[] = {
    DSATTN_MFMA_VARIANT(80, 2, 1, 0, 2), DSATTN_MFMA_VARIANT(80, 2, 1, 1, 2),
    DSATTN_MFMA_VARIANT(80, 2, 2, 0, 2), DSATTN_MFMA_VARIANT(80, 2, 2, 1, 2),
    DSATTN_MFMA_VARIANT(80, 2, 3, 0, 2), DSATTN_MFMA_VARIANT(80, 2, 3, 1, 2),
    // up to 64 global frames: four global key tiles held in registers; 1 head(s) per wavefront
    // keep the global context small enough for two wavefronts per SIMD
    DSATTN_MFMA_VARIANT(80, 1, 1, 4, 2), DSATTN_MFMA_VARIANT(80, 1, 2, 4, 2),
};

const MfmaVariant *mfma_variants_d80(int *n)
{
    *n = (int)(sizeof(kVariantsD80) / sizeof(kVariantsD80[0]));
    return kVariantsD80;
}

}  // namespace dsattn
