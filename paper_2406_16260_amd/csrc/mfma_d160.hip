// Instantiations of the bf16 MFMA streaming kernel for head_dim 160 (1 head(s) per wavefront:
// 160 contiguous channels per frame row).
#include "mfma_kernel.h"

namespace dsattn {

static const MfmaVariant kVariantsD160[] = {
    DSATTN_MFMA_VARIANT(160, 1, 1, 0, 2), DSATTN_MFMA_VARIANT(160, 1, 1, 1, 2),
    DSATTN_MFMA_VARIANT(160, 1, 2, 0, 2), DSATTN_MFMA_VARIANT(160, 1, 2, 1, 2),
    DSATTN_MFMA_VARIANT(160, 1, 3, 0, 2), DSATTN_MFMA_VARIANT(160, 1, 3, 1, 2),
    // up to 64 global frames: four global key tiles held in registers, one wavefront per SIMD
    DSATTN_MFMA_VARIANT(160, 1, 1, 4, 1), DSATTN_MFMA_VARIANT(160, 1, 2, 4, 1),
};

const MfmaVariant *mfma_variants_d160(int *n)
{
    *n = (int)(sizeof(kVariantsD160) / sizeof(kVariantsD160[0]));
    return kVariantsD160;
}

}  // namespace dsattn
