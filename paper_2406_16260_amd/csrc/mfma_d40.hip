// Instantiations of the bf16 MFMA streaming kernel for head_dim 40 (4 head(s) per wavefront:
// 160 contiguous channels per frame row).
#include "mfma_kernel.h"

namespace dsattn {

static const MfmaVariant kVariantsD40[] = {
    DSATTN_MFMA_VARIANT(40, 4, 1, 0, 2), DSATTN_MFMA_VARIANT(40, 4, 1, 1, 2),
    DSATTN_MFMA_VARIANT(40, 4, 2, 0, 2), DSATTN_MFMA_VARIANT(40, 4, 2, 1, 2),
    DSATTN_MFMA_VARIANT(40, 4, 3, 0, 2), DSATTN_MFMA_VARIANT(40, 4, 3, 1, 2),
    // up to 64 global frames: four global key tiles held in registers; 2 head(s) per wavefront
    // keep the global context small enough for two wavefronts per SIMD
    DSATTN_MFMA_VARIANT(40, 2, 1, 4, 2), DSATTN_MFMA_VARIANT(40, 2, 2, 4, 2),
};

const MfmaVariant *mfma_variants_d40(int *n)
{
    *n = (int)(sizeof(kVariantsD40) / sizeof(kVariantsD40[0]));
    return kVariantsD40;
}

}  // namespace dsattn
