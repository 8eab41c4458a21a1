// Instantiations of the bf16 MFMA streaming kernel for head_dim 128.
#include "mfma_kernel.h"

namespace dsattn {

static const MfmaVariant kVariantsD128[] = {
    // no or up to 16 global frames (one global key tile), 1 to 3 local key tiles
    DSATTN_MFMA_SET(128, 1, 2),  // 1 head(s) per wavefront: rows of 128 channels
    // up to 64 global frames: four global key tiles held in registers
    DSATTN_MFMA_SET_G4(128, 1, 1),
    // (eight global key tiles do not fit a wavefront's registers at this head size: 65 to 128
    // global frames run the generic kernel)
};

const MfmaVariant *mfma_variants_d128(int *n)
{
    *n = (int)(sizeof(kVariantsD128) / sizeof(kVariantsD128[0]));
    return kVariantsD128;
}

}  // namespace dsattn
