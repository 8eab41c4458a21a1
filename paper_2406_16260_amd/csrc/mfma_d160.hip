// Instantiations of the bf16 MFMA streaming kernel for head_dim 160.
#include "mfma_kernel.h"

namespace dsattn {

static const MfmaVariant kVariantsD160[] = {
    // no or up to 16 global frames (one global key tile), 1 to 3 local key tiles
    DSATTN_MFMA_SET(160, 1, 2),  // 1 head(s) per wavefront: rows of 160 channels
    // up to 64 global frames: four global key tiles held in registers
    DSATTN_MFMA_SET_G4(160, 1, 1),
    // (eight global key tiles do not fit a wavefront's registers at this head size: 65 to 128
    // global frames run the generic kernel)
};

const MfmaVariant *mfma_variants_d160(int *n)
{
    *n = (int)(sizeof(kVariantsD160) / sizeof(kVariantsD160[0]));
    return kVariantsD160;
}

}  // namespace dsattn
