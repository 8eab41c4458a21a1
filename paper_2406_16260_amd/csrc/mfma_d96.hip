// Instantiations of the bf16 MFMA streaming kernel for head_dim 96.
#include "mfma_kernel.h"

namespace dsattn {

static const MfmaVariant kVariantsD96[] = {
    // no or up to 16 global frames (one global key tile), 1 to 3 local key tiles
    DSATTN_MFMA_SET(96, 2, 2),  // 2 head(s) per wavefront: rows of 192 channels
    DSATTN_MFMA_SET(96, 1, 2),  // 1 head(s) per wavefront: rows of 96 channels
    // up to 64 global frames: four global key tiles held in registers
    DSATTN_MFMA_SET_G4(96, 1, 2),
    // up to 128 global frames: eight global key tiles held in registers
    DSATTN_MFMA_SET_G8(96, 1, 1),
};

const MfmaVariant *mfma_variants_d96(int *n)
{
    *n = (int)(sizeof(kVariantsD96) / sizeof(kVariantsD96[0]));
    return kVariantsD96;
}

}  // namespace dsattn
