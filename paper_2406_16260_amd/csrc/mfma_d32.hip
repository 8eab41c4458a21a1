// Instantiations of the bf16 MFMA streaming kernel for head_dim 32.
#include "mfma_kernel.h"

namespace dsattn {

static const MfmaVariant kVariantsD32[] = {
    // no or up to 16 global frames (one global key tile), 1 to 3 local key tiles
    DSATTN_MFMA_SET(32, 4, 2),  // 4 head(s) per wavefront: rows of 128 channels
    DSATTN_MFMA_SET(32, 2, 2),  // 2 head(s) per wavefront: rows of 64 channels
    DSATTN_MFMA_SET(32, 1, 2),  // 1 head(s) per wavefront: rows of 32 channels
    // up to 64 global frames: four global key tiles held in registers
    DSATTN_MFMA_SET_G4(32, 2, 2),
    DSATTN_MFMA_SET_G4(32, 1, 2),
    // up to 128 global frames: eight global key tiles held in registers
    DSATTN_MFMA_SET_G8(32, 1, 2),
};

const MfmaVariant *mfma_variants_d32(int *n)
{
    *n = (int)(sizeof(kVariantsD32) / sizeof(kVariantsD32[0]));
    return kVariantsD32;
}

}  // namespace dsattn
