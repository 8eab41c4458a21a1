// Instantiations of the bf16 MFMA streaming kernel for head_dim 40.
#include "mfma_kernel.h"

namespace dsattn {

static const MfmaVariant kVariantsD40[] = {
    // no or up to 16 global frames (one global key tile), 1 to 3 local key tiles
    DSATTN_MFMA_SET(40, 4, 2),  // 4 head(s) per wavefront: rows of 160 channels
    DSATTN_MFMA_SET(40, 2, 2),  // 2 head(s) per wavefront: rows of 80 channels
    DSATTN_MFMA_SET(40, 1, 2),  // 1 head(s) per wavefront: rows of 40 channels
    // up to 64 global frames: four global key tiles held in registers
    // (two heads per wavefront with three local key tiles would spill: that shape takes one head)
    DSATTN_MFMA_VARIANT(40, 2, 1, 4, 2), DSATTN_MFMA_VARIANT(40, 2, 2, 4, 2),
    DSATTN_MFMA_SET_G4(40, 1, 2),
    // up to 128 global frames: eight global key tiles held in registers
    DSATTN_MFMA_SET_G8(40, 2, 1),
    DSATTN_MFMA_VARIANT(40, 1, 1, 8, 2), DSATTN_MFMA_VARIANT(40, 1, 2, 8, 2),
};

const MfmaVariant *mfma_variants_d40(int *n)
{
    *n = (int)(sizeof(kVariantsD40) / sizeof(kVariantsD40[0]));
    return kVariantsD40;
}

}  // namespace dsattn
