/* Plain-C user of the dsattn C ABI: builds a host-only plan (no GPU needed), reads the context
 * table back and checks it against the list written out by hand for the tiny workload
 * (2 clips x 4 frames, w = 1, global frames {0, 4}; Section 4.1 / 4.2 definitions). */
#include <stdio.h>
#include <string.h>

#include "dsattn.h"

int main(void)
{
    dsattn_desc d;
    memset(&d, 0, sizeof(d));
    d.clip_len = 4;
    d.n_clips = 2;
    d.local_ctx = 1;
    d.spatial = 16;
    d.heads = 1;
    d.head_dim = 8;
    d.io_dtype = DSATTN_F32;
    d.out_dtype = DSATTN_F32;
    const int32_t gidx[2] = {0, 4};
    dsattn_plan_t *plan = NULL;
    int rc = dsattn_plan(&d, gidx, 2, -1, &plan);
    if (rc != DSATTN_OK) {
        printf("dsattn_plan failed: %s (%s)\n", dsattn_strerror(rc), dsattn_last_error());
        return 1;
    }
    int32_t lk = 0;
    if (dsattn_plan_ctx_max(plan, &lk) != DSATTN_OK || lk != 7) return 2;
    int32_t idx[14], len[2];
    if (dsattn_plan_ctx_indices(plan, idx, len) != DSATTN_OK) return 3;
    static const int32_t want[14] = {0, 1, 2, 3, 4, 0, 4, 3, 4, 5, 6, 7, 0, 4};
    if (len[0] != 7 || len[1] != 7 || memcmp(idx, want, sizeof(want)) != 0) return 4;
    dsattn_launch_info info;
    if (dsattn_plan_launch_info(plan, &info) != DSATTN_OK || info.kernel != 0) return 5;
    /* device work on a host-only plan is refused, not attempted */
    if (dsattn_forward(plan, (void *)16, (void *)16, (void *)16, (void *)32, NULL) != DSATTN_ENODEVICE)
        return 6;
    d.clip_len = 0;
    dsattn_plan_t *bad = NULL;
    if (dsattn_plan(&d, gidx, 2, -1, &bad) != DSATTN_EINVAL || bad != NULL) return 7;
    dsattn_gn_desc g;
    memset(&g, 0, sizeof(g));
    g.clip_len = 16; g.n_clips = 4; g.spatial = 8; g.channels = 320; g.groups = 32;
    g.io_dtype = DSATTN_BF16; g.eps = 1e-5f;
    size_t ws = 0;
    if (dsattn_groupnorm_workspace(&g, &ws) != DSATTN_OK || ws == 0) return 8;
    dsattn_plan_destroy(plan);
    dsattn_plan_destroy(NULL);
    printf("ok lk_max=%d workspace=%zu\n", (int)lk, ws);
    return 0;
}
