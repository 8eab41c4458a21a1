// Internal plan object and launcher prototypes shared by the host files of libdsattn.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "dsattn.h"

struct dsattn_plan_s {
    dsattn_desc desc;
    int32_t F;       // N * clip_len
    int32_t C;       // heads * head_dim
    int32_t lk_max;  // longest context list
    float scale;     // resolved softmax scale
    int32_t window;  // sliding-window radius of the local scope, -1 = none
    int device;      // HIP ordinal or -1

    std::vector<int32_t> global_idx;  // host copy, caller order
    std::vector<int32_t> ctx_idx;     // host [N][lk_max], -1 padded
    std::vector<int32_t> ctx_len;     // host [N]

    int32_t *d_ctx_idx = nullptr;     // device [N][lk_max]
    int32_t *d_ctx_len = nullptr;     // device [N]
    int32_t *d_global_idx = nullptr;  // device [max(1, n_global)]

    dsattn_launch_info launch;

    // resolved once by the planner for the matrix-core kernel, so that a launch searches nothing
    const void *mfma_fn = nullptr;  // the variant's kernel
    uint64_t gdup = 0;              // bit j: global entry j (< 64) repeats an earlier entry
};

namespace dsattn {

// Records a failure detail for dsattn_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);

// Launchers; each validates nothing (the API layer has) and returns a hipError_t.
hipError_t launch_gather(const dsattn_plan_t &pl, const void *X, void *Xctx, hipStream_t st);
hipError_t launch_copy(void *dst, const void *src, int64_t bytes, hipStream_t st);

// Generic vector-ALU attention. ctx_mode = false: K/V are [F,P,C] and keys are
// fetched through ctx_idx; true: K/V are [N, lk_max, P, C] and key j of clip i is row j.
bool generic_supported(const dsattn_plan_t &pl);
hipError_t generic_prepare(const dsattn_plan_t &pl);  // once per plan, plan's device current
hipError_t launch_generic(const dsattn_plan_t &pl, const void *Q, const void *K, const void *V,
                          void *O, bool ctx_mode, hipStream_t st);

// bf16 MFMA streaming kernel. `fill` reports whether a variant exists for the plan's
// shape; when it does, it completes pl.launch.
bool mfma_plan(dsattn_plan_t &pl);
hipError_t mfma_prepare(const dsattn_plan_t &pl);  // once per plan, plan's device current
// ctx_mode: K and V are the materialised contexts [N, lk_max, P, C] (one clip per chunk)
hipError_t launch_mfma(const dsattn_plan_t &pl, const void *Q, const void *K, const void *V,
                       void *O, bool ctx_mode, hipStream_t st);

}  // namespace dsattn
