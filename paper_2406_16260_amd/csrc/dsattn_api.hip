// C-ABI layer of libdsattn: argument validation, the plan object (context index
// table of Section 4.1 / 4.2), the launch planner and dispatch to the kernels.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "plan.h"

namespace dsattn {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static int hip_fail(hipError_t e, const char *what)
{
    return fail(DSATTN_EHIP, "%s: %s", what, hipGetErrorString(e));
}

static size_t dtype_size(int32_t dt) { return dt == DSATTN_BF16 ? 2 : 4; }

// Context list of every clip: the truncated local frame range, ascending, then the
// global indices in caller order (Section 4.1 c_pre/c_post, Section 4.2 Concat).
static void build_ctx_table(dsattn_plan_t &pl)
{
    const dsattn_desc &d = pl.desc;
    const int64_t Fc = d.clip_len, N = d.n_clips, w = d.local_ctx;
    const int64_t F = Fc * N;
    const int64_t G = (int64_t)pl.global_idx.size();
    int64_t lk_max = 0;
    pl.ctx_len.assign(N, 0);
    for (int64_t i = 0; i < N; ++i) {
        int64_t lo = std::max<int64_t>(0, i * Fc - w);
        int64_t hi = std::min<int64_t>(F, (i + 1) * Fc + w);
        pl.ctx_len[i] = (int32_t)(hi - lo + G);
        lk_max = std::max<int64_t>(lk_max, pl.ctx_len[i]);
    }
    pl.lk_max = (int32_t)lk_max;
    pl.ctx_idx.assign((size_t)(N * lk_max), -1);
    for (int64_t i = 0; i < N; ++i) {
        int64_t lo = std::max<int64_t>(0, i * Fc - w);
        int64_t hi = std::min<int64_t>(F, (i + 1) * Fc + w);
        int32_t *row = pl.ctx_idx.data() + i * lk_max;
        int64_t n = 0;
        for (int64_t f = lo; f < hi; ++f) row[n++] = (int32_t)f;
        for (int64_t j = 0; j < G; ++j) row[n++] = pl.global_idx[j];
    }
}

// Launch planner: one decision per U-Net level (P, h, D differ per level, Section 3).
static void run_planner(dsattn_plan_t &pl)
{
    const dsattn_desc &d = pl.desc;
    dsattn_launch_info &li = pl.launch;
    memset(&li, 0, sizeof(li));
    li.algorithmic_bytes = (int64_t)pl.F * d.spatial * pl.C *
                           (int64_t)(3 * dtype_size(d.io_dtype) + dtype_size(d.out_dtype));
    bool force_generic = (d.flags & DSATTN_FLAG_FORCE_GENERIC) != 0;
    if (const char *e = getenv("DSATTN_FORCE_GENERIC"))
        if (e[0] == '1') force_generic = true;
    if (!force_generic && mfma_plan(pl)) return;
    // generic kernel: one wavefront per (clip, position, head)
    li.kernel = 0;
    li.variant = -1;
    li.heads_per_wave = 1;
    li.clips_per_task = 1;
    li.block_threads = 64;
    const int64_t tasks = (int64_t)d.n_clips * d.spatial * d.heads;
    li.n_tasks = tasks <= 0x7fffffffLL ? (int32_t)tasks : 0;  // 0: too many for one launch
    li.lds_bytes = (int32_t)((pl.lk_max + d.head_dim) * sizeof(float));
}

}  // namespace dsattn

using namespace dsattn;

extern "C" {

int dsattn_plan(const dsattn_desc *desc, const int32_t *global_idx, int32_t n_global, int device,
                dsattn_plan_t **out)
{
    if (!desc || !out) return fail(DSATTN_EINVAL, "dsattn_plan: null desc or out");
    *out = nullptr;
    const dsattn_desc &d = *desc;
    if (d.clip_len < 1 || d.n_clips < 1 || d.local_ctx < 0 || d.spatial < 1 || d.heads < 1 ||
        d.head_dim < 1)
        return fail(DSATTN_EINVAL, "dsattn_plan: sizes must be positive (local_ctx >= 0)");
    if (n_global < 0 || (n_global > 0 && !global_idx))
        return fail(DSATTN_EINVAL, "dsattn_plan: bad global index list");
    if ((d.io_dtype != DSATTN_F32 && d.io_dtype != DSATTN_BF16) ||
        (d.out_dtype != DSATTN_F32 && d.out_dtype != DSATTN_BF16))
        return fail(DSATTN_EINVAL, "dsattn_plan: unknown dtype");
    if (d.io_dtype == DSATTN_F32 && d.out_dtype != DSATTN_F32)
        return fail(DSATTN_EINVAL, "dsattn_plan: fp32 input requires fp32 output");
    if (!(d.scale == d.scale) || std::isinf(d.scale))
        return fail(DSATTN_EINVAL, "dsattn_plan: scale is not finite");
    if (!std::isfinite(d.bias_local) || !std::isfinite(d.bias_global))
        return fail(DSATTN_EINVAL, "dsattn_plan: scope biases must be finite");
    if (d.flags & ~(DSATTN_FLAG_FORCE_GENERIC | DSATTN_FLAG_SLIDING_WINDOW | DSATTN_FLAG_DEDUP_GLOBAL))
        return fail(DSATTN_EINVAL, "dsattn_plan: unknown flag bits 0x%x", d.flags);
    if ((d.flags & DSATTN_FLAG_SLIDING_WINDOW) && d.window < 0)
        return fail(DSATTN_EINVAL, "dsattn_plan: sliding window radius must be >= 0");
    const int64_t F = (int64_t)d.clip_len * d.n_clips;
    const int64_t C = (int64_t)d.heads * d.head_dim;
    const int64_t lk_bound = (int64_t)d.clip_len + 2 * (int64_t)d.local_ctx + n_global;
    if (F > (1 << 24) || C > (1 << 20) || F * (int64_t)d.spatial * C > ((int64_t)1 << 40) ||
        lk_bound > (1 << 20))
        return fail(DSATTN_EINVAL, "dsattn_plan: problem too large");
    for (int32_t j = 0; j < n_global; ++j)
        if (global_idx[j] < 0 || global_idx[j] >= F)
            return fail(DSATTN_EINVAL, "dsattn_plan: global_idx[%d] = %d outside [0, %lld)", j,
                        global_idx[j], (long long)F);
    if (device < -1) return fail(DSATTN_EINVAL, "dsattn_plan: bad device ordinal");

    dsattn_plan_t *pl = new (std::nothrow) dsattn_plan_t();
    if (!pl) return fail(DSATTN_ENOMEM, "dsattn_plan: host allocation failed");
    try {
        pl->desc = d;
        pl->F = (int32_t)F;
        pl->C = (int32_t)C;
        pl->device = device;
        pl->scale = d.scale > 0.f ? d.scale : 1.0f / sqrtf((float)d.head_dim);
        pl->window = (d.flags & DSATTN_FLAG_SLIDING_WINDOW) ? d.window : -1;
        pl->global_idx.assign(global_idx, global_idx + n_global);
        build_ctx_table(*pl);
    } catch (const std::bad_alloc &) {
        delete pl;
        return fail(DSATTN_ENOMEM, "dsattn_plan: host allocation failed");
    }
    run_planner(*pl);

    if (device >= 0) {
        int prev = 0;
        hipError_t e = hipGetDevice(&prev);
        if (e == hipSuccess) e = hipSetDevice(device);
        if (e != hipSuccess) {
            delete pl;
            return hip_fail(e, "dsattn_plan: hipSetDevice");
        }
        const size_t nb_idx = pl->ctx_idx.size() * sizeof(int32_t);
        const size_t nb_len = pl->ctx_len.size() * sizeof(int32_t);
        const size_t nb_g = std::max<size_t>(1, pl->global_idx.size()) * sizeof(int32_t);
        e = hipMalloc((void **)&pl->d_ctx_idx, std::max<size_t>(nb_idx, 4));
        if (e == hipSuccess) e = hipMalloc((void **)&pl->d_ctx_len, nb_len);
        if (e == hipSuccess) e = hipMalloc((void **)&pl->d_global_idx, nb_g);
        if (e == hipSuccess && nb_idx)
            e = hipMemcpy(pl->d_ctx_idx, pl->ctx_idx.data(), nb_idx, hipMemcpyHostToDevice);
        if (e == hipSuccess)
            e = hipMemcpy(pl->d_ctx_len, pl->ctx_len.data(), nb_len, hipMemcpyHostToDevice);
        if (e == hipSuccess && !pl->global_idx.empty())
            e = hipMemcpy(pl->d_global_idx, pl->global_idx.data(),
                          pl->global_idx.size() * sizeof(int32_t), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = pl->launch.kernel == 1 ? mfma_prepare(*pl) : generic_prepare(*pl);
        (void)hipSetDevice(prev);
        if (e != hipSuccess) {
            int code = e == hipErrorOutOfMemory ? DSATTN_ENOMEM : DSATTN_EHIP;
            fail(code, "dsattn_plan: device tables: %s", hipGetErrorString(e));
            dsattn_plan_destroy(pl);
            return code;
        }
    }
    *out = pl;
    return DSATTN_OK;
}

void dsattn_plan_destroy(dsattn_plan_t *plan)
{
    if (!plan) return;
    if (plan->device >= 0) {
        if (plan->d_ctx_idx) (void)hipFree(plan->d_ctx_idx);
        if (plan->d_ctx_len) (void)hipFree(plan->d_ctx_len);
        if (plan->d_global_idx) (void)hipFree(plan->d_global_idx);
    }
    delete plan;
}

int dsattn_plan_ctx_max(const dsattn_plan_t *plan, int32_t *lk_max)
{
    if (!plan || !lk_max) return fail(DSATTN_EINVAL, "dsattn_plan_ctx_max: null argument");
    *lk_max = plan->lk_max;
    return DSATTN_OK;
}

int dsattn_plan_ctx_indices(const dsattn_plan_t *plan, int32_t *ctx_idx, int32_t *ctx_len)
{
    if (!plan) return fail(DSATTN_EINVAL, "dsattn_plan_ctx_indices: null plan");
    if (ctx_idx && !plan->ctx_idx.empty())
        memcpy(ctx_idx, plan->ctx_idx.data(), plan->ctx_idx.size() * sizeof(int32_t));
    if (ctx_len) memcpy(ctx_len, plan->ctx_len.data(), plan->ctx_len.size() * sizeof(int32_t));
    return DSATTN_OK;
}

int dsattn_plan_launch_info(const dsattn_plan_t *plan, dsattn_launch_info *info)
{
    if (!plan || !info) return fail(DSATTN_EINVAL, "dsattn_plan_launch_info: null argument");
    *info = plan->launch;
    return DSATTN_OK;
}

static bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

static bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
    return x < y + nb && y < x + na;
}

// RAII: make the plan's device current for the duration of a launch.
struct DeviceGuard {
    int prev = -1;
    hipError_t err;
    explicit DeviceGuard(int dev)
    {
        err = hipGetDevice(&prev);
        if (err == hipSuccess && prev != dev) err = hipSetDevice(dev);
    }
    ~DeviceGuard()
    {
        int cur = -1;
        if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

int dsattn_gather_context(const dsattn_plan_t *plan, const void *K, const void *V, void *Kctx,
                          void *Vctx, void *stream)
{
    if (!plan) return fail(DSATTN_EINVAL, "dsattn_gather_context: null plan");
    if (plan->device < 0) return fail(DSATTN_ENODEVICE, "dsattn_gather_context: host-only plan");
    if ((K == nullptr) != (Kctx == nullptr) || (V == nullptr) != (Vctx == nullptr) ||
        (!K && !V))
        return fail(DSATTN_EINVAL, "dsattn_gather_context: pass (K,Kctx) and/or (V,Vctx)");
    if (misaligned(K) || misaligned(V) || misaligned(Kctx) || misaligned(Vctx))
        return fail(DSATTN_EINVAL, "dsattn_gather_context: pointers must be 16-byte aligned");
    DeviceGuard g(plan->device);
    if (g.err != hipSuccess) return hip_fail(g.err, "dsattn_gather_context: hipSetDevice");
    hipStream_t st = (hipStream_t)stream;
    if (K) {
        hipError_t e = launch_gather(*plan, K, Kctx, st);
        if (e != hipSuccess) return hip_fail(e, "dsattn_gather_context: launch (K)");
    }
    if (V) {
        hipError_t e = launch_gather(*plan, V, Vctx, st);
        if (e != hipSuccess) return hip_fail(e, "dsattn_gather_context: launch (V)");
    }
    return DSATTN_OK;
}

int dsattn_forward(const dsattn_plan_t *plan, const void *Q, const void *K, const void *V, void *O,
                   void *stream)
{
    if (!plan || !Q || !K || !V || !O) return fail(DSATTN_EINVAL, "dsattn_forward: null argument");
    if (plan->device < 0) return fail(DSATTN_ENODEVICE, "dsattn_forward: host-only plan");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(DSATTN_EINVAL, "dsattn_forward: pointers must be 16-byte aligned");
    const size_t n = (size_t)plan->F * plan->desc.spatial * plan->C;
    const size_t nin = n * dtype_size(plan->desc.io_dtype);
    const size_t nout = n * dtype_size(plan->desc.out_dtype);
    if (overlaps(O, nout, Q, nin) || overlaps(O, nout, K, nin) || overlaps(O, nout, V, nin))
        return fail(DSATTN_EINVAL, "dsattn_forward: O overlaps an input");
    if (plan->launch.kernel != 1 && !generic_supported(*plan))
        return fail(DSATTN_EUNSUPPORTED, "dsattn_forward: context list or problem too large for "
                                         "the generic kernel");
    DeviceGuard g(plan->device);
    if (g.err != hipSuccess) return hip_fail(g.err, "dsattn_forward: hipSetDevice");
    hipError_t e = plan->launch.kernel == 1
                       ? launch_mfma(*plan, Q, K, V, O, false, (hipStream_t)stream)
                       : launch_generic(*plan, Q, K, V, O, false, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "dsattn_forward: launch");
    return DSATTN_OK;
}

int dsattn_forward_ctx(const dsattn_plan_t *plan, const void *Q, const void *Kctx, const void *Vctx,
                       void *O, void *stream)
{
    if (!plan || !Q || !Kctx || !Vctx || !O)
        return fail(DSATTN_EINVAL, "dsattn_forward_ctx: null argument");
    if (plan->device < 0) return fail(DSATTN_ENODEVICE, "dsattn_forward_ctx: host-only plan");
    if (misaligned(Q) || misaligned(Kctx) || misaligned(Vctx) || misaligned(O))
        return fail(DSATTN_EINVAL, "dsattn_forward_ctx: pointers must be 16-byte aligned");
    const size_t n = (size_t)plan->F * plan->desc.spatial * plan->C;
    const size_t nctx = (size_t)plan->desc.n_clips * plan->lk_max * plan->desc.spatial * plan->C *
                        dtype_size(plan->desc.io_dtype);
    const size_t nin = n * dtype_size(plan->desc.io_dtype);
    const size_t nout = n * dtype_size(plan->desc.out_dtype);
    if (overlaps(O, nout, Q, nin) || overlaps(O, nout, Kctx, nctx) || overlaps(O, nout, Vctx, nctx))
        return fail(DSATTN_EINVAL, "dsattn_forward_ctx: O overlaps an input");
    if (plan->launch.kernel != 1 && !generic_supported(*plan))
        return fail(DSATTN_EUNSUPPORTED, "dsattn_forward_ctx: context list or problem too large "
                                         "for the generic kernel");
    DeviceGuard g(plan->device);
    if (g.err != hipSuccess) return hip_fail(g.err, "dsattn_forward_ctx: hipSetDevice");
    hipError_t e = plan->launch.kernel == 1
                       ? launch_mfma(*plan, Q, Kctx, Vctx, O, true, (hipStream_t)stream)
                       : launch_generic(*plan, Q, Kctx, Vctx, O, true, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "dsattn_forward_ctx: launch");
    return DSATTN_OK;
}

// One [F, P, C] tensor of the layer's workspace, rounded up so that the next one stays aligned.
static size_t layer_slab_bytes(const dsattn_plan_t &pl)
{
    const size_t n = (size_t)pl.F * pl.desc.spatial * pl.C * dtype_size(pl.desc.io_dtype);
    return (n + 255) / 256 * 256;
}

int dsattn_temporal_layer_workspace(const dsattn_plan_t *plan, size_t *bytes)
{
    if (!plan || !bytes) return fail(DSATTN_EINVAL, "dsattn_temporal_layer_workspace: null argument");
    *bytes = 4 * layer_slab_bytes(*plan);
    return DSATTN_OK;
}

int dsattn_temporal_layer(const dsattn_plan_t *plan, const void *X, const void *const *W,
                          const float *const *bias, void *workspace, size_t workspace_bytes, void *Y,
                          void *stream)
{
    const char *who = "dsattn_temporal_layer";
    if (!plan || !X || !W || !workspace || !Y) return fail(DSATTN_EINVAL, "%s: null argument", who);
    if (plan->device < 0) return fail(DSATTN_ENODEVICE, "%s: host-only plan", who);
    if (plan->desc.out_dtype != plan->desc.io_dtype)
        return fail(DSATTN_EUNSUPPORTED, "%s: the plan's out_dtype must equal its io_dtype (the "
                                         "attention's output is the output projection's input)", who);
    const size_t slab = layer_slab_bytes(*plan);
    if (workspace_bytes < 4 * slab)
        return fail(DSATTN_EINVAL, "%s: workspace of %zu bytes, %zu needed", who, workspace_bytes,
                    4 * slab);
    if (misaligned(X) || misaligned(Y) || ((uintptr_t)workspace & 255u))
        return fail(DSATTN_EINVAL, "%s: X and Y must be 16-byte and the workspace 256-byte aligned", who);
    const size_t n = (size_t)plan->F * plan->desc.spatial * plan->C * dtype_size(plan->desc.io_dtype);
    if (overlaps(workspace, 4 * slab, X, n) || overlaps(workspace, 4 * slab, Y, n))
        return fail(DSATTN_EINVAL, "%s: the workspace overlaps X or Y", who);
    if (X != Y && overlaps(X, n, Y, n))
        return fail(DSATTN_EINVAL, "%s: Y overlaps X without being X", who);
    unsigned char *ws = (unsigned char *)workspace;
    void *q = ws, *k = ws + slab, *v = ws + 2 * slab, *o = ws + 3 * slab;
    DeviceGuard g(plan->device);
    if (g.err != hipSuccess) return hip_fail(g.err, "dsattn_temporal_layer: hipSetDevice");
    dsattn_linear_desc l{};
    l.rows = (int64_t)plan->F * plan->desc.spatial;
    l.c_in = l.c_out = plan->C;
    l.io_dtype = l.out_dtype = plan->desc.io_dtype;
    l.flags = plan->desc.flags & DSATTN_FLAG_FORCE_GENERIC;
    // stage 1: Q, K, V from the tokens, X read once
    l.n_out = 3;
    void *const qkv[3] = {q, k, v};
    int rc = dsattn_linear(&l, X, W, bias, qkv, stream);
    if (rc != DSATTN_OK) return rc;
    // stage 2: Dual-scope attention
    rc = dsattn_forward(plan, q, k, v, o, stream);
    if (rc != DSATTN_OK) return rc;
    // stage 3: output projection
    l.n_out = 1;
    const float *const bo = bias ? bias[3] : nullptr;
    return dsattn_linear(&l, o, W + 3, bias ? &bo : nullptr, &Y, stream);
}

int dsattn_copy_probe(void *dst, const void *src, int64_t bytes, void *stream)
{
    if (!dst || !src || bytes <= 0 || (bytes & 15) || misaligned(dst) || misaligned(src))
        return fail(DSATTN_EINVAL, "dsattn_copy_probe: need 16-byte aligned pointers and size");
    if (overlaps(dst, (size_t)bytes, src, (size_t)bytes))
        return fail(DSATTN_EINVAL, "dsattn_copy_probe: buffers overlap");
    hipError_t e = launch_copy(dst, src, bytes, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "dsattn_copy_probe: launch");
    return DSATTN_OK;
}

const char *dsattn_strerror(int code)
{
    switch (code) {
    case DSATTN_OK: return "ok";
    case DSATTN_EINVAL: return "invalid argument";
    case DSATTN_EUNSUPPORTED: return "unsupported combination";
    case DSATTN_ENOMEM: return "out of memory";
    case DSATTN_EHIP: return "HIP runtime error";
    case DSATTN_ENODEVICE: return "plan has no device";
    default: return "unknown dsattn status";
    }
}

const char *dsattn_last_error(void) { return g_err; }

}  // extern "C"
