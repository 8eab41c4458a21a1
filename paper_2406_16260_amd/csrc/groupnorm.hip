// Clip-parallel group normalisation (Section 4.2, "Group normalization") for one GPU that holds
// every clip: the statistics of a channel group are those of the whole video, then
// y = (x - mean) * rstd * gamma + beta.  The paper has every device compute its clip's mean,
// average the means, then compute and average the squared deviations about the global mean: two
// rounds, because averaging per-clip deviations about per-clip means would be wrong.  The same
// global mean and variance come out of ONE pass if every part reports (count, mean, sum of squared
// deviations about its own mean) and the parts are merged with the pairwise update of Chan et
// al.; that is what is done here (one read of X for the statistics instead of two), and between
// devices it would be one exchange instead of two.
//
// All kernels stream X ([F, P, C], C fastest) with 16-byte lanes; a lane's 16 bytes belong to at
// most two groups.  Reductions are deterministic: per-thread fp32 sums about a per-thread pilot,
// a fixed-order merge per workgroup into a table in the caller's workspace, and a small
// finalising kernel in fp64.
#include <hip/hip_bf16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>

#include "plan.h"

namespace dsattn {

namespace {

struct GnShape {
    int vec;        // elements per 16-byte lane
    int ch;         // lanes per row = C / vec
    int cg;         // channels per group
    int rpb;        // rows handled together by a workgroup (blockDim.y)
    int bpc;        // workgroups per clip
    int64_t rows_per_clip;
    int64_t rows_per_block;
};

bool gn_shape(const dsattn_gn_desc &d, GnShape &s)
{
    s.vec = d.io_dtype == DSATTN_BF16 ? 8 : 4;
    if (d.channels % d.groups != 0 || d.channels % s.vec != 0) return false;
    s.cg = d.channels / d.groups;
    // a 16-byte lane may straddle two groups, not more
    if (s.cg < s.vec && s.vec % s.cg != 0) return false;
    if (s.cg < s.vec) return false;
    s.ch = d.channels / s.vec;
    if (s.ch > 1024) return false;
    s.rpb = std::max(1, 512 / s.ch);
    s.rows_per_clip = (int64_t)d.clip_len * d.spatial;
    // about eight workgroups per compute unit over the whole tensor, at least one per clip
    const int64_t want = std::max<int64_t>(1, (256 * 8) / d.n_clips);
    const int64_t max_bpc = std::max<int64_t>(1, s.rows_per_clip / (4 * s.rpb));
    s.bpc = (int)std::min<int64_t>(want, max_bpc);
    s.rows_per_block = (s.rows_per_clip + s.bpc - 1) / s.bpc;
    return true;
}

__device__ inline void unpack(const uint4 &v, float (&x)[8], __hip_bfloat16 *)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = __uint_as_float(w[i] << 16);
        x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ inline void unpack(const uint4 &v, float (&x)[8], float *)
{
    x[0] = __uint_as_float(v.x);
    x[1] = __uint_as_float(v.y);
    x[2] = __uint_as_float(v.z);
    x[3] = __uint_as_float(v.w);
}

// Merging two sets of (count, mean, sum of squared deviations about the own mean): the parallel
// form of Welford's update (Chan et al.), stable whatever the means are.
struct GnMoments {
    double n, mean, m2;
};
__device__ inline void gn_merge(GnMoments &a, double n, double mean, double m2)
{
    if (n <= 0.0) return;
    const double tot = a.n + n, delta = mean - a.mean;
    a.mean += delta * (n / tot);
    a.m2 += m2 + delta * delta * (a.n * n / tot);
    a.n = tot;
}

// Statistics pass: one read of X gives, per workgroup and group, the count, the mean and the
// sum of squared deviations about that mean of the elements the workgroup saw.  Every thread
// accumulates sum(x - p) and sum((x - p)^2) in fp32 about a pilot p of its own (the first
// element it reads: same channel, nearby rows, so the sums stay small and nothing cancels),
// turns them into (count, mean, M2), and one thread per group merges, in a fixed order, the
// threads that hold the group's channels.  blockIdx = (workgroup within clip, clip);
// thread (x, y) = (lane of the row, row phase).  A lane's VEC channels lie in group g0 (the
// first `split` of them) and, when the lane straddles a boundary, in group g0 + 1.
// Means travel as a pair of floats (pilot or leading part, remainder), so that a mean much
// larger than the spread loses nothing.  partial is [N][bpc][groups][4].
template <typename T>
__global__ __launch_bounds__(1024) void gn_moments_kernel(const uint4 *__restrict__ X,
                                                          float *__restrict__ partial, int ch,
                                                          int cg, int groups,
                                                          int64_t rows_per_clip)
{
    constexpr int VEC = sizeof(T) == 2 ? 8 : 4;
    constexpr int UNR = 4;  // independent row loads in flight per thread
    extern __shared__ float red[];  // [8][blockDim.y][ch]: (count, mean hi, mean lo, M2) for g0, then g0 + 1
    const int lane = threadIdx.x, ry = threadIdx.y, ny = blockDim.y;
    const int clip = blockIdx.y;
    const int g0 = (lane * VEC) / cg;
    const int split = min(VEC, (g0 + 1) * cg - lane * VEC);
    const uint4 *base = X + (int64_t)clip * rows_per_clip * ch + lane;
    // Per element slot of the lane: running sums of (x - pilot) and (x - pilot)^2.  The pilot of a
    // slot is the lane's first element of the slot's group, so every slot of a group is taken about
    // the same value and the slots' sums add up to the group's; three vector operations per element.
    float pv[VEC], a[VEC], q[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) pv[i] = a[i] = q[i] = 0.f;
    int rows = 0;
    auto add_row = [&](const uint4 &v) __attribute__((always_inline)) {
        float x[8];
        unpack(v, x, (T *)nullptr);
        if (rows == 0) {
            const float p0 = x[0], p1 = x[split < VEC ? split : 0];
#pragma unroll
            for (int i = 0; i < VEC; ++i) pv[i] = i < split ? p0 : p1;
        }
        ++rows;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const float d = x[i] - pv[i];
            a[i] += d;
            q[i] = fmaf(d, d, q[i]);
        }
    };
    // The workgroups of a clip take its rows in interleaved bites of UNR * ny rows, so that they
    // sweep the clip together and the chip reads a few long streams instead of one per workgroup.
    const int64_t bite = (int64_t)UNR * ny;
    for (int64_t rb = (int64_t)blockIdx.x * bite; rb < rows_per_clip; rb += (int64_t)gridDim.x * bite) {
        const int64_t r = rb + ry;
        if (rb + bite <= rows_per_clip) {
            uint4 v[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) v[u] = base[(r + (int64_t)u * ny) * ch];
#pragma unroll
            for (int u = 0; u < UNR; ++u) add_row(v[u]);
        } else {
            for (int u = 0; u < UNR; ++u)
                if (r + (int64_t)u * ny < rows_per_clip) add_row(base[(r + (int64_t)u * ny) * ch]);
        }
    }

    float p0 = pv[0], p1 = pv[VEC - 1];
    float a0 = 0.f, q0 = 0.f, a1 = 0.f, q1 = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        const bool lo = i < split;
        a0 += lo ? a[i] : 0.f;
        q0 += lo ? q[i] : 0.f;
        a1 += lo ? 0.f : a[i];
        q1 += lo ? 0.f : q[i];
    }
    const int t = ry * ch + lane, nt = ny * ch;
    const float c0 = (float)rows * (float)split, c1 = (float)rows * (float)(VEC - split);
    red[0 * nt + t] = c0;
    red[1 * nt + t] = p0;
    red[2 * nt + t] = c0 > 0.f ? a0 / c0 : 0.f;
    red[3 * nt + t] = c0 > 0.f ? q0 - a0 * a0 / c0 : 0.f;
    red[4 * nt + t] = c1;
    red[5 * nt + t] = p1;
    red[6 * nt + t] = c1 > 0.f ? a1 / c1 : 0.f;
    red[7 * nt + t] = c1 > 0.f ? q1 - a1 * a1 / c1 : 0.f;
    __syncthreads();
    // one thread per group merges, in a fixed order, the lanes that hold its channels
    if (t < groups) {
        const int g = t;
        const int l0 = (g * cg) / VEC, l1 = ((g + 1) * cg - 1) / VEC;
        GnMoments m = {0.0, 0.0, 0.0};
        for (int y = 0; y < ny; ++y)
            for (int l = l0; l <= l1; ++l) {
                const int lg0 = (l * VEC) / cg, e = y * ch + l;
                if (lg0 == g)
                    gn_merge(m, red[0 * nt + e], (double)red[1 * nt + e] + (double)red[2 * nt + e],
                             red[3 * nt + e]);
                if (lg0 == g - 1)
                    gn_merge(m, red[4 * nt + e], (double)red[5 * nt + e] + (double)red[6 * nt + e],
                             red[7 * nt + e]);
            }
        float *out = partial + (((int64_t)clip * gridDim.x + blockIdx.x) * groups + g) * 4;
        const float hi = (float)m.mean;
        out[0] = (float)m.n;
        out[1] = hi;
        out[2] = (float)(m.mean - (double)hi);
        out[3] = (float)m.m2;
    }
}

// One workgroup per group merges the workgroups' moments in fp64, in a fixed order:
// stats[g] = mean, stats[groups + g] = 1 / sqrt(M2 / n + eps) (the biased variance).
__global__ __launch_bounds__(256) void gn_finalize_kernel(const float *__restrict__ partial,
                                                          float *__restrict__ stats,
                                                          int64_t n_blocks, int groups, float eps)
{
    __shared__ double rn[256], rm[256], rq[256];
    const int g = blockIdx.x;
    GnMoments m = {0.0, 0.0, 0.0};
    for (int64_t i = threadIdx.x; i < n_blocks; i += 256) {
        const float *p = partial + (i * groups + g) * 4;
        gn_merge(m, p[0], (double)p[1] + (double)p[2], p[3]);
    }
    rn[threadIdx.x] = m.n;
    rm[threadIdx.x] = m.mean;
    rq[threadIdx.x] = m.m2;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            GnMoments a = {rn[threadIdx.x], rm[threadIdx.x], rq[threadIdx.x]};
            gn_merge(a, rn[threadIdx.x + w], rm[threadIdx.x + w], rq[threadIdx.x + w]);
            rn[threadIdx.x] = a.n;
            rm[threadIdx.x] = a.mean;
            rq[threadIdx.x] = a.m2;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        stats[g] = (float)rm[0];
        stats[groups + g] = (float)(1.0 / sqrt(rq[0] / rn[0] + (double)eps));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gn_apply_kernel(const uint4 *__restrict__ X,
                                                       uint4 *__restrict__ Y,
                                                       const float *__restrict__ stats,
                                                       const float *__restrict__ gamma,
                                                       const float *__restrict__ beta, int ch,
                                                       int cg, int groups, int64_t n16)
{
    constexpr int VEC = sizeof(T) == 2 ? 8 : 4;
    constexpr int UNR = 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    auto one = [&](int64_t i, const uint4 &v) __attribute__((always_inline)) {
        const int lane = (int)(i % ch);
        const int g0 = (lane * VEC) / cg;
        const int split = min(VEC, (g0 + 1) * cg - lane * VEC);
        const float mu0 = stats[g0], rs0 = stats[groups + g0];
        const float mu1 = split < VEC ? stats[g0 + 1] : 0.f;
        const float rs1 = split < VEC ? stats[groups + g0 + 1] : 0.f;
        float x[8];
        unpack(v, x, (T *)nullptr);
        float y[8];
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const int c = lane * VEC + k;
            const float ga = gamma ? gamma[c] : 1.f;
            const float be = beta ? beta[c] : 0.f;
            const bool lo = k < split;
            y[k] = (x[k] - (lo ? mu0 : mu1)) * (lo ? rs0 : rs1) * ga + be;
        }
        uint4 o;
        if constexpr (sizeof(T) == 2) {
            uint32_t w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const __hip_bfloat16 lo = __float2bfloat16(y[2 * k]);      // RNE
                const __hip_bfloat16 hi = __float2bfloat16(y[2 * k + 1]);
                w[k] = (uint32_t)__builtin_bit_cast(unsigned short, lo) |
                       ((uint32_t)__builtin_bit_cast(unsigned short, hi) << 16);
            }
            o = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
            o = make_uint4(__float_as_uint(y[0]), __float_as_uint(y[1]), __float_as_uint(y[2]),
                           __float_as_uint(y[3]));
        }
        Y[i] = o;
    };
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + (UNR - 1) * stride < n16; i += UNR * stride) {
        uint4 v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) v[u] = X[i + u * stride];
#pragma unroll
        for (int u = 0; u < UNR; ++u) one(i + u * stride, v[u]);
    }
    for (; i < n16; i += stride) one(i, X[i]);
}

int gn_validate(const dsattn_gn_desc *d, GnShape &s, const char *who)
{
    if (!d) return fail(DSATTN_EINVAL, "%s: null descriptor", who);
    if (d->clip_len < 1 || d->n_clips < 1 || d->spatial < 1 || d->channels < 1 || d->groups < 1)
        return fail(DSATTN_EINVAL, "%s: sizes must be positive", who);
    if (d->io_dtype != DSATTN_F32 && d->io_dtype != DSATTN_BF16)
        return fail(DSATTN_EINVAL, "%s: unknown dtype", who);
    if (!(d->eps >= 0.f) || std::isinf(d->eps))
        return fail(DSATTN_EINVAL, "%s: eps must be finite and >= 0", who);
    if (d->channels % d->groups != 0)
        return fail(DSATTN_EINVAL, "%s: channels must split evenly into groups", who);
    if ((int64_t)d->clip_len * d->n_clips * d->spatial * d->channels > ((int64_t)1 << 40) ||
        d->n_clips > 65535)
        return fail(DSATTN_EINVAL, "%s: problem too large", who);
    if (!gn_shape(*d, s))
        return fail(DSATTN_EUNSUPPORTED,
                    "%s: need channels %% %d == 0, channels per group >= %d and channels <= %d", who,
                    d->io_dtype == DSATTN_BF16 ? 8 : 4, d->io_dtype == DSATTN_BF16 ? 8 : 4,
                    d->io_dtype == DSATTN_BF16 ? 8192 : 4096);
    return DSATTN_OK;
}

size_t gn_workspace_bytes(const dsattn_gn_desc &d, const GnShape &s)
{
    // moments [N][bpc][groups][4] + statistics [2 * groups] (mean, then 1/sqrt(var + eps))
    return (4 * (size_t)d.n_clips * s.bpc * d.groups + 2 * (size_t)d.groups) * sizeof(float);
}

// Enqueues the three kernels (and the copy of the statistics); everything is validated.
hipError_t gn_enqueue(const dsattn_gn_desc &d, const GnShape &s, const void *X, const float *gamma,
                      const float *beta, void *Y, float *stats, void *workspace, hipStream_t st)
{
    float *partial = (float *)workspace;
    float *wstats = partial + 4 * (size_t)d.n_clips * s.bpc * d.groups;
    const dim3 grid(s.bpc, d.n_clips), block(s.ch, s.rpb);
    const size_t lds = 8 * (size_t)s.ch * s.rpb * sizeof(float);
    const int64_t n16 = (int64_t)d.clip_len * d.n_clips * d.spatial * s.ch;
    int64_t ablocks = (n16 + 256 * 8 - 1) / (256 * 8);
    ablocks = std::max<int64_t>(1, std::min<int64_t>(ablocks, 1 << 20));

#define DSATTN_GN_RUN(T)                                                                          \
    do {                                                                                          \
        hipLaunchKernelGGL((gn_moments_kernel<T>), grid, block, lds, st, (const uint4 *)X,        \
                           partial, s.ch, s.cg, d.groups, s.rows_per_clip);                       \
        hipLaunchKernelGGL(gn_finalize_kernel, dim3(d.groups), dim3(256), 0, st, partial, wstats, \
                           (int64_t)d.n_clips * s.bpc, d.groups, d.eps);                          \
        hipLaunchKernelGGL(gn_apply_kernel<T>, dim3((unsigned)ablocks), dim3(256), 0, st,         \
                           (const uint4 *)X, (uint4 *)Y, (const float *)wstats, gamma, beta,      \
                           s.ch, s.cg, d.groups, n16);                                           \
    } while (0)
    if (d.io_dtype == DSATTN_BF16)
        DSATTN_GN_RUN(__hip_bfloat16);
    else
        DSATTN_GN_RUN(float);
#undef DSATTN_GN_RUN
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && stats)
        e = hipMemcpyAsync(stats, wstats, 2 * (size_t)d.groups * sizeof(float),
                           hipMemcpyDeviceToDevice, st);
    return e;
}

// Scratch of dsattn_groupnorm_static: the per-workgroup moments and the statistics live in a
// file-scope device array instead of a caller's workspace, so that the entry point allocates
// nothing.  Every device the library runs on holds its own copy of the array at its own address
// until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address it returns for the current device is what the kernels get.
constexpr size_t kGnStaticBytes = (size_t)4 << 20;
constexpr int kGnMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kGnStaticBytes];

// Device address of the array on the current device, looked up once per device.
hipError_t gn_static_scratch(void **out)
{
    static std::mutex mu;
    static void *addr[kGnMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kGnMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev] = p;
    }
    *out = addr[dev];
    return hipSuccess;
}

}  // namespace
}  // namespace dsattn

using namespace dsattn;

extern "C" {

int dsattn_groupnorm_workspace(const dsattn_gn_desc *desc, size_t *bytes)
{
    GnShape s;
    if (!bytes) return fail(DSATTN_EINVAL, "dsattn_groupnorm_workspace: null argument");
    const int rc = gn_validate(desc, s, "dsattn_groupnorm_workspace");
    if (rc != DSATTN_OK) return rc;
    *bytes = gn_workspace_bytes(*desc, s);
    return DSATTN_OK;
}

int dsattn_groupnorm(const dsattn_gn_desc *desc, const void *X, const float *gamma,
                     const float *beta, void *Y, float *stats, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    GnShape s;
    const int rc = gn_validate(desc, s, "dsattn_groupnorm");
    if (rc != DSATTN_OK) return rc;
    const dsattn_gn_desc &d = *desc;
    if (!X || !Y || !workspace) return fail(DSATTN_EINVAL, "dsattn_groupnorm: null pointer");
    if (((uintptr_t)X | (uintptr_t)Y | (uintptr_t)workspace) & 15u)
        return fail(DSATTN_EINVAL, "dsattn_groupnorm: pointers must be 16-byte aligned");
    if (workspace_bytes < gn_workspace_bytes(d, s))
        return fail(DSATTN_EINVAL, "dsattn_groupnorm: workspace too small (%zu < %zu bytes)",
                    workspace_bytes, gn_workspace_bytes(d, s));
    const hipError_t e = gn_enqueue(d, s, X, gamma, beta, Y, stats, workspace, (hipStream_t)stream);
    if (e != hipSuccess) return fail(DSATTN_EHIP, "dsattn_groupnorm: %s", hipGetErrorString(e));
    return DSATTN_OK;
}

size_t dsattn_groupnorm_static_max_bytes(void) { return kGnStaticBytes; }

int dsattn_groupnorm_static(const dsattn_gn_desc *desc, const void *X, const float *gamma,
                            const float *beta, void *Y, float *stats, void *stream)
{
    GnShape s;
    const int rc = gn_validate(desc, s, "dsattn_groupnorm_static");
    if (rc != DSATTN_OK) return rc;
    const dsattn_gn_desc &d = *desc;
    if (!X || !Y) return fail(DSATTN_EINVAL, "dsattn_groupnorm_static: null pointer");
    if (((uintptr_t)X | (uintptr_t)Y) & 15u)
        return fail(DSATTN_EINVAL, "dsattn_groupnorm_static: pointers must be 16-byte aligned");
    const size_t need = gn_workspace_bytes(d, s);
    if (need > kGnStaticBytes)
        return fail(DSATTN_EUNSUPPORTED,
                    "dsattn_groupnorm_static: this shape needs %zu bytes of scratch, the static "
                    "array holds %zu; use dsattn_groupnorm with a workspace",
                    need, (size_t)kGnStaticBytes);
    void *ws = nullptr;
    hipError_t e = gn_static_scratch(&ws);
    if (e == hipSuccess)
        e = gn_enqueue(d, s, X, gamma, beta, Y, stats, ws, (hipStream_t)stream);
    if (e != hipSuccess)
        return fail(DSATTN_EHIP, "dsattn_groupnorm_static: %s", hipGetErrorString(e));
    return DSATTN_OK;
}

}  // extern "C"
