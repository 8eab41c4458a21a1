// Shape-generic kernels of libdsattn for gfx950:
//   * context gather (Section 4.1 context c^i, Section 4.2 Concat(local, global)) as an
//     index-driven slab copy;
//   * the generic vector-ALU Dual-scope attention (any dtype, head_dim, clip length), one
//     wavefront per (clip, position, head); it is the fp32 path and the fallback of the
//     MFMA kernel, on the original tensors or on a materialised context;
//   * a plain copy kernel used as the bandwidth yardstick.
#include <hip/hip_bf16.h>
#include <hip/hip_runtime.h>

#include <algorithm>

#include "plan.h"

namespace dsattn {

// ---------------------------------------------------------------- copy / gather

__global__ __launch_bounds__(256) void copy16_kernel(uint4 *__restrict__ dst,
                                                     const uint4 *__restrict__ src, int64_t n16)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_copy(void *dst, const void *src, int64_t bytes, hipStream_t st)
{
    const int64_t n16 = bytes / 16;
    // 8 x 16 B per thread keeps enough loads in flight without a long tail
    int64_t blocks = (n16 + 256 * 8 - 1) / (256 * 8);
    if (blocks < 1) blocks = 1;
    if (blocks > (1 << 20)) blocks = 1 << 20;
    hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint4 *)dst,
                       (const uint4 *)src, n16);
    return hipGetLastError();
}

// One context row (clip i, slot j) per blockIdx.x; blockIdx.y strides over the frame slab.
// slab16 = 16-byte units in one frame slab [P, C].
__global__ __launch_bounds__(256) void gather16_kernel(uint4 *__restrict__ dst,
                                                       const uint4 *__restrict__ src,
                                                       const int32_t *__restrict__ ctx_idx,
                                                       int64_t slab16)
{
    const int64_t row = blockIdx.x;
    const int32_t f = ctx_idx[row];
    uint4 *out = dst + row * slab16;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    int64_t i = (int64_t)blockIdx.y * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.y * blockDim.x;
    if (f >= 0) {
        const uint4 *in = src + (int64_t)f * slab16;
        for (; i < slab16; i += stride) out[i] = in[i];
    } else {
        for (; i < slab16; i += stride) out[i] = zero;
    }
}

// Fallback when a frame slab is not a multiple of 16 bytes: element-wise (2- or 4-byte units).
template <typename T>
__global__ __launch_bounds__(256) void gather_elem_kernel(T *__restrict__ dst,
                                                          const T *__restrict__ src,
                                                          const int32_t *__restrict__ ctx_idx,
                                                          int64_t slab)
{
    const int64_t row = blockIdx.x;
    const int32_t f = ctx_idx[row];
    T *out = dst + row * slab;
    int64_t i = (int64_t)blockIdx.y * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.y * blockDim.x;
    for (; i < slab; i += stride) out[i] = f >= 0 ? src[(int64_t)f * slab + i] : T(0);
}

hipError_t launch_gather(const dsattn_plan_t &pl, const void *X, void *Xctx, hipStream_t st)
{
    const int64_t rows = (int64_t)pl.desc.n_clips * pl.lk_max;
    if (rows == 0) return hipSuccess;
    if (rows > 0x7fffffffLL) return hipErrorInvalidValue;
    const int64_t esz = pl.desc.io_dtype == DSATTN_BF16 ? 2 : 4;
    const int64_t slab_bytes = (int64_t)pl.desc.spatial * pl.C * esz;
    if (slab_bytes % 16 == 0) {
        const int64_t slab16 = slab_bytes / 16;
        int64_t bx = (slab16 + 256 * 4 - 1) / (256 * 4);
        bx = bx < 1 ? 1 : (bx > 4096 ? 4096 : bx);
        hipLaunchKernelGGL(gather16_kernel, dim3((unsigned)rows, (unsigned)bx), dim3(256), 0, st,
                           (uint4 *)Xctx, (const uint4 *)X, pl.d_ctx_idx, slab16);
    } else {
        const int64_t slab = slab_bytes / esz;
        int64_t bx = (slab + 256 * 4 - 1) / (256 * 4);
        bx = bx < 1 ? 1 : (bx > 4096 ? 4096 : bx);
        if (esz == 2)
            hipLaunchKernelGGL(gather_elem_kernel<uint16_t>, dim3((unsigned)rows, (unsigned)bx),
                               dim3(256), 0, st, (uint16_t *)Xctx, (const uint16_t *)X,
                               pl.d_ctx_idx, slab);
        else
            hipLaunchKernelGGL(gather_elem_kernel<uint32_t>, dim3((unsigned)rows, (unsigned)bx),
                               dim3(256), 0, st, (uint32_t *)Xctx, (const uint32_t *)X,
                               pl.d_ctx_idx, slab);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- generic attention

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(__hip_bfloat16 x) { return __bfloat162float(x); }
__device__ inline void store_out(float *p, float x) { *p = x; }
__device__ inline void store_out(__hip_bfloat16 *p, float x) { *p = __float2bfloat16(x); }  // RNE

__device__ inline float wave_max(float x)
{
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ inline float wave_sum(float x)
{
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// One wavefront per (clip i, position p, head g); queries of the clip are taken in turn.
// Scores: lanes stride over keys, each lane does one full q.k dot product in fp32.
// Output: lanes stride over head channels, each lane sums over keys in list order.
// Dynamic LDS: float sp[lk_max] (scores, then weights) followed by float sq[D].
template <typename Tin, typename Tout>
__global__ __launch_bounds__(64) void generic_attn_kernel(
    const Tin *__restrict__ Q, const Tin *__restrict__ K, const Tin *__restrict__ V,
    Tout *__restrict__ O, const int32_t *__restrict__ ctx_idx, const int32_t *__restrict__ ctx_len,
    int clip_len, int P, int h, int D, int lk_max, float scale, int ctx_mode, int n_global,
    float bias_local, float bias_global, int window, int dedup)
{
    extern __shared__ float smem[];
    float *sp = smem;
    float *sq = smem + lk_max;

    const int lane = threadIdx.x;
    int64_t task = blockIdx.x;
    const int g = (int)(task % h);
    task /= h;
    const int p = (int)(task % P);
    const int i = (int)(task / P);

    const int64_t C = (int64_t)h * D;
    const int64_t FS = (int64_t)P * C;  // frame stride in elements
    const int64_t rowoff = (int64_t)p * C + (int64_t)g * D;
    const int L = ctx_len[i];
    const int32_t *ctx = ctx_idx + (int64_t)i * lk_max;

    for (int a = i * clip_len; a < (i + 1) * clip_len; ++a) {
        const Tin *q = Q + (int64_t)a * FS + rowoff;
        for (int d = lane; d < D; d += 64) sq[d] = to_f32(q[d]);
        __syncthreads();

        float m = -INFINITY;
        for (int j = lane; j < L; j += 64) {
            const int64_t fr = ctx_mode ? (int64_t)i * lk_max + j : (int64_t)ctx[j];
            const Tin *k = K + fr * FS + rowoff;
            float dot = 0.f;
            for (int d = 0; d < D; ++d) dot = fmaf(sq[d], to_f32(k[d]), dot);
            // scope weights: keys [0, L - n_global) are local, the rest global
            float s = dot * scale + (j < L - n_global ? bias_local : bias_global);
            // sliding window: a local key further than `window` frames from the query is hidden
            if (window >= 0 && j < L - n_global && abs(ctx[j] - a) > window) s = -INFINITY;
            // set union: a global entry is dropped if the query already sees its frame, as a
            // visible local key (the local part is the frame range ctx[0] .. ctx[nl - 1]) or as an
            // earlier global entry
            if (dedup && j >= L - n_global) {
                const int nl = L - n_global, f = ctx[j];
                bool seen = nl > 0 && f >= ctx[0] && f <= ctx[nl - 1] &&
                            (window < 0 || abs(f - a) <= window);
                for (int jj = nl; jj < j && !seen; ++jj) seen = ctx[jj] == f;
                if (seen) s = -INFINITY;
            }
            sp[j] = s;
            m = fmaxf(m, s);
        }
        m = wave_max(m);
        float z = 0.f;
        for (int j = lane; j < L; j += 64) {
            const float e = expf(sp[j] - m);
            sp[j] = e;
            z += e;
        }
        z = wave_sum(z);
        __syncthreads();

        const float inv = 1.0f / z;
        Tout *o = O + (int64_t)a * FS + rowoff;
        for (int d = lane; d < D; d += 64) {
            float acc = 0.f;
            for (int j = 0; j < L; ++j) {
                const int64_t fr = ctx_mode ? (int64_t)i * lk_max + j : (int64_t)ctx[j];
                acc = fmaf(sp[j], to_f32(V[fr * FS + rowoff + d]), acc);
            }
            store_out(o + d, acc * inv);
        }
        __syncthreads();
    }
}

// Orders the LDS accesses of one wavefront's lanes (they execute in issue order; only the
// compiler has to be kept from moving them).
__device__ inline void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Same arithmetic, in the same order, with the clip's keys and values staged once in LDS as fp32:
// one workgroup of up to four wavefronts per (clip, position, head), the wavefronts taking the
// clip's queries in turn.  The plain kernel above reads every key and value row from memory again
// for each of the clip's queries; this one is used whenever the rows fit in LDS.
// Dynamic LDS: float sk[lk_max][KS] (the lanes of the score loop walk keys: KS = D + 4 when rows
// are whole 16-byte pieces, so that eight consecutive rows cover all banks under 16-byte reads,
// else D made odd), sv[lk_max][D], then per wavefront sp[lk_max] (scores, then weights) and sq[D]
// (the query row).  Per-wavefront regions start on 16-byte boundaries when D % 4 == 0.
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void generic_attn_staged_kernel(
    const Tin *__restrict__ Q, const Tin *__restrict__ K, const Tin *__restrict__ V,
    Tout *__restrict__ O, const int32_t *__restrict__ ctx_idx, const int32_t *__restrict__ ctx_len,
    int clip_len, int P, int h, int D, int lk_max, float scale, int ctx_mode, int n_global,
    float bias_local, float bias_global, int window, int dedup)
{
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int KS = (D & 3) == 0 ? D + 4 : (D | 1);
    float *sk = smem;
    float *sv = sk + (size_t)lk_max * KS;
    const int Lp = (lk_max + 3) & ~3;
    float *sp = sv + (size_t)lk_max * D + (size_t)wv * (Lp + D);
    float *sq = sp + Lp;

    int64_t task = blockIdx.x;
    const int g = (int)(task % h);
    task /= h;
    const int p = (int)(task % P);
    const int i = (int)(task / P);

    const int64_t C = (int64_t)h * D;
    const int64_t FS = (int64_t)P * C;  // frame stride in elements
    const int64_t rowoff = (int64_t)p * C + (int64_t)g * D;
    const int L = ctx_len[i];
    const int32_t *ctx = ctx_idx + (int64_t)i * lk_max;

    for (int j = wv; j < L; j += nw) {
        const int64_t fr = ctx_mode ? (int64_t)i * lk_max + j : (int64_t)ctx[j];
        const Tin *k = K + fr * FS + rowoff;
        const Tin *v = V + fr * FS + rowoff;
        for (int d = lane; d < D; d += 64) {
            sk[(size_t)j * KS + d] = to_f32(k[d]);
            sv[(size_t)j * D + d] = to_f32(v[d]);
        }
    }
    __syncthreads();

    for (int a = i * clip_len + wv; a < (i + 1) * clip_len; a += nw) {
        const Tin *q = Q + (int64_t)a * FS + rowoff;
        for (int d = lane; d < D; d += 64) sq[d] = to_f32(q[d]);
        wave_lds_sync();

        float m = -INFINITY;
        for (int j = lane; j < L; j += 64) {
            const float *k = sk + (size_t)j * KS;
            float dot = 0.f;
            if ((D & 3) == 0) {  // rows of whole 16-byte pieces (KS = D + 4): 16-byte LDS reads
                for (int d = 0; d < D; d += 4) {
                    const float4 x = *(const float4 *)(sq + d), y = *(const float4 *)(k + d);
                    dot = fmaf(x.x, y.x, dot);
                    dot = fmaf(x.y, y.y, dot);
                    dot = fmaf(x.z, y.z, dot);
                    dot = fmaf(x.w, y.w, dot);
                }
            } else {
                for (int d = 0; d < D; ++d) dot = fmaf(sq[d], k[d], dot);
            }
            float s = dot * scale + (j < L - n_global ? bias_local : bias_global);
            if (window >= 0 && j < L - n_global && abs(ctx[j] - a) > window) s = -INFINITY;
            if (dedup && j >= L - n_global) {
                const int nl = L - n_global, f = ctx[j];
                bool seen = nl > 0 && f >= ctx[0] && f <= ctx[nl - 1] &&
                            (window < 0 || abs(f - a) <= window);
                for (int jj = nl; jj < j && !seen; ++jj) seen = ctx[jj] == f;
                if (seen) s = -INFINITY;
            }
            sp[j] = s;
            m = fmaxf(m, s);
        }
        m = wave_max(m);
        float z = 0.f;
        for (int j = lane; j < L; j += 64) {
            const float e = expf(sp[j] - m);
            sp[j] = e;
            z += e;
        }
        z = wave_sum(z);
        wave_lds_sync();

        const float inv = 1.0f / z;
        Tout *o = O + (int64_t)a * FS + rowoff;
        for (int d = lane; d < D; d += 64) {
            float acc = 0.f;
            for (int j = 0; j < L; ++j) acc = fmaf(sp[j], sv[(size_t)j * D + d], acc);
            store_out(o + d, acc * inv);
        }
        wave_lds_sync();
    }
}

// LDS bytes of the staged kernel with nw wavefronts per workgroup
static size_t staged_lds_bytes(const dsattn_plan_t &pl, int nw)
{
    const size_t D = (size_t)pl.desc.head_dim, L = (size_t)pl.lk_max;
    const size_t KS = (D & 3) == 0 ? D + 4 : (D | 1);
    const size_t Lp = (L + 3) & ~(size_t)3;  // per-wavefront score rows padded to 16 bytes
    return (L * (KS + D) + (size_t)nw * (Lp + D)) * sizeof(float);
}
static int staged_waves(const dsattn_plan_t &pl) { return std::min(4, std::max(1, pl.desc.clip_len)); }
constexpr size_t kGenericLdsMax = 160 * 1024;

template <typename Tin, typename Tout>
static const void *staged_fn()
{
    return (const void *)&generic_attn_staged_kernel<Tin, Tout>;
}
static const void *staged_fn_for(const dsattn_desc &d)
{
    if (d.io_dtype == DSATTN_F32) return staged_fn<float, float>();
    if (d.out_dtype == DSATTN_F32) return staged_fn<__hip_bfloat16, float>();
    return staged_fn<__hip_bfloat16, __hip_bfloat16>();
}

// Raises the staged kernel's dynamic LDS cap (once per plan, outside the launch path).
hipError_t generic_prepare(const dsattn_plan_t &pl)
{
    if (staged_lds_bytes(pl, staged_waves(pl)) > kGenericLdsMax) return hipSuccess;
    return hipFuncSetAttribute(staged_fn_for(pl.desc), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)kGenericLdsMax);
}

// The generic kernel keeps one clip's scores and one query row in LDS (64 KB cap) and
// numbers its wavefront tasks in 31 bits.
bool generic_supported(const dsattn_plan_t &pl)
{
    const dsattn_desc &d = pl.desc;
    const int64_t tasks = (int64_t)d.n_clips * d.spatial * d.heads;
    const size_t lds = (size_t)(pl.lk_max + d.head_dim) * sizeof(float);
    return tasks <= 0x7fffffffLL && lds <= 64 * 1024;
}

hipError_t launch_generic(const dsattn_plan_t &pl, const void *Q, const void *K, const void *V,
                          void *O, bool ctx_mode, hipStream_t st)
{
    const dsattn_desc &d = pl.desc;
    const int64_t tasks = (int64_t)d.n_clips * d.spatial * d.heads;
    if (tasks > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t lds = (size_t)(pl.lk_max + d.head_dim) * sizeof(float);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    const int nw = staged_waves(pl);
    const size_t slds = staged_lds_bytes(pl, nw);
    if (slds <= kGenericLdsMax) {
        const dim3 sgrid((unsigned)tasks), sblock(64 * nw);
#define DSATTN_LAUNCH_STAGED(TI, TO)                                                              \
    hipLaunchKernelGGL((generic_attn_staged_kernel<TI, TO>), sgrid, sblock, slds, st,             \
                       (const TI *)Q, (const TI *)K, (const TI *)V, (TO *)O, pl.d_ctx_idx,        \
                       pl.d_ctx_len, d.clip_len, d.spatial, d.heads, d.head_dim, pl.lk_max,       \
                       pl.scale, ctx_mode ? 1 : 0, (int)pl.global_idx.size(), d.bias_local,       \
                       d.bias_global, pl.window, (d.flags & DSATTN_FLAG_DEDUP_GLOBAL) ? 1 : 0)
        if (d.io_dtype == DSATTN_F32)
            DSATTN_LAUNCH_STAGED(float, float);
        else if (d.out_dtype == DSATTN_F32)
            DSATTN_LAUNCH_STAGED(__hip_bfloat16, float);
        else
            DSATTN_LAUNCH_STAGED(__hip_bfloat16, __hip_bfloat16);
#undef DSATTN_LAUNCH_STAGED
        return hipGetLastError();
    }
    const dim3 grid((unsigned)tasks), block(64);
#define DSATTN_LAUNCH_GENERIC(TI, TO)                                                             \
    hipLaunchKernelGGL((generic_attn_kernel<TI, TO>), grid, block, lds, st, (const TI *)Q,        \
                       (const TI *)K, (const TI *)V, (TO *)O, pl.d_ctx_idx, pl.d_ctx_len,         \
                       d.clip_len, d.spatial, d.heads, d.head_dim, pl.lk_max, pl.scale,           \
                       ctx_mode ? 1 : 0, (int)pl.global_idx.size(), d.bias_local, d.bias_global,    \
                       pl.window, (d.flags & DSATTN_FLAG_DEDUP_GLOBAL) ? 1 : 0)
    if (d.io_dtype == DSATTN_F32)
        DSATTN_LAUNCH_GENERIC(float, float);
    else if (d.out_dtype == DSATTN_F32)
        DSATTN_LAUNCH_GENERIC(__hip_bfloat16, float);
    else
        DSATTN_LAUNCH_GENERIC(__hip_bfloat16, __hip_bfloat16);
#undef DSATTN_LAUNCH_GENERIC
    return hipGetLastError();
}

}  // namespace dsattn
