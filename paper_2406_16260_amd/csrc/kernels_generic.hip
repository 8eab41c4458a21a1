// Shape-generic kernels of libdsattn for gfx950:
//   * context gather (Section 4.1 context c^i, Section 4.2 Concat(local, global)) as an
//     index-driven slab copy;
//   * the generic vector-ALU Dual-scope attention (any dtype, head_dim, clip length), one
//     wavefront per (clip, position, head); it is the fp32 path and the fallback of the
//     MFMA kernel, on the original tensors or on a materialised context;
//   * a plain copy kernel used as the bandwidth yardstick.
#include <hip/hip_bf16.h>
#include <hip/hip_runtime.h>

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
