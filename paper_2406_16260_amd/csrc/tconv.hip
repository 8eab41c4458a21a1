// Clip-parallel temporal convolution (Section 4.2 of the paper, "Convolution module") on gfx950.
//
//   Y[f][p][co] = bias[co] + sum_t sum_ci W[t][co][ci] * X[f + t - n][p][ci],  zeros outside [0, F)
//
// With rows m = f * P + p, tap t reads row m + (t - n) * P of the same matrix X[M][c_in]: the
// module is the sum over taps of  shift_t(X) * W_t^T, an implicit GEMM of M x c_out x (taps * c_in)
// whose A operand is X itself at a row offset (no im2col buffer, no halo copy: the c_pre / c_post
// frames of a clip are simply the neighbouring rows) and whose operands are both contiguous
// along the contraction.  It is a dense contraction (2 * taps * c_in flop per output element
// against 2 + 2 bytes): bound by the matrix cores, not by HBM.
//
// MFMA kernel.  A workgroup of 4 wavefronts (one per SIMD, 512 registers each) computes a
// (64 MI) x (64 NJ) tile of Y; wavefront (wm, wn) owns a (32 MI) x (32 NJ) quarter as MI x NJ
// accumulators of v_mfma_f32_32x32x16_bf16.  The contraction runs in steps of 64 channels of one
// tap: the step's X rows and W rows go global -> registers -> LDS (double buffered, one barrier
// per step) while the previous step is multiplied out of the other buffer.  LDS rows are 128 B
// of data padded to 144 B, which makes both the 16-byte row writes and the 16-byte operand
// reads (32 consecutive rows, same chunk) free of bank conflicts.  Workgroups are numbered so
// that each XCD walks a contiguous run of tiles (all column tiles of a few neighbouring row
// tiles): the W slabs and the rows shared between taps are then served by that XCD's L2.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <mutex>

#include "dsattn.h"
#include "plan.h"

namespace dsattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;       // contraction depth per step (bf16 elements)
constexpr int kRS = 144;      // LDS row stride in bytes: 128 B of data + 16 B of padding
constexpr int kXcds = 8;

struct ConvArgs {
    const void *X, *W;
    const float *bias;
    void *Y;
    int64_t M;                 // rows = F * P
    int32_t P, Cin, Cout, n;
    int32_t KC;                // steps per tap = ceil(c_in / 64)
    int32_t KS;                // steps in all = taps * KC
    int32_t tiles_n, tiles;    // column tiles, all tiles
    int32_t per_xcd;           // ceil(tiles / 8)
};

template <int MI, int NJ, bool OUT_F32>
__global__ __launch_bounds__(256, 1) void tconv_mfma_kernel(const ConvArgs a)
{
    constexpr int BM = 64 * MI, BN = 64 * NJ;
    constexpr int LA = BM / 32, LB = BN / 32;  // 16-byte loads per thread and step for X and W
    constexpr int ABYTES = BM * kRS, BBYTES = BN * kRS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    // workgroup -> tile: XCD x (= blockIdx % 8) walks tiles [x * per_xcd, (x + 1) * per_xcd)
    const int tile = (int)(blockIdx.x % kXcds) * a.per_xcd + (int)(blockIdx.x / kXcds);
    if (tile >= a.tiles) return;  // whole workgroup: no barrier has been reached yet
    const int mt = tile / a.tiles_n, nt = tile - mt * a.tiles_n;
    const int64_t m0 = (int64_t)mt * BM;
    const int n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int lrow = tid >> 3;  // row (mod 32) this thread loads
    const int lch = tid & 7;    // 16-byte chunk of the 128-byte step row

    const __bf16 *X = (const __bf16 *)a.X;
    const __bf16 *W = (const __bf16 *)a.W;

    uint4 ra[LA], rb[LB];
    // step ks = tap * KC + channel block: rows of X at the tap's frame offset, rows of W_tap
    auto gload = [&](int ks) __attribute__((always_inline)) {
        const int t = ks / a.KC, kc = ks - t * a.KC;
        const int ci = kc * kBK + lch * 8;
        const bool cok = ci < a.Cin;  // c_in is a multiple of 8: a chunk is all in or all out
        const int64_t mrow = m0 + (int64_t)(t - a.n) * a.P + lrow;
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            const int64_t m = mrow + 32 * j;
            uint4 x = make_uint4(0, 0, 0, 0);
            if (cok && m >= 0 && m < a.M) x = *(const uint4 *)(X + m * a.Cin + ci);
            ra[j] = x;
        }
        const __bf16 *Wt = W + (int64_t)t * a.Cout * a.Cin;
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            const int co = n0 + lrow + 32 * j;
            uint4 x = make_uint4(0, 0, 0, 0);
            if (cok && co < a.Cout) x = *(const uint4 *)(Wt + (int64_t)co * a.Cin + ci);
            rb[j] = x;
        }
    };
    auto lstore = [&](int buf) __attribute__((always_inline)) {
        unsigned char *As = smem + buf * (ABYTES + BBYTES);
        unsigned char *Bs = As + ABYTES;
#pragma unroll
        for (int j = 0; j < LA; ++j) *(uint4 *)(As + (lrow + 32 * j) * kRS + lch * 16) = ra[j];
#pragma unroll
        for (int j = 0; j < LB; ++j) *(uint4 *)(Bs + (lrow + 32 * j) * kRS + lch * 16) = rb[j];
    };

    f32x16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    gload(0);
    lstore(0);
    __syncthreads();

    // operand addresses: MFMA row/column lane & 31, contraction group lane >> 5 (8 bf16 each)
    const int arow = (wm * 32 * MI + (lane & 31)) * kRS + (lane >> 5) * 16;
    const int brow = (wn * 32 * NJ + (lane & 31)) * kRS + (lane >> 5) * 16;

    for (int ks = 0; ks < a.KS; ++ks) {
        const int cur = ks & 1;
        const bool more = ks + 1 < a.KS;
        if (more) gload(ks + 1);
        const unsigned char *As = smem + cur * (ABYTES + BBYTES);
        const unsigned char *Bs = As + ABYTES;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            bf16x8 af[MI], bfr[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[i] = *(const bf16x8 *)(As + arow + i * 32 * kRS + kk * 32);
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                bfr[j] = *(const bf16x8 *)(Bs + brow + j * 32 * kRS + kk * 32);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0,
                                                                        0, 0);
        }
        // the other buffer was last read in step ks - 1, which every wavefront has left
        if (more) lstore(cur ^ 1);
        __syncthreads();
    }

    // epilogue: accumulator element e of lane l is row 8 (e / 4) + 4 (l / 32) + e % 4, column
    // l % 32 of its 32 x 32 block
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int co = n0 + wn * 32 * NJ + 32 * j + (lane & 31);
        if (co >= a.Cout) continue;
        const float b = a.bias ? a.bias[co] : 0.f;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m0 + wm * 32 * MI + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (m < a.M) {
                    const float y = acc[i][j][e] + b;
                    if constexpr (OUT_F32)
                        ((float *)a.Y)[m * a.Cout + co] = y;
                    else
                        ((__bf16 *)a.Y)[m * a.Cout + co] = (__bf16)y;
                }
            }
    }
}

// Plain vector kernel for every other case (fp32 tensors, c_in not a multiple of 8): one
// thread per output element, output channel fastest.
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void tconv_generic_kernel(const Tin *X, const Tin *W,
                                                            const float *bias, Tout *Y, int64_t M,
                                                            int P, int Cin, int Cout, int n)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= M * Cout) return;
    const int64_t m = idx / Cout;
    const int co = (int)(idx - m * Cout);
    float acc = bias ? bias[co] : 0.f;
    for (int t = 0; t <= 2 * n; ++t) {
        const int64_t ms = m + (int64_t)(t - n) * P;
        if (ms < 0 || ms >= M) continue;
        const Tin *x = X + ms * Cin;
        const Tin *w = W + ((int64_t)t * Cout + co) * Cin;
        for (int ci = 0; ci < Cin; ++ci) acc = fmaf((float)w[ci], (float)x[ci], acc);
    }
    Y[idx] = (Tout)acc;
}

struct ConvVariant {
    int MI, NJ;
    const void *fn[2];  // bf16 / fp32 output
};
const ConvVariant kConvVariants[] = {
    {4, 4, {(const void *)&tconv_mfma_kernel<4, 4, false>, (const void *)&tconv_mfma_kernel<4, 4, true>}},
    {3, 5, {(const void *)&tconv_mfma_kernel<3, 5, false>, (const void *)&tconv_mfma_kernel<3, 5, true>}},
};

int conv_validate(const dsattn_conv_desc *d, const char *who)
{
    if (!d) return fail(DSATTN_EINVAL, "%s: null descriptor", who);
    if (d->clip_len < 1 || d->n_clips < 1 || d->spatial < 1 || d->c_in < 1 || d->c_out < 1)
        return fail(DSATTN_EINVAL, "%s: sizes must be positive", who);
    if (d->reach < 0 || d->reach > d->clip_len)
        return fail(DSATTN_EINVAL,
                    "%s: reach %d outside [0, clip_len = %d] (the context of a clip comes from "
                    "its two neighbouring clips only)", who, d->reach, d->clip_len);
    if ((d->io_dtype != DSATTN_F32 && d->io_dtype != DSATTN_BF16) ||
        (d->out_dtype != DSATTN_F32 && d->out_dtype != DSATTN_BF16))
        return fail(DSATTN_EINVAL, "%s: unknown dtype", who);
    if (d->io_dtype == DSATTN_F32 && d->out_dtype != DSATTN_F32)
        return fail(DSATTN_EINVAL, "%s: fp32 inputs need an fp32 output", who);
    if (d->flags & ~DSATTN_FLAG_FORCE_GENERIC)
        return fail(DSATTN_EINVAL, "%s: unknown flag bits 0x%x", who, d->flags);
    const int64_t F = (int64_t)d->clip_len * d->n_clips;
    if (F * d->spatial > ((int64_t)1 << 40) || F > 0x7fffffffLL)
        return fail(DSATTN_EINVAL, "%s: video too long", who);
    return DSATTN_OK;
}

// Tile shape: the variant that wastes the fewest output columns, then the fewest output rows.
const ConvVariant *conv_pick(const dsattn_conv_desc &d, int64_t M)
{
    if (d.io_dtype != DSATTN_BF16 || d.c_in % 8 != 0 || (d.flags & DSATTN_FLAG_FORCE_GENERIC))
        return nullptr;
    const ConvVariant *best = nullptr;
    double best_cost = 0;
    for (const ConvVariant &v : kConvVariants) {
        const int64_t bm = 64 * v.MI, bn = 64 * v.NJ;
        const int64_t tm = (M + bm - 1) / bm, tn = (d.c_out + bn - 1) / bn;
        if (tm * tn > 0x7fffffffLL / 2) continue;
        const double cost = (double)(tm * bm) * (double)(tn * bn);  // multiplied-out area
        if (!best || cost < best_cost) {
            best = &v;
            best_cost = cost;
        }
    }
    return best;
}

int conv_lds_bytes(const ConvVariant &v) { return 2 * (64 * v.MI + 64 * v.NJ) * kRS; }

}  // namespace

}  // namespace dsattn

using namespace dsattn;

extern "C" {

int dsattn_temporal_conv_info(const dsattn_conv_desc *desc, dsattn_conv_info *info)
{
    const int rc = conv_validate(desc, "dsattn_temporal_conv_info");
    if (rc != DSATTN_OK) return rc;
    if (!info) return fail(DSATTN_EINVAL, "dsattn_temporal_conv_info: null output");
    const dsattn_conv_desc &d = *desc;
    const int64_t F = (int64_t)d.clip_len * d.n_clips;
    const int64_t M = F * d.spatial;
    const int64_t taps = 2 * (int64_t)d.reach + 1;
    *info = dsattn_conv_info{};
    const ConvVariant *v = conv_pick(d, M);
    if (v) {
        const int64_t bm = 64 * v->MI, bn = 64 * v->NJ;
        const int64_t tiles = ((M + bm - 1) / bm) * ((d.c_out + bn - 1) / bn);
        info->kernel = 1;
        info->tile_m = (int32_t)bm;
        info->tile_n = (int32_t)bn;
        info->tile_k = kBK;
        info->n_blocks = (int32_t)(((tiles + kXcds - 1) / kXcds) * kXcds);
        info->block_threads = 256;
        info->lds_bytes = conv_lds_bytes(*v);
    } else {
        info->kernel = 0;
        info->tile_n = 1;
        info->tile_k = 1;
        info->n_blocks = (int32_t)std::min<int64_t>((M * d.c_out + 255) / 256, 0x7fffffff);
        info->block_threads = 256;
    }
    // tap t of frame f is inside the video unless f + t - n falls off an end: n (n + 1) pairs do
    const int64_t pairs = taps * F - (int64_t)d.reach * (d.reach + 1);
    info->useful_flops = 2 * pairs * d.spatial * d.c_in * d.c_out;
    const int64_t in_b = d.io_dtype == DSATTN_BF16 ? 2 : 4, out_b = d.out_dtype == DSATTN_BF16 ? 2 : 4;
    info->algorithmic_bytes =
        M * d.c_in * in_b + taps * d.c_out * d.c_in * in_b + M * d.c_out * out_b;
    return DSATTN_OK;
}

int dsattn_temporal_conv(const dsattn_conv_desc *desc, const void *X, const void *W,
                         const float *bias, void *Y, void *stream)
{
    const int rc = conv_validate(desc, "dsattn_temporal_conv");
    if (rc != DSATTN_OK) return rc;
    const dsattn_conv_desc &d = *desc;
    if (!X || !W || !Y) return fail(DSATTN_EINVAL, "dsattn_temporal_conv: null pointer");
    if (((uintptr_t)X | (uintptr_t)W | (uintptr_t)Y) & 15u)
        return fail(DSATTN_EINVAL, "dsattn_temporal_conv: pointers must be 16-byte aligned");
    if (bias && ((uintptr_t)bias & 3u))
        return fail(DSATTN_EINVAL, "dsattn_temporal_conv: bias must be 4-byte aligned");
    const int64_t F = (int64_t)d.clip_len * d.n_clips;
    const int64_t M = F * d.spatial;
    const int64_t in_b = d.io_dtype == DSATTN_BF16 ? 2 : 4, out_b = d.out_dtype == DSATTN_BF16 ? 2 : 4;
    {
        // an output row is written while neighbouring input rows are still being read by others
        const uintptr_t x0 = (uintptr_t)X, x1 = x0 + (uintptr_t)(M * d.c_in * in_b);
        const uintptr_t y0 = (uintptr_t)Y, y1 = y0 + (uintptr_t)(M * d.c_out * out_b);
        if (x0 < y1 && y0 < x1)
            return fail(DSATTN_EINVAL, "dsattn_temporal_conv: Y overlaps X");
    }
    hipStream_t st = (hipStream_t)stream;
    const ConvVariant *v = conv_pick(d, M);
    hipError_t e = hipSuccess;
    if (v) {
        const void *fn = v->fn[d.out_dtype == DSATTN_F32 ? 1 : 0];
        const int lds = conv_lds_bytes(*v);
        // the default cap on dynamic LDS is 64 KB: raised once per kernel and device
        static std::mutex mu;
        static uint64_t prepared[sizeof(kConvVariants) / sizeof(kConvVariants[0])][2] = {};
        int dev = 0;
        e = hipGetDevice(&dev);
        if (e == hipSuccess && dev < 64) {
            std::lock_guard<std::mutex> lock(mu);
            uint64_t &mask = prepared[v - kConvVariants][d.out_dtype == DSATTN_F32 ? 1 : 0];
            if (!(mask >> dev & 1)) {
                e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
                if (e == hipSuccess) mask |= (uint64_t)1 << dev;
            }
        } else if (e == hipSuccess) {
            e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        }
        if (e == hipSuccess) {
            ConvArgs a;
            a.X = X;
            a.W = W;
            a.bias = bias;
            a.Y = Y;
            a.M = M;
            a.P = d.spatial;
            a.Cin = d.c_in;
            a.Cout = d.c_out;
            a.n = d.reach;
            a.KC = (d.c_in + kBK - 1) / kBK;
            a.KS = (2 * d.reach + 1) * a.KC;
            const int64_t bm = 64 * v->MI, bn = 64 * v->NJ;
            a.tiles_n = (int32_t)((d.c_out + bn - 1) / bn);
            a.tiles = (int32_t)(((M + bm - 1) / bm) * a.tiles_n);
            a.per_xcd = (a.tiles + kXcds - 1) / kXcds;
            void *params[] = {&a};
            e = hipLaunchKernel(fn, dim3((unsigned)(a.per_xcd * kXcds)), dim3(256), params,
                                (size_t)lds, st);
        }
    } else {
        const int64_t total = M * d.c_out;
        if ((total + 255) / 256 > 0x7fffffffLL)
            return fail(DSATTN_EUNSUPPORTED, "dsattn_temporal_conv: too large for the generic kernel");
        const dim3 grid((unsigned)((total + 255) / 256)), block(256);
        if (d.io_dtype == DSATTN_F32)
            hipLaunchKernelGGL((tconv_generic_kernel<float, float>), grid, block, 0, st,
                               (const float *)X, (const float *)W, bias, (float *)Y, M, d.spatial,
                               d.c_in, d.c_out, d.reach);
        else if (d.out_dtype == DSATTN_F32)
            hipLaunchKernelGGL((tconv_generic_kernel<__bf16, float>), grid, block, 0, st,
                               (const __bf16 *)X, (const __bf16 *)W, bias, (float *)Y, M,
                               d.spatial, d.c_in, d.c_out, d.reach);
        else
            hipLaunchKernelGGL((tconv_generic_kernel<__bf16, __bf16>), grid, block, 0, st,
                               (const __bf16 *)X, (const __bf16 *)W, bias, (__bf16 *)Y, M,
                               d.spatial, d.c_in, d.c_out, d.reach);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return fail(DSATTN_EHIP, "dsattn_temporal_conv: %s", hipGetErrorString(e));
    return DSATTN_OK;
}

}  // extern "C"
