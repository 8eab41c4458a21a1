// Host side of the bf16 MFMA streaming kernel: variant lookup, the launch planner's choices
// for it (heads per wavefront, wavefronts per workgroup, clips per chunk) and the launcher.
#include <algorithm>
#include <cmath>
#include <cstdlib>

#include "mfma_kernel.h"
#include "plan.h"

namespace dsattn {

namespace {

constexpr int kLdsPerCu = 160 * 1024;  // gfx950 LDS per compute unit, also the per-workgroup cap
constexpr int kCus = 256;

typedef const MfmaVariant *(*VariantTable)(int *);
const VariantTable kTables[] = {mfma_variants_d160, mfma_variants_d128, mfma_variants_d96,
                                mfma_variants_d80,  mfma_variants_d64,  mfma_variants_d40,
                                mfma_variants_d32};

const MfmaVariant *find_variant(int D, int HPW, int NLT, int NGT, bool out_f32)
{
    for (VariantTable tab : kTables) {
        int n = 0;
        const MfmaVariant *v = tab(&n);
        for (int i = 0; i < n; ++i)
            if (v[i].D == D && v[i].HPW == HPW && v[i].NLT == NLT && v[i].NGT == NGT &&
                v[i].out_f32 == out_f32)
                return &v[i];
    }
    return nullptr;
}

int env_int(const char *name, int dflt)
{
    const char *e = getenv(name);
    return e && *e ? atoi(e) : dflt;
}

}  // namespace

bool mfma_plan(dsattn_plan_t &pl)
{
    const dsattn_desc &d = pl.desc;
    if (d.io_dtype != DSATTN_BF16 || d.clip_len != 16) return false;
    if (pl.C % 8 != 0) return false;
    // the kernel addresses the 16 frame rows of a tile with 32-bit byte offsets
    if ((int64_t)d.spatial * pl.C * 2 * 16 >= ((int64_t)1 << 32)) return false;
    const int G = (int)pl.global_idx.size();
    // global key tiles: variants exist for 0, 1 and 4 tiles; a partly used tile is masked
    if (G > 64) return false;
    const int NGT = G == 0 ? 0 : (G <= 16 ? 1 : 4);
    const int R = 16 + 2 * d.local_ctx;
    const int NLT = (R + 15) / 16;
    const bool out_f32 = d.out_dtype == DSATTN_F32;

    // heads per wavefront: prefer the variant that keeps two wavefronts per SIMD (more loads in
    // flight, compute of one wavefront hidden behind the other), then the widest rows; a
    // wavefront never straddles two positions
    const MfmaVariant *var = nullptr;
    const int force_hpw = env_int("DSATTN_HEADS_PER_WAVE", 0);
    for (int wpe : {2, 1}) {
        for (int cand : {4, 2, 1}) {
            if (force_hpw && cand != force_hpw) continue;
            if (d.heads % cand != 0) continue;
            const MfmaVariant *v = find_variant(d.head_dim, cand, NLT, NGT, out_f32);
            if (v && v->WPE == wpe) {
                var = v;
                break;
            }
        }
        if (var) break;
    }
    if (!var) return false;
    // the set-union option is built into the variants with one global key tile, and into the
    // four-tile variants that run one wavefront per SIMD (head_dim 160 and 128)
    if ((d.flags & DSATTN_FLAG_DEDUP_GLOBAL) && NGT == 4 && var->WPE != 1) return false;
    const int hpw = var->HPW;
    const int lds_wave = (2 * R + 16) * row_stride_bytes(d.head_dim * hpw);
    if (lds_wave > kLdsPerCu) return false;
    const int RG = d.spatial * (d.heads / hpw);

    // wavefronts per workgroup.  The wavefronts of a workgroup fetch neighbouring rows together
    // (one barrier per clip), so a workgroup should span at least one whole position (all its
    // heads: a contiguous, line-aligned run per frame).  Beyond that, two workgroups per compute
    // unit are better than one: while one starts or drains a chunk the other keeps streaming.
    const int max_waves_cu = std::min(4 * var->WPE, kLdsPerCu / lds_wave);
    const int waves_per_pos = d.heads / hpw;
    const int want = std::min(max_waves_cu, std::max(waves_per_pos, max_waves_cu / 2));
    int wpb = 1;
    for (int cand : {8, 4, 2, 1})
        if (cand <= want && RG % cand == 0) {
            wpb = cand;
            break;
        }
    {
        const int e = env_int("DSATTN_WAVES_PER_BLOCK", wpb);
        if (e >= 1 && e <= 8 && e <= max_waves_cu && RG % e == 0) wpb = e;
    }
    const int blocks_cu = std::max(1, max_waves_cu / wpb);
    const int bpc = RG / wpb;

    // chunks per row group: fewer chunks re-read less context (2w boundary frames + G global
    // frames of K and V per chunk); more chunks fill the machine.  Model: time ~ traffic x fill,
    // where the workgroups run in rounds of `slots`.  With few rounds the workgroups stay in
    // step and a last round less than 85 % full costs a whole round; after about six rounds they have
    // drifted apart and the tail costs little more than its share.  Fewer workgroups than slots
    // leave compute units idle.
    const double slots = (double)kCus * blocks_cu;
    int best_nc = 1;
    double best_cost = 1e300;
    for (int nc = 1; nc <= d.n_clips; ++nc) {
        const int m = (d.n_clips + nc - 1) / nc;
        if ((d.n_clips + m - 1) / m != nc) continue;  // same chunking as a smaller nc
        const double rounds = (double)bpc * nc / slots;
        const double whole = std::floor(rounds);
        const double rem = rounds - whole;
        const double rounds_eff =
            rounds <= 1.0 ? 1.0
                          : whole + (rem > 1e-9 ? (whole < 6.0 && rem < 0.85 ? 1.0
                                                                              : std::max(rem, 0.6))
                                                : 0.0);
        const double fill = rounds_eff / rounds;
        const double kv = (16.0 * m + (nc > 1 ? 2.0 * d.local_ctx : 0.0) + G) / (16.0 * m);
        const double cost = (2.0 + 2.0 * kv) / 4.0 * fill;
        if (cost < best_cost - 1e-12) {
            best_cost = cost;
            best_nc = nc;
        }
    }
    int m = (d.n_clips + best_nc - 1) / best_nc;
    m = std::max(1, std::min(d.n_clips, env_int("DSATTN_CLIPS_PER_TASK", m)));
    const int NC = (d.n_clips + m - 1) / m;
    if ((int64_t)RG * NC > 0x7fffffffLL) return false;

    dsattn_launch_info &li = pl.launch;
    li.kernel = 1;
    li.heads_per_wave = hpw;
    li.local_tiles = NLT;
    li.global_tiles = NGT;
    li.clips_per_task = m;
    li.n_tasks = RG * NC;
    li.block_threads = 64 * wpb;
    li.lds_bytes = lds_wave * wpb;
    return true;
}

// Raises the kernel's dynamic-LDS cap on the current device to the whole 160 KB (the default
// cap is 64 KB).  Done once per plan, outside the launch path, so that dsattn_forward makes no
// call other than the launch itself (it can be captured into a HIP graph).  The cap is always
// the maximum: plans that share a variant must not lower each other's limit.
hipError_t mfma_prepare(const dsattn_plan_t &pl)
{
    const dsattn_desc &d = pl.desc;
    const dsattn_launch_info &li = pl.launch;
    const MfmaVariant *v = find_variant(d.head_dim, li.heads_per_wave, li.local_tiles,
                                        li.global_tiles, d.out_dtype == DSATTN_F32);
    if (!v) return hipErrorInvalidValue;
    return hipFuncSetAttribute(v->fn, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsPerCu);
}

hipError_t launch_mfma(const dsattn_plan_t &pl, const void *Q, const void *K, const void *V,
                       void *O, bool ctx_mode, hipStream_t st)
{
    const dsattn_desc &d = pl.desc;
    const dsattn_launch_info &li = pl.launch;
    const MfmaVariant *v = find_variant(d.head_dim, li.heads_per_wave, li.local_tiles,
                                        li.global_tiles, d.out_dtype == DSATTN_F32);
    if (!v) return hipErrorInvalidValue;
    const int wpb = li.block_threads / 64;

    MfmaArgs a;
    a.Q = (const __bf16 *)Q;
    a.K = (const __bf16 *)K;
    a.V = (const __bf16 *)V;
    a.O = O;
    a.gidx = pl.d_global_idx;
    a.N = d.n_clips;
    a.F = pl.F;
    a.h = d.heads;
    a.w = d.local_ctx;
    a.G = (int32_t)pl.global_idx.size();
    a.R = 16 + 2 * d.local_ctx;
    a.window = pl.window;
    a.M = ctx_mode ? 1 : li.clips_per_task;
    a.cstride = ctx_mode ? (int64_t)pl.lk_max * d.spatial * pl.C : 0;
    a.RG = d.spatial * (d.heads / li.heads_per_wave);
    a.BPC = a.RG / wpb;
    a.C = pl.C;
    a.FS = (int64_t)d.spatial * pl.C;
    a.sc = pl.scale * 1.4426950408889634f;
    a.gshift = (d.bias_global - d.bias_local) / pl.scale;
    a.dedup = (d.flags & DSATTN_FLAG_DEDUP_GLOBAL) ? 1 : 0;
    a.gdup = 0;  // entries that repeat an earlier one (the kernel is used for at most 64 entries)
    for (size_t j = 0; j < pl.global_idx.size() && j < 64; ++j)
        for (size_t jj = 0; jj < j; ++jj)
            if (pl.global_idx[jj] == pl.global_idx[j]) {
                a.gdup |= (uint64_t)1 << j;
                break;
            }

    // the grid must be exactly chunks x workgroups-per-chunk, each workgroup wpb whole row groups
    const int NC = (d.n_clips + a.M - 1) / a.M;
    if (a.RG % wpb != 0 || (!ctx_mode && (int64_t)a.BPC * NC * wpb != (int64_t)li.n_tasks) ||
        (int64_t)a.BPC * NC > 0x7fffffffLL)
        return hipErrorInvalidValue;

    void *params[] = {&a};
    return hipLaunchKernel(v->fn, dim3((unsigned)(a.BPC * NC)), dim3((unsigned)li.block_threads),
                           params, (size_t)li.lds_bytes, st);
}

}  // namespace dsattn
