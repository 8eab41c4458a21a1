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

// Position of a variant in the concatenation of the per-head_dim tables: the id that
// dsattn_launch_info reports.
const MfmaVariant *find_variant(int D, int HPW, int NLT, int NGT, bool out_f32, int *id = nullptr)
{
    int base = 0;
    for (VariantTable tab : kTables) {
        int n = 0;
        const MfmaVariant *v = tab(&n);
        for (int i = 0; i < n; ++i)
            if (v[i].D == D && v[i].HPW == HPW && v[i].NLT == NLT && v[i].NGT == NGT &&
                v[i].out_f32 == out_f32) {
                if (id) *id = base + i;
                return &v[i];
            }
        base += n;
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
    // The kernel works on query tiles of 16 frames; a clip is a whole number of them.
    if (d.io_dtype != DSATTN_BF16 || d.clip_len % 16 != 0) return false;
    if (pl.C % 8 != 0) return false;
    // the kernel addresses the 16 frame rows of a tile with 32-bit byte offsets
    if ((int64_t)d.spatial * pl.C * 2 * 16 >= ((int64_t)1 << 32)) return false;
    const int G = (int)pl.global_idx.size();
    // global key tiles: variants exist for 0, 1, 4 and (where a wavefront's registers hold
    // them) 8 tiles; a partly used tile is masked
    if (G > 128) return false;
    const int NGT = G == 0 ? 0 : (G <= 16 ? 1 : (G <= 64 ? 4 : 8));
    // Frames a tile's local scope can reach beyond the tile on each side: up to the end of the
    // clip's local range (the rest of the clip plus the neighbour's context frames), or the
    // sliding window's radius when that is shorter.  With 16-frame clips and no window this is
    // the clip's local context width.
    const int64_t reach = (int64_t)d.clip_len - 16 + d.local_ctx;
    const int64_t wr64 = pl.window >= 0 ? std::min<int64_t>(pl.window, reach) : reach;
    if (wr64 > 16) return false;  // local key tiles: variants exist for 1 to 3
    const int wr = (int)wr64;
    const int n_tiles = pl.F / 16;
    const int R = 16 + 2 * wr;
    const int NLT = (R + 15) / 16;
    const bool out_f32 = d.out_dtype == DSATTN_F32;

    // heads per wavefront: prefer the variant that keeps two wavefronts per SIMD (more loads in
    // flight, compute of one wavefront hidden behind the other), then the widest rows; a
    // wavefront never straddles two positions
    // The set-union option is built into the variants with one global key tile, and into the
    // four-tile variants that run one wavefront per SIMD (head_dim 160 and 128): with that option
    // and four tiles only those are candidates.
    // With eight tiles it is not built in (the generic kernel takes those).
    if ((d.flags & DSATTN_FLAG_DEDUP_GLOBAL) && NGT == 8) return false;
    const bool need_wpe1 = (d.flags & DSATTN_FLAG_DEDUP_GLOBAL) && NGT == 4;
    const MfmaVariant *var = nullptr;
    int var_id = -1;
    const int force_hpw = env_int("DSATTN_HEADS_PER_WAVE", 0);
    for (int wpe : {2, 1}) {
        if (need_wpe1 && wpe != 1) continue;
        for (int cand : {4, 2, 1}) {
            if (force_hpw && cand != force_hpw) continue;
            if (d.heads % cand != 0) continue;
            int id = -1;
            const MfmaVariant *v = find_variant(d.head_dim, cand, NLT, NGT, out_f32, &id);
            if (v && v->WPE == wpe) {
                var = v;
                var_id = id;
                break;
            }
        }
        if (var) break;
    }
    if (!var) return false;
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
    // leave compute units idle.  Every chunk also pays for its start, which decides short videos
    // (four clips: one chunk per row group beats two).
    const double slots = (double)kCus * blocks_cu;
    int best_nc = 1;
    double best_cost = 1e300;
    // (past a few dozen rounds the fill term is 1 and more chunks only add traffic)
    const int nc_cap = (int)std::min<double>(n_tiles, std::max(4096.0, 64.0 * slots / bpc));
    for (int nc = 1; nc <= nc_cap; ++nc) {
        const int m = (n_tiles + nc - 1) / nc;
        if ((n_tiles + m - 1) / m != nc) continue;  // same chunking as a smaller nc
        const double rounds = (double)bpc * nc / slots;
        const double whole = std::floor(rounds);
        const double rem = rounds - whole;
        const double rounds_eff =
            rounds <= 1.0 ? 1.0
                          : whole + (rem > 1e-9 ? (whole < 6.0 && rem < 0.85 ? 1.0
                                                                              : std::max(rem, 0.6))
                                                : 0.0);
        const double fill = rounds_eff / rounds;
        const double kv = (16.0 * m + (nc > 1 ? 2.0 * wr : 0.0) + G) / (16.0 * m);
        // a chunk's start (two memory round trips before its first tile) costs about one tile
        const double cost = (2.0 + 2.0 * kv) / 4.0 * fill * (1.0 + 1.0 / m);
        if (cost < best_cost - 1e-12) {
            best_cost = cost;
            best_nc = nc;
        }
    }
    int m = (n_tiles + best_nc - 1) / best_nc;
    m = std::max(1, std::min(n_tiles, env_int("DSATTN_CLIPS_PER_TASK", m)));
    const int NC = (n_tiles + m - 1) / m;
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
    li.variant = var_id;
    li.ring_reach = wr;

    // everything a launch needs that does not depend on the tensors
    pl.mfma_fn = var->fn;
    pl.gdup = 0;  // entries that repeat an earlier one (the kernel takes at most 64 entries)
    for (size_t j = 0; j < pl.global_idx.size() && j < 64; ++j)
        for (size_t jj = 0; jj < j; ++jj)
            if (pl.global_idx[jj] == pl.global_idx[j]) {
                pl.gdup |= (uint64_t)1 << j;
                break;
            }
    return true;
}

// Raises the kernel's dynamic-LDS cap on the current device to the whole 160 KB (the default
// cap is 64 KB).  Done once per plan, outside the launch path, so that dsattn_forward makes no
// call other than the launch itself (it can be captured into a HIP graph).  The cap is always
// the maximum: plans that share a variant must not lower each other's limit.
hipError_t mfma_prepare(const dsattn_plan_t &pl)
{
    if (!pl.mfma_fn) return hipErrorInvalidValue;
    return hipFuncSetAttribute(pl.mfma_fn, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsPerCu);
}

hipError_t launch_mfma(const dsattn_plan_t &pl, const void *Q, const void *K, const void *V,
                       void *O, bool ctx_mode, hipStream_t st)
{
    // the variant and the duplicate mask were resolved by mfma_plan: nothing is searched here
    const dsattn_desc &d = pl.desc;
    const dsattn_launch_info &li = pl.launch;
    if (!pl.mfma_fn) return hipErrorInvalidValue;
    const int wpb = li.block_threads / 64;

    MfmaArgs a;
    a.Q = (const __bf16 *)Q;
    a.K = (const __bf16 *)K;
    a.V = (const __bf16 *)V;
    a.O = O;
    a.gidx = pl.d_global_idx;
    const int n_tiles = pl.F / 16;
    a.N = n_tiles;
    a.F = pl.F;
    a.h = d.heads;
    a.w = li.ring_reach;
    a.G = (int32_t)pl.global_idx.size();
    a.R = 16 + 2 * li.ring_reach;
    a.clip_len = d.clip_len;
    a.wl = d.local_ctx;
    a.window = pl.window;
    a.M = ctx_mode ? d.clip_len / 16 : li.clips_per_task;
    a.cstride = ctx_mode ? (int64_t)pl.lk_max * d.spatial * pl.C : 0;
    a.RG = d.spatial * (d.heads / li.heads_per_wave);
    a.BPC = a.RG / wpb;
    a.C = pl.C;
    a.FS = (int64_t)d.spatial * pl.C;
    a.sc = pl.scale * 1.4426950408889634f;
    a.gshift = (d.bias_global - d.bias_local) / pl.scale;
    a.dedup = (d.flags & DSATTN_FLAG_DEDUP_GLOBAL) ? 1 : 0;
    a.gdup = pl.gdup;

    // the grid must be exactly chunks x workgroups-per-chunk, each workgroup wpb whole row groups
    const int NC = (n_tiles + a.M - 1) / a.M;
    if (a.RG % wpb != 0 || (!ctx_mode && (int64_t)a.BPC * NC * wpb != (int64_t)li.n_tasks) ||
        (int64_t)a.BPC * NC > 0x7fffffffLL)
        return hipErrorInvalidValue;

    void *params[] = {&a};
    return hipLaunchKernel(pl.mfma_fn, dim3((unsigned)(a.BPC * NC)), dim3((unsigned)li.block_threads),
                           params, (size_t)li.lds_bytes, st);
}

}  // namespace dsattn
