// bf16 MFMA streaming kernel for Dual-scope temporal attention on gfx950 (Section 4.2 of the
// paper: keys/values of a clip = Concat(local frames, global frames)).
//
// The unit of work is a "query tile": 16 consecutive frames of one clip (the whole clip when a
// clip has 16 frames; below, "clip" in the description of the walk means such a tile).  A tile
// sees the frames within w of it that lie in its clip's local range (the clip's own frames plus
// the context frames of its two neighbours, Section 4.1), where w is the distance the local scope
// can reach beyond the tile: the clip's local context width for 16-frame clips, and for longer
// clips the sliding-window radius of Section 4.2 (or, without a window, the rest of the clip).
//
// Work decomposition.  One wavefront owns a "row group": one spatial position and HPW
// consecutive heads, whose channels are SEG = HPW*D contiguous bf16 per frame, and walks M
// consecutive clips (a "chunk") of that row group in frame order.  A workgroup is WPB
// wavefronts on WPB consecutive row groups of the same chunk, i.e. a contiguous span of
// WPB*SEG channels per frame; one barrier per clip keeps their memory requests close in
// time, so that neighbouring rows' cache lines and DRAM pages are touched together.
// Workgroups are numbered chunk-major: the whole machine sweeps the same frames at once.
//   * Global K/V (G frames) are loaded once per task and kept in registers, already in MFMA
//     operand form.
//   * Local K/V live in an LDS ring of R = 16 + 2w frame rows per wavefront.  Clip i needs
//     frames [16i - w, 16i + 16 + w); stepping to clip i+1 replaces exactly the 16 oldest rows,
//     so every frame of the chunk is read from HBM once and the boundary frames shared with
//     the neighbouring clips (c_pre / c_post of Section 4.1) are reused on chip.
//   * The next clip's Q/K/V rows are in flight in registers while the current clip is computed.
// Per clip and head:  S^T = K Q^T  (16x16x32 bf16 MFMA, keys on M, the 16 query frames on N),
// fp32 softmax over keys (maximum: in-lane plus two cross-lane row swaps; weights exp2 with the
// scale folded in), P^T rounded to bf16 and fed straight back as the B operand of  O^T = V^T P^T
// (16x16x16 bf16 MFMA per key tile, or 16x16x32 per pair of key tiles when both scopes have an even
// number of tiles).  The denominator is the sum of the rounded weights, taken by one more MFMA
// with an all-ones A operand.  V^T operands are made from row-major V rows with an MFMA against a
// 0/1 selector matrix, which is exact.
// Options of the scopes: the biases of the two scopes' logits enter as one shift of the raw global
// scores (a softmax sees only their difference); a sliding window |key frame - query frame| <= r
// on the local scope is a per-lane mask on the local scores; the set-union option drops, per
// query, the global keys whose frame that query already sees.
//
// LDS regions are private to a wavefront; the barrier orders nothing, it only paces.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dsattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct MfmaArgs {
    const __bf16 *Q, *K, *V;
    void *O;
    const int32_t *gidx;  // device [G]
    int32_t N;    // query tiles of 16 frames in the video = F / 16 (= clips when a clip has 16 frames)
    int32_t F, h;
    int32_t w;    // frames the ring holds beyond a query tile on each side, R = 16 + 2 w
    int32_t G, R;
    int32_t clip_len;  // F_clip, a multiple of 16
    int32_t wl;        // local context width of a clip (frames taken from each neighbouring clip)
    int32_t window;  // sliding-window radius of the local scope, -1 = none
    int32_t M;    // query tiles per chunk
    int32_t RG;   // row groups = P * h / HPW
    int32_t BPC;  // workgroups per chunk = RG / WPB
    int32_t C;
    int64_t FS;   // frame stride in elements = P * C
    float sc;     // scale * log2(e), > 0
    float gshift; // (bias_global - bias_local) / scale: the scope biases as a shift of the raw
                  // global scores (the softmax only sees the difference of the two biases)
    int32_t dedup;   // set union: drop a global entry whose frame the query already sees
    uint64_t gdup;   // bit j: global entry j repeats an earlier global entry
    int64_t cstride; // 0: K and V are [F, P, C].  Otherwise they are materialised contexts
                     // [n_clips, lk_max, P, C] (clip i: its local frames ascending, then the
                     // global entries) with cstride = lk_max * P * C elements per clip, and a
                     // chunk is exactly one clip (M = clip_len / 16)
};

struct MfmaVariant {
    int D, HPW, NLT, NGT, WPE;
    bool out_f32;
    const void *fn;
};

// LDS row stride in bytes for a row of `seg` bf16: padded so that consecutive rows start 4 banks
// apart modulo 8 (16-byte reads of 8 consecutive rows then touch all 32 banks once).
__host__ __device__ constexpr int row_stride_bytes(int seg)
{
    return ((seg / 2 + 4) % 8 == 4) ? seg * 2 + 16 : seg * 2 + 32;
}

// Orders LDS accesses of the wavefront's lanes: LDS operations of one wavefront execute in
// issue order, so only the compiler has to be kept from moving them.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Maximum over the lanes l, l ^ 16, l ^ 32, l ^ 48 (the four row groups of one MFMA column) with
// the row-swap instructions of gfx950: no trip through the LDS crossbar.  A swap of x with itself
// leaves the partner row's value in one of the two results.
__device__ __forceinline__ float colmax(float x)
{
    {
        const unsigned a = __builtin_bit_cast(unsigned, x);
        const auto r = __builtin_amdgcn_permlane16_swap(a, a, false, false);
        const unsigned r0 = r[0], r1 = r[1];
        x = fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
    }
    {
        const unsigned a = __builtin_bit_cast(unsigned, x);
        const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
        const unsigned r0 = r[0], r1 = r[1];
        x = fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
    }
    return x;
}

// The multiply-accumulate of the accumulator chains of O^T = V^T P^T and of the denominator.  A
// kernel variant takes its key tiles either in pairs (32 keys per 16x16x32 instruction) or one
// by one (16 keys per 16x16x16 instruction), never both.  The matrix cores hand an accumulator
// from one instruction straight to the next only between instructions of the same shape; a
// 16x16x32 that takes a 16x16x16's result as its C operand right behind it reads elements 2 and
// 3 before they are written (the other way round: elements 0 and 1), and this toolchain puts no
// wait state between the two.  Checked with a two-instruction probe on the device: no wait,
// those elements stale in every lane; a few s_nop in between, or the same shape twice, correct.
// Every step of those chains goes through PvChain<kPairs>::mac, whose operand types fit one
// instruction only, so a chain that mixes the two does not compile.
template <bool PAIRS>
struct PvChain;
template <>
struct PvChain<true> {
    static __device__ __forceinline__ f32x4 mac(const bf16x8 a, const bf16x8 b, const f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <>
struct PvChain<false> {
    static __device__ __forceinline__ f32x4 mac(const bf16x4 a, const bf16x4 b, const f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a),
                                                        __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
    }
};

// WPE = wavefronts per SIMD the register budget is sized for (2: 256 VGPRs, 1: 512); a
// workgroup is at most 4 * WPE wavefronts so that it fits one compute unit.
template <int D, int HPW, int NLT, int NGT, int WPE, bool OUT_F32>
__global__ __launch_bounds__(256 * WPE, WPE) void dsattn_mfma_kernel(const MfmaArgs a)
{
    constexpr int SEG = D * HPW;          // bf16 per frame row of this row group
    constexpr int NCH = SEG / 8;          // 16-byte chunks per row
    constexpr int NLD = (NCH + 3) / 4;    // 64-lane load instructions per 16-row tile
    constexpr int RS = row_stride_bytes(SEG);
    constexpr int NKB = (D + 31) / 32;    // 32-wide contraction blocks of QK^T
    constexpr int NDT = (D + 15) / 16;    // 16-row tiles of O^T
    constexpr int DCH = D / 8;            // chunks per head
    constexpr int NT = NLT + NGT;
    static_assert(D % 8 == 0, "head_dim must be a multiple of 8");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int R = a.R;
    const int lane = threadIdx.x & 63;
    // (readfirstlane tells the compiler that everything derived from the wavefront's index is
    // uniform: the row group's base pointers and the buffer descriptors then live in scalar
    // registers)
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int WPB = blockDim.x >> 6;
    unsigned char *kring = smem + wv * ((2 * R + 16) * RS);
    unsigned char *vring = kring + R * RS;
    unsigned char *qo = kring + 2 * R * RS;

    const int l16 = lane & 15;  // MFMA row (A) / column (B, C) index
    const int lg = lane >> 4;   // MFMA k-group (A, B) / row-group (C) index

    // ---- task decode, chunk-major: workgroup b handles chunk b / BPC
    const int ck = blockIdx.x / a.BPC;
    const int rg = (blockIdx.x - ck * a.BPC) * WPB + wv;
    const int hg = a.h / HPW;
    const int p = rg / hg;
    const int g0 = (rg - p * hg) * HPW;
    const int64_t rowoff = (int64_t)p * a.C + (int64_t)g0 * D;
    const int c0 = ck * a.M;
    const int c1 = min(a.N, c0 + a.M);
    const int w = a.w;
    const int F = a.F;
    const int64_t FSB = a.FS * 2;  // frame stride in bytes

    const unsigned char *Qb = (const unsigned char *)(a.Q + rowoff);
    const unsigned char *Kb = (const unsigned char *)(a.K + rowoff);
    const unsigned char *Vb = (const unsigned char *)(a.V + rowoff);
    // Materialised context (one clip per chunk): row j of clip c0's slab is local frame lo + j,
    // then global entry j - (hi - lo).  Moving the bases so that "frame f" of the slab sits at
    // f * FSB keeps every local address below as it is; global entry j becomes "frame" hi + j.
    // Frames that may be read at all: the video, or the clip's slab.
    int gfirst = -1;
    int flo = 0, fhi = F;
    if (a.cstride != 0) {
        const int ci = ck;  // one clip per chunk
        const int lo = max(0, ci * a.clip_len - a.wl), hi = min(F, (ci + 1) * a.clip_len + a.wl);
        const int64_t shift = ((int64_t)ci * a.cstride - (int64_t)lo * a.FS) * 2;
        Kb += shift;
        Vb += shift;
        gfirst = hi;
        flo = lo;
        fhi = hi;
    }

    // per-lane load geometry: lane-load `r` covers tile row fq[r], 16-byte chunk cq;
    // voff = byte offset from the tile's first frame row, loff = byte offset in a 16-row LDS tile
    constexpr bool kFullTile = (16 * NCH) % 64 == 0;  // every lane of every load is in the tile
    uint32_t voff[NLD], loff[NLD], coff[NLD];
    int fq[NLD];
#pragma unroll
    for (int r = 0; r < NLD; ++r) {
        const int idx = lane + 64 * r;
        fq[r] = idx / NCH;
        const int cq = idx - fq[r] * NCH;
        coff[r] = (uint32_t)cq * 16u;
        voff[r] = (uint32_t)fq[r] * (uint32_t)FSB + coff[r];
        loff[r] = (uint32_t)(fq[r] * RS) + coff[r];
    }
    // only the last of the NLD lane-loads can reach past the 16-row tile, and only when the
    // tile is not a whole number of 64-lane loads
    auto in_tile = [&](int r) __attribute__((always_inline)) -> bool {
        return kFullTile || r + 1 < NLD || lane + 64 * r < 16 * NCH;
    };

    // 16 consecutive frames starting at frame0 (wave-uniform); rows >= nrows and frames
    // outside [lo, hi) give zeros.  A tile that lies inside [lo, hi) is read with plain loads.
    // Any other is read through a buffer descriptor that covers exactly the frames that may be
    // read: it starts at the first such frame and ends with the last, so a lane whose row lies
    // before (its offset wraps to a huge unsigned value; 16 frame rows span less than 2^32
    // bytes) or after gets zeros from the hardware's range check, with no per-lane test and no
    // branch per load (the tiles at the ends of the video and of a clip's slab, which are every
    // other tile of a short video); no frame readable: loads that touch no memory.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr uint32_t kOob = 0xfffffff0u;
    auto load_rows = [&](const unsigned char *base, int frame0, int nrows, int lo, int hi,
                         uint4(&st)[NLD]) __attribute__((always_inline)) {
        if (nrows == 16 && frame0 >= lo && frame0 + 16 <= hi) {
            const unsigned char *tb = base + (int64_t)frame0 * FSB;
#pragma unroll
            for (int r = 0; r < NLD; ++r) {
                if (kFullTile || r + 1 < NLD) {
                    st[r] = *(const uint4 *)(tb + voff[r]);
                } else {
                    uint4 x = make_uint4(0, 0, 0, 0);
                    if (in_tile(r)) x = *(const uint4 *)(tb + voff[r]);
                    st[r] = x;
                }
            }
        } else {
            const int bf = max(frame0, lo);          // first frame that may be read
            const int hv = min(hi, frame0 + nrows);  // one past the last
            const uint32_t delta = (uint32_t)(bf - frame0) * (uint32_t)FSB;
            const int64_t span = (int64_t)(hv - bf) * FSB;
            const uint32_t nrec = span > 0 ? (uint32_t)span : 0u;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(base + (int64_t)(nrec ? bf : 0) * FSB), 0, (int)nrec, 0x00020000);
#pragma unroll
            for (int r = 0; r < NLD; ++r) {
                uint32_t off = voff[r] - delta;
                if (!(kFullTile || r + 1 < NLD)) off = in_tile(r) ? off : kOob;
                const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
                st[r] = make_uint4(x[0], x[1], x[2], x[3]);
            }
        }
    };
    // tile rows to LDS rows (slot0 + fq) mod ring of `buf`; rows >= nrows are not written
    auto store_rows = [&](unsigned char *buf, int slot0, int nrows, int ring,
                          const uint4(&st)[NLD]) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < NLD; ++r) {
            const int wrap = (slot0 + fq[r] >= ring) ? ring : 0;
            if (in_tile(r) && fq[r] < nrows)
                *(uint4 *)(buf + (slot0 - wrap) * RS + loff[r]) = st[r];
        }
    };
    // the same for a whole 16-row tile
    auto store_tile = [&](unsigned char *buf, int slot0, int ring, const uint4(&st)[NLD])
                          __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < NLD; ++r) {
            const int wrap = (slot0 + fq[r] >= ring) ? ring : 0;
            if (in_tile(r)) *(uint4 *)(buf + (slot0 - wrap) * RS + loff[r]) = st[r];
        }
    };

    // A/B operand of the 16x16x32 MFMA: row `row` of an LDS tile, head `hh`, block `kb`;
    // channels past the head's D are zero.  When D is not a multiple of 32 the lanes past the head
    // read the first 16 bytes of the row's padding instead, which are cleared once below and
    // never written again (tile stores write the rows' data chunks only).
    constexpr bool kPadChunk = D % 32 != 0;
    if constexpr (kPadChunk) {
        for (int r = lane; r < 2 * R + 16; r += 64)
            *(uint4 *)(kring + r * RS + SEG * 2) = make_uint4(0, 0, 0, 0);
        wave_sync();
    }
    auto read_op32 = [&](const unsigned char *buf, int row, int hh, int kb)
                         __attribute__((always_inline)) -> bf16x8 {
        const int ch = 4 * kb + lg;  // chunk within the head
        int off = (hh * DCH + ch) * 16;
        if (!(4 * kb + 3 < DCH) && ch >= DCH) off = SEG * 2;
        const uint4 x = *(const uint4 *)(buf + row * RS + off);
        return __builtin_bit_cast(bf16x8, x);
    };

    // 0/1 selector operands: sel[hf] picks channels 16*hf .. 16*hf+15 of a 32-wide block
    bf16x8 sel[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int e = 0; e < 8; ++e)
            sel[hf][e] = (8 * lg + e == 16 * hf + l16) ? (__bf16)1.0f : (__bf16)0.0f;

    // A operands that are all ones (row sums of P^T)
    bf16x8 ones8;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones8[e] = (__bf16)1.0f;
    const bf16x4 ones4 = __builtin_shufflevector(ones8, ones8, 0, 1, 2, 3);

    // V^T operand for channels 16*(2kb+hf) .. +15 from the V operand `av` (16 keys x 32 channels):
    // an exact transpose through the matrix core.  The lane gets keys 4 lg .. 4 lg + 3 of channel
    // l16: the A operand of the 16x16x16 MFMA, or one half of the A operand of a 16x16x32 MFMA
    // over a pair of key tiles.
    auto vt_from = [&](const bf16x8 av, int hf) __attribute__((always_inline)) -> bf16x4 {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, sel[hf], z, 0, 0, 0);
        bf16x4 b;
#pragma unroll
        for (int e = 0; e < 4; ++e) b[e] = (__bf16)z[e];  // exact: z holds bf16 values
        return b;
    };
    auto join = [](const bf16x4 x, const bf16x4 y) __attribute__((always_inline)) -> bf16x8 {
        return __builtin_shufflevector(x, y, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // When both scopes have an even number of key tiles, the tiles enter O^T = V^T P^T in pairs
    // (32 keys per 16x16x32 MFMA: k-group lg holds keys 4 lg .. 4 lg + 3 of the pair's first tile,
    // then of its second, in both operands).  Otherwise every tile goes through the 16x16x16 MFMA:
    // an accumulator chain never mixes the two instructions.
    constexpr bool kPairs = NGT % 2 == 0 && NLT % 2 == 0;
    using Chain = PvChain<kPairs>;
    constexpr int NGP = kPairs ? NGT / 2 : 0, NLP = kPairs ? NLT / 2 : 0;  // tile pairs
    constexpr int NGS = NGT - 2 * NGP, NLS = NLT - 2 * NLP;                // single tiles
    // The accumulator chains of O^T and of the denominator run over the pairs (16x16x32) and
    // over the single tiles (16x16x16): one of the two sets must be empty.
    static_assert((NGP + NLP == 0) || (NGS + NLS == 0),
                  "an accumulator chain would mix the 16x16x32 and the 16x16x16 instruction");

    // ---- prologue.  Independent loads are issued together so that the chunk starts after
    // two memory round trips: (1) global frame indices, boundary frames, Q of the first clip;
    // (2) global K/V rows, K/V of the first clip.
    bf16x8 kg[NGT > 0 ? NGT : 1][HPW][NKB];
    bf16x8 vgp[NGP > 0 ? NGP : 1][HPW][NDT];  // V^T of the global tile pairs
    bf16x4 vgs[NGS > 0 ? NGS : 1][HPW][NDT];  // V^T of the single global tiles
    // Rows on their way from memory: a tile's rows are asked for one tile ahead of their use.
    // (Asking two tiles ahead, with a second register set where a wavefront has a whole SIMD's
    // registers, was measured and changed nothing: the kernel is not short of loads in flight.)
    uint4 stQ[NLD], stK[NLD], stV[NLD];
    uint4 gK[NLD], gV[NLD];

    // global K/V rows of key tile tg -> gK, gV (zeros past the G-th global frame)
    auto load_global_tile = [&](int tg) __attribute__((always_inline)) {
        int gf[NLD];
#pragma unroll
        for (int r = 0; r < NLD; ++r) {
            const int j = 16 * tg + fq[r];
            gf[r] = -1;
            if (in_tile(r) && j < a.G) gf[r] = gfirst >= 0 ? gfirst + j : a.gidx[j];
        }
#pragma unroll
        for (int r = 0; r < NLD; ++r) {
            gK[r] = make_uint4(0, 0, 0, 0);
            gV[r] = make_uint4(0, 0, 0, 0);
            if (gf[r] >= 0) {
                const int64_t goff = (int64_t)gf[r] * FSB + coff[r];
                gK[r] = *(const uint4 *)(Kb + goff);
                gV[r] = *(const uint4 *)(Vb + goff);
            }
        }
    };

    // boundary frames that precede the first bulk tile: 2w rows, 16 per local tile
    if constexpr (NLT >= 2) {
        load_rows(Kb, 16 * c0 - w, min(16, 2 * w), flo, fhi, stK);
        load_rows(Vb, 16 * c0 - w, min(16, 2 * w), flo, fhi, stV);
    }
    load_rows(Qb, 16 * c0, 16, 0, F, stQ);
    if constexpr (NGT > 0) load_global_tile(0);
    if constexpr (NLT >= 2) {
        const int s0 = (16 * c0) % R;  // slot of frame f is (f + w) mod R
        store_rows(kring, s0, min(16, 2 * w), R, stK);
        store_rows(vring, s0, min(16, 2 * w), R, stV);
    }
#pragma unroll
    for (int tl = 1; tl + 1 < NLT; ++tl) {
        const int nrows = min(16, 2 * w - 16 * tl);
        if (nrows > 0) {
            const int f0 = 16 * c0 - w + 16 * tl;
            load_rows(Kb, f0, nrows, flo, fhi, stK);
            load_rows(Vb, f0, nrows, flo, fhi, stV);
            const int s0 = (16 * c0 + 16 * tl) % R;
            store_rows(kring, s0, nrows, R, stK);
            store_rows(vring, s0, nrows, R, stV);
        }
    }
    // first bulk tile of K/V: frames [16 c0 + w, +16)
    load_rows(Kb, 16 * c0 + w, 16, flo, fhi, stK);
    load_rows(Vb, 16 * c0 + w, 16, flo, fhi, stV);

    // global context into registers in MFMA operand form, staged through the Q/O buffer
#pragma unroll
    for (int tg = 0; tg < NGT; ++tg) {
        if (tg > 0) load_global_tile(tg);
        wave_sync();
        store_tile(qo, 0, 16, gK);
        wave_sync();
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) kg[tg][hh][kb] = read_op32(qo, l16, hh, kb);
        wave_sync();
        store_tile(qo, 0, 16, gV);
        wave_sync();
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const bf16x8 av = read_op32(qo, l16, hh, kb);
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
                    if (2 * kb + hf < NDT) {
                        const bf16x4 t = vt_from(av, hf);
                        if (tg < 2 * NGP) {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                vgp[tg / 2][hh][2 * kb + hf][4 * (tg & 1) + e] = t[e];
                        } else {
                            vgs[tg - 2 * NGP][hh][2 * kb + hf] = t;
                        }
                    }
            }
    }

    // weights of local keys past the ring's R rows are cleared after rounding (their scores
    // repeat row R - 1, see arow below): masks of this lane's keys 4 lg + e of local tile tl
    // (R is even, so the two keys of a packed pair are kept or cleared together)
    bool pkeep[NLT][2];
#pragma unroll
    for (int tl = 0; tl < NLT; ++tl)
#pragma unroll
        for (int q = 0; q < 2; ++q) pkeep[tl][q] = 16 * tl + 4 * lg + 2 * q < R;
    // no option and no partly used global tile: interior clips need no per-score masks
    // The set-union option is built into the variants with one global key tile and into the
    // four-tile variants that have a whole SIMD's registers (the others have none to spare; the
    // planner does not pick them with that option).
    constexpr bool kDedup = NGT == 1 || (NGT == 4 && WPE == 1);
    const bool plain_opts = a.window < 0 && a.gshift == 0.f && a.G == 16 * NGT &&
                            !(kDedup && a.dedup);

    // set union: lane j keeps the frame of global entry j
    int gown = -1;
    if (kDedup && a.dedup && lane < a.G) gown = a.gidx[lane];

    int s_bulk = (16 * c0 + 2 * w) % R;  // ring slot of the bulk tile's first row
    int b0 = (16 * c0) % R;              // ring slot of the window's first frame (16 i - w)

    for (int i = c0; i < c1; ++i) {
        if (WPB > 1) __builtin_amdgcn_s_barrier();  // pacing only: no data crosses wavefronts
        wave_sync();
        store_tile(qo, 0, 16, stQ);
        store_tile(kring, s_bulk, R, stK);
        store_tile(vring, s_bulk, R, stV);
        // (past the chunk's last tile: zero rows, loads that touch no memory)
        const int nnext = i + 1 < c1 ? 16 : 0;
        load_rows(Qb, 16 * (i + 1), nnext, 0, F, stQ);
        load_rows(Kb, 16 * (i + 1) + w, nnext, flo, fhi, stK);
        load_rows(Vb, 16 * (i + 1) + w, nnext, flo, fhi, stV);
        wave_sync();

        // validity of this lane's local keys: C/D row 4*lg + e of local tile tl is ring slot
        // 16 tl + 4 lg + e, holding frame 16 i - w + ((slot - b0) mod R)
        // The tile's clip and that clip's local range [clo, chi): the clip's own frames plus wl
        // frames of each neighbouring clip, cut at the ends of the video (Section 4.1).
        const int clip = (16 * i) / a.clip_len;
        const int clo = max(0, clip * a.clip_len - a.wl);
        const int chi = min(F, (clip + 1) * a.clip_len + a.wl);
        bool lvalid[NLT][4];
        int arow[NLT];  // ring row this lane feeds as MFMA row l16 of local tile tl (clamped)
        const bool interior = 16 * i - w >= clo && 16 * i + 16 + w <= chi;
#pragma unroll
        for (int tl = 0; tl < NLT; ++tl) {
            arow[tl] = min(16 * tl + l16, R - 1);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int s = 16 * tl + 4 * lg + e;
                bool ok = s < R;
                if (!interior || a.window >= 0) {
                    int rel = s - b0;
                    if (rel < 0) rel += R;
                    const int f = 16 * i - w + rel;
                    ok = ok && f >= clo && f < chi;
                    // sliding window: key frame f against this lane's query frame 16 i + l16
                    if (a.window >= 0) ok = ok && abs(rel - w - l16) <= a.window;
                }
                lvalid[tl][e] = ok;
            }
        }

        // set union: bit 4 tg + e says that this lane's global key 16 tg + 4 lg + e is dropped for
        // its query (frame 16 i + l16): it repeats an earlier global entry, or its frame is a
        // visible local key of that query
        uint32_t ghid = 0;
        if (kDedup && a.dedup) {
            const int lo = max(clo, 16 * i - w), hi = min(chi, 16 * i + 16 + w);
            const int aq = 16 * i + l16;
#pragma unroll
            for (int tg = 0; tg < NGT; ++tg)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int jk = 16 * tg + 4 * lg + e;
                    const int gf = __shfl(gown, jk);
                    bool hid = (a.gdup >> jk) & 1;
                    hid = hid || (gf >= lo && gf < hi && (a.window < 0 || abs(gf - aq) <= a.window));
                    ghid |= (uint32_t)hid << (4 * tg + e);
                }
        }

#pragma unroll
        for (int hh = 0; hh < HPW; ++hh) {
            // ---- S^T = K Q^T for all key tiles
            f32x4 s[NT];
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) s[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const bf16x8 qop = read_op32(qo, l16, hh, kb);
#pragma unroll
                for (int tg = 0; tg < NGT; ++tg)
                    s[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kg[tg][hh][kb], qop, s[tg], 0, 0,
                                                                    0);
#pragma unroll
                for (int tl = 0; tl < NLT; ++tl) {
                    const bf16x8 ak = read_op32(kring, arow[tl], hh, kb);
                    s[NGT + tl] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak, qop, s[NGT + tl], 0, 0, 0);
                }
            }

            // ---- softmax over keys, per query column (fp32).  The maximum is taken over raw
            // scores (scale > 0), weights are exp2(raw * sc - max * sc); masked keys sit at -inf
            // and come out as exact zeros.  The scope bias enters as a shift of the global scores.
            float mx = -INFINITY;
            if (plain_opts && interior) {
                // every ring row and every global row is a key; rows past R repeat row R - 1, so
                // they do not change the maximum, and their weights are cleared below
#pragma unroll
                for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) mx = fmaxf(mx, s[tt][e]);
            } else {
                const bool g_full = a.G == 16 * NGT;  // no partly used global key tile
#pragma unroll
                for (int tg = 0; tg < NGT; ++tg)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float x = s[tg][e];
                        if (a.gshift != 0.f) x += a.gshift;
                        if (!g_full && !(16 * tg + 4 * lg + e < a.G)) x = -INFINITY;
                        if (kDedup && a.dedup && ((ghid >> (4 * tg + e)) & 1)) x = -INFINITY;
                        s[tg][e] = x;
                        mx = fmaxf(mx, x);
                    }
#pragma unroll
                for (int tl = 0; tl < NLT; ++tl)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float x = lvalid[tl][e] ? s[NGT + tl][e] : -INFINITY;
                        s[NGT + tl][e] = x;
                        mx = fmaxf(mx, x);
                    }
            }
            mx = colmax(mx);
            const float nm = -mx * a.sc;
            // rounded weights of key tile tt (this lane: keys 4 lg + e, query l16)
            auto weights = [&](int tt) __attribute__((always_inline)) -> bf16x4 {
                bf16x4 pb;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    pb[e] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[tt][e], a.sc, nm));  // RNE
                if (tt > NGT) {  // a local tile after the first may reach past the ring
                    uint2 u = __builtin_bit_cast(uint2, pb);
                    u.x = pkeep[tt - NGT][0] ? u.x : 0u;
                    u.y = pkeep[tt - NGT][1] ? u.y : 0u;
                    pb = __builtin_bit_cast(bf16x4, u);
                }
                return pb;
            };
            bf16x8 ptp[NGP + NLP > 0 ? NGP + NLP : 1];  // global pairs, then local pairs
            bf16x4 ptg[NGS > 0 ? NGS : 1], ptl[NLS > 0 ? NLS : 1];  // single tiles
            // the denominator is the sum of the *rounded* weights, taken on the matrix core:
            // a row of ones times P^T leaves sum_k P^T[k][a] in every row of column a
            f32x4 den = {0.f, 0.f, 0.f, 0.f};
            if constexpr (kPairs) {
#pragma unroll
                for (int u = 0; u < NGP; ++u) {
                    ptp[u] = join(weights(2 * u), weights(2 * u + 1));
                    den = Chain::mac(ones8, ptp[u], den);
                }
#pragma unroll
                for (int u = 0; u < NLP; ++u) {
                    ptp[NGP + u] = join(weights(NGT + 2 * u), weights(NGT + 2 * u + 1));
                    den = Chain::mac(ones8, ptp[NGP + u], den);
                }
            } else {
#pragma unroll
                for (int u = 0; u < NGS; ++u) {
                    ptg[u] = weights(u);
                    den = Chain::mac(ones4, ptg[u], den);
                }
#pragma unroll
                for (int u = 0; u < NLS; ++u) {
                    ptl[u] = weights(NGT + u);
                    den = Chain::mac(ones4, ptl[u], den);
                }
            }
            const float inv = __builtin_amdgcn_rcpf(den[0]);  // within 1 ulp

            // ---- O^T = V^T P^T
            f32x4 o[NDT];
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
            if constexpr (kPairs) {
#pragma unroll
                for (int u = 0; u < NGP; ++u)
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) o[dt] = Chain::mac(vgp[u][hh][dt], ptp[u], o[dt]);
#pragma unroll
                for (int u = 0; u < NLP; ++u)
#pragma unroll
                    for (int kb = 0; kb < NKB; ++kb) {
                        const bf16x8 av0 = read_op32(vring, arow[2 * u], hh, kb);
                        const bf16x8 av1 = read_op32(vring, arow[2 * u + 1], hh, kb);
#pragma unroll
                        for (int hf = 0; hf < 2; ++hf) {
                            const int dt = 2 * kb + hf;
                            if (dt < NDT)
                                o[dt] = Chain::mac(join(vt_from(av0, hf), vt_from(av1, hf)),
                                                   ptp[NGP + u], o[dt]);
                        }
                    }
            } else {
#pragma unroll
                for (int u = 0; u < NGS; ++u)
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) o[dt] = Chain::mac(vgs[u][hh][dt], ptg[u], o[dt]);
#pragma unroll
                for (int u = 0; u < NLS; ++u)
#pragma unroll
                    for (int kb = 0; kb < NKB; ++kb) {
                        const bf16x8 av = read_op32(vring, arow[u], hh, kb);
#pragma unroll
                        for (int hf = 0; hf < 2; ++hf) {
                            const int dt = 2 * kb + hf;
                            if (dt < NDT) o[dt] = Chain::mac(vt_from(av, hf), ptl[u], o[dt]);
                        }
                    }
            }

            // ---- normalise; lane holds channels 16 dt + 4 lg + {0..3} of query frame l16
            if constexpr (OUT_F32) {
                float *Ob = (float *)a.O + rowoff + (int64_t)(16 * i + l16) * a.FS + hh * D;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    const int d = 16 * dt + 4 * lg;
                    if (16 * dt + 15 < D || d < D) {
                        f32x4 y = o[dt] * inv;
                        *(f32x4 *)(Ob + d) = y;
                    }
                }
            } else {
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    const int d = 16 * dt + 4 * lg;
                    if (16 * dt + 15 < D || d < D) {
                        bf16x4 y;
#pragma unroll
                        for (int e = 0; e < 4; ++e) y[e] = (__bf16)(o[dt][e] * inv);
                        *(bf16x4 *)(qo + l16 * RS + (hh * D + d) * 2) = y;
                    }
                }
            }
        }

        if constexpr (!OUT_F32) {
            // ---- O rows back out of LDS as full 16-byte lanes, coalesced along channels
            wave_sync();
            unsigned char *Ob = (unsigned char *)((__bf16 *)a.O + rowoff) + (int64_t)(16 * i) * FSB;
#pragma unroll
            for (int r = 0; r < NLD; ++r)
                if (in_tile(r)) *(uint4 *)(Ob + voff[r]) = *(const uint4 *)(qo + loff[r]);
        }

        s_bulk += 16;
        if (s_bulk >= R) s_bulk -= R;
        b0 += 16;
        if (b0 >= R) b0 -= R;
    }
}

// Variant tables, one translation unit per head_dim.
const MfmaVariant *mfma_variants_d160(int *n);
const MfmaVariant *mfma_variants_d128(int *n);
const MfmaVariant *mfma_variants_d96(int *n);
const MfmaVariant *mfma_variants_d80(int *n);
const MfmaVariant *mfma_variants_d64(int *n);
const MfmaVariant *mfma_variants_d40(int *n);
const MfmaVariant *mfma_variants_d32(int *n);

#define DSATTN_MFMA_VARIANT(D, HPW, NLT, NGT, WPE)                                             \
    {D, HPW, NLT, NGT, WPE, false,                                                             \
     (const void *)&dsattn_mfma_kernel<D, HPW, NLT, NGT, WPE, false>},                         \
    {D, HPW, NLT, NGT, WPE, true, (const void *)&dsattn_mfma_kernel<D, HPW, NLT, NGT, WPE, true>}

// local context 0..16 frames (1 to 3 local key tiles), no or one global key tile
#define DSATTN_MFMA_SET(D, HPW, WPE)                                                           \
    DSATTN_MFMA_VARIANT(D, HPW, 1, 0, WPE), DSATTN_MFMA_VARIANT(D, HPW, 1, 1, WPE),            \
    DSATTN_MFMA_VARIANT(D, HPW, 2, 0, WPE), DSATTN_MFMA_VARIANT(D, HPW, 2, 1, WPE),            \
    DSATTN_MFMA_VARIANT(D, HPW, 3, 0, WPE), DSATTN_MFMA_VARIANT(D, HPW, 3, 1, WPE)

// four global key tiles, local context 0..16 frames
#define DSATTN_MFMA_SET_G4(D, HPW, WPE)                                                        \
    DSATTN_MFMA_VARIANT(D, HPW, 1, 4, WPE), DSATTN_MFMA_VARIANT(D, HPW, 2, 4, WPE),            \
    DSATTN_MFMA_VARIANT(D, HPW, 3, 4, WPE)

// eight global key tiles (up to 128 global frames), local context 0..16 frames
#define DSATTN_MFMA_SET_G8(D, HPW, WPE)                                                        \
    DSATTN_MFMA_VARIANT(D, HPW, 1, 8, WPE), DSATTN_MFMA_VARIANT(D, HPW, 2, 8, WPE),            \
    DSATTN_MFMA_VARIANT(D, HPW, 3, 8, WPE)

}  // namespace dsattn
