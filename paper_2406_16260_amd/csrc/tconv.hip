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
// MFMA kernel.  A workgroup of WVM x WVN = 8 wavefronts (two per SIMD) computes a
// (32 MI WVM) x (32 NJ WVN) tile of Y; wavefront (wm, wn) owns a (32 MI) x (32 NJ) part as
// 16 x 16 accumulators of v_mfma_f32_16x16x32_bf16 (W rows as the A operand, X rows as the B
// operand).
// The contraction runs in stages of 64 channels of one tap, taps innermost.  A stage's X rows
// and W rows (one 128-byte cache line each) go from global memory straight into LDS with
// buffer_load ... lds, into one of two slots, while the other slot is multiplied out; one
// barrier per stage.  The LDS rows are unpadded (the load instruction fixes the layout) and
// XOR-swizzled in 16-byte chunks, which keeps the operand reads free of bank conflicts.  The
// matrix instructions, the LDS reads of the next fragments and the issue of the next stage's
// loads are interleaved by hand.  Rows outside the video are zeroed by the buffer descriptor's
// range check, not by code.  The workgroups are persistent: at most one per compute unit, the
// same number on every XCD, each walking its share of the output tiles as one continuous stream
// of stages (the next tile's first stage is loading while the finished tile is stored).  An XCD
// walks a contiguous run of tiles (all column tiles of a few neighbouring row tiles): the W
// slabs, and the X rows shared between taps and column tiles, are then served by that XCD's L2.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstdlib>
#include <type_traits>
#include <atomic>

#include "dsattn.h"
#include "plan.h"

namespace dsattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;       // contraction depth per stage (bf16 elements)
constexpr int kRow = 128;     // bytes of one LDS row: the 64 channels of a stage = one cache line
constexpr int kSlots = 2;     // LDS ring: one stage in use, one on its way
constexpr int kXcds = 8;

// One row of the bf16 epilogue's staging area: the 64-byte pieces of NJ column blocks, padded.
__host__ __device__ constexpr int stage_row_bytes(int NJ) { return 64 * NJ + 8; }

constexpr int kMaxGroups = 4;  // weight sets applied to the same input in one launch

struct ConvArgs {
    const void *X;
    const void *W[kMaxGroups];     // per group: [taps][c_out][c_in]
    const float *bias[kMaxGroups]; // per group: [c_out] or null
    void *Y[kMaxGroups];           // per group: [M][c_out]
    int32_t groups;
    int64_t M;                 // rows = F * P
    int32_t P, Cin, Cout, n;
    int32_t KC;                // stages per tap = ceil(c_in / 64)
    int32_t KS;                // stages in all = taps * KC
    int32_t tiles_m, tiles_n;  // row tiles, column tiles per group
    int32_t tiles;             // all tiles = groups x row tiles x column tiles
    int32_t per_xcd;           // ceil(tiles / 8)
    int32_t w_bytes;           // taps * c_out * c_in * 2
};

// LDS layout: ring slot 0, a gap, ring slot 1, the bias slab.  The bf16 epilogue stages every
// wavefront's (32 rows) x (32 NJ channels) block in the slot the tile's last stage has just left
// (the other one already holds the next tile's first stage) and may spill into the gap: from
// slot 0 forwards, from slot 1 backwards.  The gap is what the staging area needs beyond one slot.
__host__ __device__ constexpr int stage_gap(int BUF, int NJ, int NW)
{
    const int need = NW * 32 * stage_row_bytes(NJ) - BUF;
    return need > 0 ? (need + 127) / 128 * 128 : 0;
}

// A wavefront's part of the tile is (32 MI) x (32 NJ); WVM x WVN = 8 wavefronts per workgroup,
// two per SIMD with 256 registers each (the hardware fills one wavefront's stalls with the
// other's matrix instructions).
//
// The workgroups are persistent: at most one per compute unit is launched, and each walks its
// share of the tiles.  The stages of successive tiles form one stream: while a tile's last
// stage is multiplied out the first stage of the workgroup's next tile is already on its way
// into the other ring slot, so only the first tile of a workgroup waits for a cold first stage,
// and no workgroup is torn down and set up between tiles.
template <int MI, int NJ, int WVM, int WVN, bool OUT_F32>
__global__ __launch_bounds__(64 * WVM * WVN, WVM * WVN / 4) void tconv_mfma_kernel(const ConvArgs a)
{
    constexpr int NW = WVM * WVN;
    constexpr int BM = 32 * MI * WVM, BN = 32 * NJ * WVN;
    constexpr int GA = BM / 8 / NW, GB = BN / 8 / NW;  // 8-row groups (one load instruction) per wavefront
    static_assert(GA * 8 * NW == BM && GB * 8 * NW == BN, "the wavefronts share the loads evenly");
    constexpr int ABYTES = BM * kRow, BUF = (BM + BN) * kRow;  // one ring slot
    constexpr int SLOT = BUF + stage_gap(BUF, NJ, NW);         // distance between the two slots
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // workgroup -> tiles: XCD x (= blockIdx % 8) owns tiles [x * per_xcd, (x + 1) * per_xcd); its
    // gridDim / 8 workgroups take them in turn, so the tiles in flight on an XCD at any time are
    // neighbours.  Tiles are numbered group outermost, then row tile, column tile fastest: the
    // tiles in flight on an XCD are all column tiles of a few neighbouring row tiles of one
    // group, about as many X slabs as W slabs (with the groups side by side they would be 2 row
    // tiles against 3 x 5 column tiles and fetch W three times as often: measured 15 GB instead
    // of 6 GB from HBM).
    const int xcd = (int)(blockIdx.x % kXcds);
    const int nper = (int)(gridDim.x / kXcds);  // workgroups per XCD
    const int t_end = min((xcd + 1) * a.per_xcd, a.tiles);
    int tile_c = xcd * a.per_xcd + (int)(blockIdx.x / kXcds);  // the tile being multiplied out
    if (tile_c >= t_end) return;  // whole workgroup: no barrier has been reached yet
    const int tiles_grp = a.tiles_m * a.tiles_n;
    auto decode = [&](int tile, int &grp, int64_t &m0, int &n0) __attribute__((always_inline)) {
        grp = tile / tiles_grp;
        const int rem = tile - grp * tiles_grp;
        const int mt = rem / a.tiles_n, nt = rem - mt * a.tiles_n;
        m0 = (int64_t)mt * BM;
        n0 = nt * BN;
    };

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wv / WVN, wn = wv - wm * WVN;

    // Global -> LDS without passing through registers: one buffer_load ... lds instruction moves
    // 8 rows x 128 B (whole cache lines: half lines cost the memory pipeline the same cycles);
    // lane l lands at LDS position l (16 B each) of the instruction's 1 KB block, i.e. row l / 8,
    // position l % 8, and fetches chunk (l % 8) ^ (l / 8) of that row: position s of row r holds
    // chunk s ^ (r % 8), which spreads a column of chunks over all banks.
    // Rows outside the video (frames before the first or after the last one) must read as
    // zeros, and do without any test: the X buffer descriptor starts at the first row the tile
    // can touch and ends with X, byte offsets are 32-bit, so a row before the video gives a
    // negative offset (huge as unsigned) and a row after it an offset past the extent, and the
    // hardware delivers zeros for both.  Channels past c_in (last block of a tap) are zeroed the
    // same way, by replacing the lane's offset.  W rows past c_out need nothing: whatever they
    // multiply into belongs to output channels that are never stored.
    const int lr = lane >> 3;
    const int lc = (lane & 7) ^ lr;
    const int rowbytes = a.Cin * 2;
    constexpr uint32_t kOob = 0xfffffff0u;
    int xoff[GA], woff[GB];  // byte offset of this lane's row and chunk within the tile's rows
    // (the empty asm keeps each offset in a register: recomputing it inside the loop would put a
    // multiply and several adds between the matrix instructions, per load)
#pragma unroll
    for (int l = 0; l < GA; ++l) {
        xoff[l] = (wv * (8 * GA) + lr + 8 * l) * rowbytes + lc * 16;
        asm volatile("" : "+v"(xoff[l]));
    }
#pragma unroll
    for (int l = 0; l < GB; ++l) {
        woff[l] = (wv * (8 * GB) + lr + 8 * l) * rowbytes + lc * 16;
        asm volatile("" : "+v"(woff[l]));
    }

    // ---- the load side: the tile whose stages are being fetched (it runs ahead of the tile being
    // multiplied out by up to two stages), its descriptors, and the per-stage load state
    int ld_tile = tile_c - nper;  // ld_open() advances before use
    bool ld_has = false;          // there is such a tile
    int ld_n0 = 0;
    int64_t ld_m0 = 0, ld_rb = 0;
    __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void *)a.X, 0, 0, 0x00020000);
    __amdgpu_buffer_rsrc_t wres = xres;
    const int taps = 2 * a.n + 1;
    int su_kc = 0, su_t = 0, su_ks = a.KS;  // channel block, tap and stage number within the load tile
    int ld_gs = 0;                          // stages set up so far: the ring slot is ld_gs % 2
    auto ld_open = [&]() __attribute__((always_inline)) {
        ld_tile += nper;
        ld_has = ld_tile < t_end;
        int grp = 0;
        decode(ld_has ? ld_tile : tile_c, grp, ld_m0, ld_n0);
        ld_rb = max((int64_t)0, ld_m0 - (int64_t)a.n * a.P);  // first row the tile can touch
        xres = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((const __bf16 *)a.X + ld_rb * a.Cin), 0,
            (int)min((a.M - ld_rb) * a.Cin * 2, (int64_t)0x7fffffff), 0x00020000);
        wres = __builtin_amdgcn_make_buffer_rsrc((void *)a.W[grp], 0, (int)a.w_bytes, 0x00020000);
        su_kc = su_t = su_ks = 0;
    };
    uint32_t ld_xstep = 0, ld_wstep = 0;
    bool ld_live = false;  // this lane's channels exist (and the stage does)
    unsigned char *ld_as = smem, *ld_bs = smem;
    // Sets up the next stage of the stream.  Stage number within a tile = channel block * taps +
    // tap: the taps of one channel block follow each other, so that the X lines they share (the
    // same rows, shifted by P per tap) are still in L2; both are counted along instead of being
    // divided out (a scalar division is some forty instructions, and they would sit between two
    // matrix instructions).  Past the workgroup's last tile every lane of the loads is an
    // out-of-range one: no traffic, the same number of loads in flight, and no branch inside the
    // multiply schedule.
    auto stage_setup = [&]() __attribute__((always_inline)) {
        if (su_ks == a.KS) ld_open();
        const int kc = su_kc, t = su_t;
        ++su_ks;
        if (++su_t == taps) {
            su_t = 0;
            ++su_kc;
        }
        ld_live = ld_has && kc * kBK + lc * 8 < a.Cin;  // c_in % 8 == 0: a chunk is all in or out
        const int64_t mshift = ld_m0 + (int64_t)(t - a.n) * a.P;  // video row of tile row 0 at this tap
        ld_xstep = (uint32_t)((int)(mshift - ld_rb) * rowbytes + kc * (kBK * 2));
        ld_wstep = (uint32_t)((t * a.Cout + ld_n0) * rowbytes + kc * (kBK * 2));
        const int slot = ld_gs & (kSlots - 1);
        ++ld_gs;
        ld_as = smem + slot * SLOT + wv * (GA * 1024);
        ld_bs = smem + slot * SLOT + ABYTES + wv * (GB * 1024);
    };
    constexpr int NL = GA + GB;  // loads per wavefront and stage
    auto issue_one = [&](int l) __attribute__((always_inline)) {
        if (l < GA)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                xres, (__attribute__((address_space(3))) void *)(ld_as + l * 1024), 16,
                ld_live ? (uint32_t)xoff[l] + ld_xstep : kOob, 0, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                wres, (__attribute__((address_space(3))) void *)(ld_bs + (l - GA) * 1024), 16,
                ld_live ? (uint32_t)woff[l - GA] + ld_wstep : kOob, 0, 0, 0);
    };

    // The wavefront's (32 MI) x (32 NJ) part is MB x NB blocks of 16 x 16, one
    // v_mfma_f32_16x16x32_bf16 accumulator each (this shape sustains about a tenth more flops
    // than 32x32x16 under the chip's power limit, measured with random operands): W rows are the
    // A operand, X rows the B operand, so that a lane ends up with 4 consecutive channels
    // (4 (lane / 16) + e of the block) of one row (lane % 16) of Y.
    constexpr int MB = 2 * MI, NB = 2 * NJ;
    constexpr int HB = MB / 2;  // X blocks of one half of a sub-step
    f32x4 acc[MB][NB];
    auto clear_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    clear_acc();

    // operand addresses: MFMA row/column lane & 15 (row % 8 = lane % 8), contraction group
    // lane >> 4; sub-step kk (32 channels) needs chunk 4 kk + (lane >> 4), which sits at position
    // chunk ^ (row % 8)
    constexpr int NKK = kBK / 32;
    static_assert(NKK == 2, "a stage is two sub-steps of 32 channels");
    int koff[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) koff[kk] = (((4 * kk) | (lane >> 4)) ^ (lane & 7)) * 16;
    const int abase = (wm * 32 * MI + (lane & 15)) * kRow;
    const int bbase = ABYTES + (wn * 32 * NJ + (lane & 15)) * kRow;

    // Operand fragments: one set of registers, refilled in place.  A sub-step's multiplies run
    // in two halves: first the X blocks [0, HB) against every W block, then the X blocks
    // [HB, MB).  The first half's X fragments are dead when the second half begins, and W
    // fragment j is dead after the second half's multiplies of column j: both are overwritten
    // with the next sub-step's values right then, under the remaining multiplies (the second
    // half's own X fragments arrive during the first half).  Double-buffered fragments of a
    // 32-channel sub-step would not fit beside the accumulators.  The loop is scheduled by hand
    // (sched_barrier pins the order): LDS reads and the issue of the next stage's loads sit
    // between the matrix instructions.
    bf16x8 af[MB], bfr[NB];
    constexpr int NMH = HB * NB;  // multiplies of one half
    // The loads of the next stage may start as soon as the barrier has freed the other slot and
    // must have landed by the next barrier; they are spread over the first kSpread multiplies
    // after the barrier (three of the four halves between two barriers), so that the memory
    // pipeline's queue never fills (a wavefront that cannot issue a load cannot issue multiplies
    // either), and the last one still has the fourth half to land.
    constexpr int TAIL = NMH;  // multiplies of a stage's last half, which follow the barrier
    constexpr int kSpread = 3 * NMH;
    auto read_a = [&](const unsigned char *base, int kk, int i) __attribute__((always_inline)) {
        af[i] = *(const bf16x8 *)(base + abase + i * (16 * kRow) + koff[kk]);
    };
    auto read_b = [&](const unsigned char *base, int kk, int j) __attribute__((always_inline)) {
        bfr[j] = *(const bf16x8 *)(base + bbase + j * (16 * kRow) + koff[kk]);
    };
    // g0 is the number of multiplies since the barrier at the half's first multiply: load q goes
    // before the multiply that is number floor(q kSpread / NL) since the barrier (when do_loads)
    auto loads_at = [&](int g, bool do_loads) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < NL; ++q)
            if (do_loads && (q * kSpread) / NL == g) {
                issue_one(q);
                __builtin_amdgcn_sched_barrier(0);
            }
    };
    // first half of sub-step kk of the slot at `base`: X blocks [0, HB); fetches the second
    // half's X fragments
    auto half1 = [&](const unsigned char *base, int kk, int g0) __attribute__((always_inline)) {
#pragma unroll
        for (int m = 0; m < NMH; ++m) {
            loads_at(g0 + m, true);
#pragma unroll
            for (int r = 0; r < HB; ++r)
                if ((r * (NMH / 2)) / HB == m) {
                    read_a(base, kk, HB + r);
                    __builtin_amdgcn_sched_barrier(0);
                }
            const int j = m / HB, i = m - j * HB;
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // second half: X blocks [HB, MB); fetches the first-half X fragments and, column by column,
    // the W fragments of the next sub-step (sub-step nkk of the slot at `nbase`)
    auto half2 = [&](const unsigned char *nbase, int nkk, int g0, bool do_loads)
                     __attribute__((always_inline)) {
#pragma unroll
        for (int m = 0; m < NMH; ++m) {
            loads_at(g0 + m, do_loads);
            const int j = m / HB, i = m - j * HB;
            if (i == 0 && j > 0) {
                read_b(nbase, nkk, j - 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (i == HB - 1 && j < HB) {  // one X fragment per column, behind the column's first multiplies
                read_a(nbase, nkk, j);
                __builtin_amdgcn_sched_barrier(0);
            }
            acc[HB + i][j] =
                __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[j], af[HB + i], acc[HB + i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        read_b(nbase, nkk, NB - 1);
        __builtin_amdgcn_sched_barrier(0);
    };
    static_assert(HB <= NB, "the first-half X fragments are fetched one per column");
    // the loads of the stage just set up that go before the first multiplies after a barrier
    auto issue_tail_loads = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < NL; ++q)
            if ((q * kSpread) / NL < TAIL) issue_one(q);
    };

    // LDS behind the two ring slots: the bias of each wavefront's 32 NJ channels
    constexpr int kBiasOff = SLOT + BUF;
    float *bl = (float *)(smem + kBiasOff) + wv * (32 * NJ);
    constexpr int NBR = (32 * NJ + 63) / 64;  // bias values a lane carries from a tile's start to its end

    // ---- start of the stream: the first tile's first stage landed, the first loads of its
    // second stage issued as the loop's tail would have.  (Bare barriers: the wait before them is
    // the only ordering needed.)
    stage_setup();
#pragma unroll
    for (int l = 0; l < NL; ++l) issue_one(l);
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    stage_setup();
    issue_tail_loads();
#pragma unroll
    for (int i = 0; i < HB; ++i) read_a(smem, 0, i);
#pragma unroll
    for (int j = 0; j < NB; ++j) read_b(smem, 0, j);

    int cs = 0;  // stages multiplied out so far: the current ring slot is cs % 2
    for (;;) {
        int grp;
        int64_t m0;
        int n0;
        decode(tile_c, grp, m0, n0);
        const float *gbias = a.bias[grp];
        void *gY = a.Y[grp];
        const int cbase = n0 + wn * 32 * NJ;      // first channel of this wavefront's part
        const int64_t mrow0 = m0 + wm * 32 * MI;  // first row of this wavefront's part
        // the bias of this wavefront's channels is fetched now and put into LDS before the
        // epilogue: the stores of the epilogue then wait for no global load
        float breg[NBR];
#pragma unroll
        for (int u = 0; u < NBR; ++u) {
            const int c = lane + 64 * u;
            breg[u] = (gbias && c < 32 * NJ && cbase + c < a.Cout) ? gbias[cbase + c] : 0.f;
        }

        for (int ks = 0; ks < a.KS; ++ks, ++cs) {
            const unsigned char *bufc = smem + (cs & 1) * SLOT;
            const unsigned char *bufn = smem + ((cs + 1) & 1) * SLOT;
            half1(bufc, 0, TAIL);
            half2(bufc, 1, TAIL + NMH, true);
            // last sub-step: its first half, then the barrier (this wavefront's loads of the
            // next stage have landed; after the barrier everybody's have, and every wavefront
            // has left the current slot), then its second half with the first fragments of the
            // next stage and the first loads of the stage after it in between.  The addresses of
            // the stage after next are worked out before the barrier, under the multiplies: every
            // load of the next stage has been issued by now (see kSpread).  After the
            // workgroup's last stage those fragments are never used: the reads stay in bounds,
            // and keeping them unconditional keeps the multiplies out of divergent control flow.
            stage_setup();
            half1(bufc, 1, TAIL + 2 * NMH);
            __builtin_amdgcn_s_waitcnt(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // After a tile's last stage the slot just left is the epilogue's staging area, so the
            // loads that would go into it wait until the epilogue is through (a scalar branch
            // around each of these few loads; two copies of the multiplies, one with and one
            // without them, made the compiler spill accumulators).
            half2(bufn, 0, 0, ks + 1 < a.KS);
        }
        // The tile's last barrier has retired every load into, and every operand read of, the slot
        // of its last stage, (cs - 1) % 2; the other slot holds the next tile's first stage.

        // ---- epilogue: accumulator element e of lane l is output channel 4 (l / 16) + e and row
        // l % 16 of its 16 x 16 block: four consecutive channels per lane.
        // (the lane index is made opaque once per tile: every address below depends on it, and
        // what the compiler could otherwise compute ahead of the tile loop and keep alive through
        // it costs the main loop its registers)
        int le = lane;
        asm volatile("" : "+v"(le));
#pragma unroll
        for (int u = 0; u < NBR; ++u)
            if (le + 64 * u < 32 * NJ) bl[le + 64 * u] = breg[u];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        bool staged = false;
        if constexpr (!OUT_F32) {
            if ((a.Cout & 7) == 0) {
                staged = true;
                // bf16 rows made of whole 16-byte pieces: the wavefront's (32 MI) x (32 NJ) part
                // goes through its own region of the staging area, one 32-row block at a time, and
                // leaves as full rows: each store instruction writes 64 NJ contiguous bytes per
                // row.  Rows are padded by 8 bytes so that the 8-byte writes of 16 consecutive rows
                // spread over the banks.
                constexpr int SR = stage_row_bytes(NJ);
                constexpr int CPR = 4 * NJ;  // 16-byte pieces per row
                unsigned char *stg = smem + (((cs - 1) & 1) ? SLOT + BUF - NW * 32 * SR : 0) + wv * (32 * SR);
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    // (without a bias the additions are left out: they are a third of this phase's
                    // vector instructions, and the phase is bound by them)
                    auto fill = [&](auto with_bias) __attribute__((always_inline)) {
#pragma unroll
                        for (int j = 0; j < NB; ++j) {
                            const int cl = 16 * j + 4 * (le >> 4);  // channel within the part
                            f32x4 b = {0.f, 0.f, 0.f, 0.f};
                            if constexpr (decltype(with_bias)::value) b = *(const f32x4 *)(bl + cl);
#pragma unroll
                            for (int h = 0; h < 2; ++h) {  // the two 16-row blocks of the pass
                                bf16x4 yb;
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    float y = acc[2 * i + h][j][e];
                                    if constexpr (decltype(with_bias)::value) y += b[e];
                                    yb[e] = (__bf16)y;
                                }
                                *(bf16x4 *)(stg + (16 * h + (le & 15)) * SR + cl * 2) = yb;
                            }
                        }
                    };
                    if (gbias)
                        fill(std::true_type{});
                    else
                        fill(std::false_type{});
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int it = 0; it < (32 * CPR + 63) / 64; ++it) {
                        const int q = le + 64 * it;
                        const int row = q / CPR, pc = q - row * CPR;
                        const int64_t m = mrow0 + 32 * i + row;
                        if (q < 32 * CPR && m < a.M && cbase + pc * 8 < a.Cout) {
                            const uint2 lo = *(const uint2 *)(stg + row * SR + pc * 16);
                            const uint2 hi = *(const uint2 *)(stg + row * SR + pc * 16 + 8);
                            *(uint4 *)((__bf16 *)gY + m * a.Cout + cbase + pc * 8) =
                                make_uint4(lo.x, lo.y, hi.x, hi.y);
                        }
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
        if (!staged) {
            // fp32 output, or bf16 rows that are not whole 16-byte pieces: straight from the registers
            const bool vec_ok = (a.Cout & 3) == 0;  // 8-byte (bf16) / 16-byte (fp32) stores stay aligned
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                    const int cl = 16 * j + 4 * (le >> 4);
                    const int co = cbase + cl;
                    const f32x4 b = *(const f32x4 *)(bl + cl);
#pragma unroll
                    for (int i = 0; i < MB; ++i) {
                        const int64_t m = mrow0 + 16 * i + (le & 15);
                        if (m >= a.M || co >= a.Cout) continue;
                        const f32x4 y = {acc[i][j][0] + b[0], acc[i][j][1] + b[1],
                                         acc[i][j][2] + b[2], acc[i][j][3] + b[3]};
                        if (vec_ok) {  // c_out % 4 == 0 and co % 4 == 0: all four channels exist
                            if constexpr (OUT_F32) {
                                *(f32x4 *)((float *)gY + m * a.Cout + co) = y;
                            } else {
                                bf16x4 yb;
#pragma unroll
                                for (int e = 0; e < 4; ++e) yb[e] = (__bf16)y[e];
                                *(bf16x4 *)((__bf16 *)gY + m * a.Cout + co) = yb;
                            }
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (co + e < a.Cout) {
                                    if constexpr (OUT_F32)
                                        ((float *)gY)[m * a.Cout + co + e] = y[e];
                                    else
                                        ((__bf16 *)gY)[m * a.Cout + co + e] = (__bf16)y[e];
                                }
                        }
                    }
                }
        }

        // ---- on to the workgroup's next tile: its first stage is in the other slot and its first
        // fragments are in registers; the loads held back above go out once every wavefront has
        // left the staging area
        tile_c += nper;
        if (tile_c >= t_end) break;
        clear_acc();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        issue_tail_loads();
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
    int MI, NJ, WVM, WVN;  // tile = (32 MI WVM) x (32 NJ WVN), WVM x WVN wavefronts
    const void *fn[2];     // bf16 / fp32 output
    int bm() const { return 32 * MI * WVM; }
    int bn() const { return 32 * NJ * WVN; }
    int waves() const { return WVM * WVN; }
};
#define DSATTN_CONV_VARIANT(MI, NJ, WVM, WVN)                                    \
    {MI, NJ, WVM, WVN,                                                           \
     {(const void *)&tconv_mfma_kernel<MI, NJ, WVM, WVN, false>,                 \
      (const void *)&tconv_mfma_kernel<MI, NJ, WVM, WVN, true>}}
// Eight wavefronts (two per SIMD) throughout: one wavefront per SIMD cannot keep the matrix cores
// busy with 16x16x32 instructions (measured: 1.46 against 2.4 PFLOP/s on idle data).
const ConvVariant kConvVariants[] = {
    DSATTN_CONV_VARIANT(4, 2, 2, 4),  // 256 x 256
    DSATTN_CONV_VARIANT(2, 5, 4, 2),  // 256 x 320
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
const ConvVariant *conv_pick(const dsattn_conv_desc &d, int64_t M, int groups = 1)
{
    if (d.io_dtype != DSATTN_BF16 || d.c_in % 8 != 0 || (d.flags & DSATTN_FLAG_FORCE_GENERIC))
        return nullptr;
    // the kernel addresses W, and the rows of X one tile can touch, with 32-bit byte offsets
    const int64_t taps = 2 * (int64_t)d.reach + 1;
    if (taps * d.c_out * d.c_in * 2 >= ((int64_t)1 << 31)) return nullptr;
    if ((320 + 2 * (int64_t)d.reach * d.spatial) * d.c_in * 2 >= ((int64_t)1 << 31)) return nullptr;
    // least multiplied-out area (padding of the last row and column tiles), then the larger
    // tile (fewer epilogues)
    const ConvVariant *best = nullptr;
    double best_area = 0;
    int64_t best_tiles = 0;
    for (const ConvVariant &v : kConvVariants) {
        const int64_t bm = v.bm(), bn = v.bn();
        const int64_t tm = (M + bm - 1) / bm, tn = (d.c_out + bn - 1) / bn;
        if (tm * tn * groups > 0x7fffffffLL / 2) continue;
        const double area = (double)(tm * bm) * (double)(tn * bn);
        const int64_t tiles = tm * tn;
        const bool better = !best || area < best_area || (area == best_area && tiles < best_tiles);
        if (better) {
            best = &v;
            best_area = area;
            best_tiles = tiles;
        }
    }
    return best;
}

// the two ring slots with the staging gap between them; behind them the bias of each
// wavefront's 32 NJ channels
int conv_lds_bytes(const ConvVariant &v)
{
    const int buf = (v.bm() + v.bn()) * kRow;
    return kSlots * buf + stage_gap(buf, v.NJ, v.waves()) + v.waves() * 32 * v.NJ * (int)sizeof(float);
}

// Compute units of the current device (one persistent workgroup is launched per unit at most).
int conv_compute_units(int dev)
{
    static std::atomic<int> cached[64];
    if (dev >= 0 && dev < 64) {
        const int c = cached[dev].load(std::memory_order_relaxed);
        if (c > 0) return c;
    }
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        n = 256;
    if (dev >= 0 && dev < 64) cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

// A linear layer over M rows is the one-tap case of the convolution (every row its own frame).
int linear_as_conv(const dsattn_linear_desc *l, dsattn_conv_desc &d, int64_t &M, const char *who)
{
    if (!l) return fail(DSATTN_EINVAL, "%s: null descriptor", who);
    if (l->rows < 1 || l->rows > 0x7fffffffLL || l->c_in < 1 || l->c_out < 1)
        return fail(DSATTN_EINVAL, "%s: sizes must be positive (rows at most 2^31 - 1)", who);
    if (l->n_out < 1 || l->n_out > kMaxGroups)
        return fail(DSATTN_EINVAL, "%s: n_out %d outside [1, %d]", who, l->n_out, kMaxGroups);
    d = dsattn_conv_desc{};
    d.clip_len = 1;
    d.n_clips = (int32_t)l->rows;
    d.spatial = 1;
    d.c_in = l->c_in;
    d.c_out = l->c_out;
    d.reach = 0;
    d.io_dtype = l->io_dtype;
    d.out_dtype = l->out_dtype;
    d.flags = l->flags;
    M = l->rows;
    return conv_validate(&d, who);
}

// Launches the implicit-GEMM kernel (when `v`) or the vector kernel for `groups` weight sets
// applied to the same X.  `d` describes one set; M = rows of X and of every Y.
hipError_t conv_launch(const dsattn_conv_desc &d, int64_t M, const ConvVariant *v, int groups,
                       const void *X, const void *const *W, const float *const *bias,
                       void *const *Y, hipStream_t st)
{
    hipError_t e = hipSuccess;
    if (v) {
        const void *fn = v->fn[d.out_dtype == DSATTN_F32 ? 1 : 0];
        const int lds = conv_lds_bytes(*v);
        // The default cap on dynamic LDS is 64 KB: raised once per kernel and device.  The launch
        // path only reads a flag (no lock); two threads that both find it clear both set the
        // attribute, which is harmless.
        static std::atomic<uint64_t> prepared[sizeof(kConvVariants) / sizeof(kConvVariants[0])][2];
        int dev = 0;
        e = hipGetDevice(&dev);  // a thread-local read in the runtime
        if (e != hipSuccess) return e;
        std::atomic<uint64_t> *mask =
            dev < 64 ? &prepared[v - kConvVariants][d.out_dtype == DSATTN_F32 ? 1 : 0] : nullptr;
        if (!mask || !(mask->load(std::memory_order_acquire) >> dev & 1)) {
            e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return e;
            if (mask) mask->fetch_or((uint64_t)1 << dev, std::memory_order_release);
        }
        ConvArgs a;
        a.X = X;
        for (int g = 0; g < kMaxGroups; ++g) {
            a.W[g] = g < groups ? W[g] : nullptr;
            a.bias[g] = g < groups && bias ? bias[g] : nullptr;
            a.Y[g] = g < groups ? Y[g] : nullptr;
        }
        a.groups = groups;
        a.M = M;
        a.P = d.spatial;
        a.Cin = d.c_in;
        a.Cout = d.c_out;
        a.n = d.reach;
        a.KC = (d.c_in + kBK - 1) / kBK;
        a.KS = (2 * d.reach + 1) * a.KC;
        const int64_t bm = v->bm(), bn = v->bn();
        a.tiles_n = (int32_t)((d.c_out + bn - 1) / bn);
        a.tiles_m = (int32_t)((M + bm - 1) / bm);
        a.tiles = a.tiles_m * a.tiles_n * groups;
        a.per_xcd = (a.tiles + kXcds - 1) / kXcds;
        a.w_bytes = (int32_t)((2 * (int64_t)d.reach + 1) * d.c_out * d.c_in * 2);
        void *params[] = {&a};
        // persistent workgroups: one per compute unit at most, the same number on every XCD
        const int per_xcd_wg = std::min(a.per_xcd, (conv_compute_units(dev) + kXcds - 1) / kXcds);
        return hipLaunchKernel(fn, dim3((unsigned)(per_xcd_wg * kXcds)), dim3(64 * v->waves()), params,
                               (size_t)lds, st);
    }
    const int64_t total = M * d.c_out;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    for (int g = 0; g < groups; ++g) {
        const float *b = bias ? bias[g] : nullptr;
        if (d.io_dtype == DSATTN_F32)
            hipLaunchKernelGGL((tconv_generic_kernel<float, float>), grid, block, 0, st,
                               (const float *)X, (const float *)W[g], b, (float *)Y[g], M, d.spatial,
                               d.c_in, d.c_out, d.reach);
        else if (d.out_dtype == DSATTN_F32)
            hipLaunchKernelGGL((tconv_generic_kernel<__bf16, float>), grid, block, 0, st,
                               (const __bf16 *)X, (const __bf16 *)W[g], b, (float *)Y[g], M,
                               d.spatial, d.c_in, d.c_out, d.reach);
        else
            hipLaunchKernelGGL((tconv_generic_kernel<__bf16, __bf16>), grid, block, 0, st,
                               (const __bf16 *)X, (const __bf16 *)W[g], b, (__bf16 *)Y[g], M,
                               d.spatial, d.c_in, d.c_out, d.reach);
    }
    return hipGetLastError();
}

// Y must not overlap X: an output row is written while other workgroups still read X
bool ranges_overlap(const void *a, int64_t abytes, const void *b, int64_t bbytes)
{
    const uintptr_t a0 = (uintptr_t)a, a1 = a0 + (uintptr_t)abytes;
    const uintptr_t b0 = (uintptr_t)b, b1 = b0 + (uintptr_t)bbytes;
    return a0 < b1 && b0 < a1;
}

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
        const int64_t bm = v->bm(), bn = v->bn();
        const int64_t tiles = ((M + bm - 1) / bm) * ((d.c_out + bn - 1) / bn);
        info->kernel = 1;
        info->tile_m = (int32_t)bm;
        info->tile_n = (int32_t)bn;
        info->tile_k = kBK;
        info->n_blocks = (int32_t)(((tiles + kXcds - 1) / kXcds) * kXcds);
        info->block_threads = 64 * v->waves();
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
    if (ranges_overlap(X, M * d.c_in * in_b, Y, M * d.c_out * out_b))
        return fail(DSATTN_EINVAL, "dsattn_temporal_conv: Y overlaps X");
    const ConvVariant *v = conv_pick(d, M);
    if (!v && (M * d.c_out + 255) / 256 > 0x7fffffffLL)
        return fail(DSATTN_EUNSUPPORTED, "dsattn_temporal_conv: too large for the generic kernel");
    const hipError_t e = conv_launch(d, M, v, 1, X, &W, &bias, &Y, (hipStream_t)stream);
    if (e != hipSuccess) return fail(DSATTN_EHIP, "dsattn_temporal_conv: %s", hipGetErrorString(e));
    return DSATTN_OK;
}

int dsattn_linear_info(const dsattn_linear_desc *desc, dsattn_conv_info *info)
{
    dsattn_conv_desc d;
    int64_t M = 0;
    const int rc = linear_as_conv(desc, d, M, "dsattn_linear_info");
    if (rc != DSATTN_OK) return rc;
    if (!info) return fail(DSATTN_EINVAL, "dsattn_linear_info: null output");
    *info = dsattn_conv_info{};
    const ConvVariant *v = conv_pick(d, M, desc->n_out);
    info->block_threads = 256;
    if (v) {
        info->block_threads = 64 * v->waves();
        const int64_t bm = v->bm(), bn = v->bn();
        const int64_t tiles = ((M + bm - 1) / bm) * ((d.c_out + bn - 1) / bn) * desc->n_out;
        info->kernel = 1;
        info->tile_m = (int32_t)bm;
        info->tile_n = (int32_t)bn;
        info->tile_k = kBK;
        info->n_blocks = (int32_t)(((tiles + kXcds - 1) / kXcds) * kXcds);
        info->lds_bytes = conv_lds_bytes(*v);
    } else {
        info->tile_n = 1;
        info->tile_k = 1;
        info->n_blocks = (int32_t)std::min<int64_t>((M * d.c_out + 255) / 256, 0x7fffffff);
    }
    const int64_t in_b = d.io_dtype == DSATTN_BF16 ? 2 : 4, out_b = d.out_dtype == DSATTN_BF16 ? 2 : 4;
    info->useful_flops = 2 * M * d.c_in * d.c_out * desc->n_out;
    info->algorithmic_bytes =
        M * d.c_in * in_b + (int64_t)desc->n_out * (d.c_out * d.c_in * in_b + M * d.c_out * out_b);
    return DSATTN_OK;
}

int dsattn_linear(const dsattn_linear_desc *desc, const void *X, const void *const *W,
                  const float *const *bias, void *const *Y, void *stream)
{
    dsattn_conv_desc d;
    int64_t M = 0;
    const int rc = linear_as_conv(desc, d, M, "dsattn_linear");
    if (rc != DSATTN_OK) return rc;
    if (!X || !W || !Y) return fail(DSATTN_EINVAL, "dsattn_linear: null pointer");
    const int64_t in_b = d.io_dtype == DSATTN_BF16 ? 2 : 4, out_b = d.out_dtype == DSATTN_BF16 ? 2 : 4;
    if ((uintptr_t)X & 15u) return fail(DSATTN_EINVAL, "dsattn_linear: X must be 16-byte aligned");
    for (int g = 0; g < desc->n_out; ++g) {
        if (!W[g] || !Y[g]) return fail(DSATTN_EINVAL, "dsattn_linear: null pointer in set %d", g);
        if (((uintptr_t)W[g] | (uintptr_t)Y[g]) & 15u)
            return fail(DSATTN_EINVAL, "dsattn_linear: pointers must be 16-byte aligned");
        if (bias && bias[g] && ((uintptr_t)bias[g] & 3u))
            return fail(DSATTN_EINVAL, "dsattn_linear: bias must be 4-byte aligned");
        if (ranges_overlap(X, M * d.c_in * in_b, Y[g], M * d.c_out * out_b))
            return fail(DSATTN_EINVAL, "dsattn_linear: output %d overlaps X", g);
        for (int h = 0; h < g; ++h)
            if (ranges_overlap(Y[h], M * d.c_out * out_b, Y[g], M * d.c_out * out_b))
                return fail(DSATTN_EINVAL, "dsattn_linear: outputs %d and %d overlap", h, g);
    }
    const ConvVariant *v = conv_pick(d, M, desc->n_out);
    if (!v && (M * d.c_out + 255) / 256 > 0x7fffffffLL)
        return fail(DSATTN_EUNSUPPORTED, "dsattn_linear: too large for the generic kernel");
    const hipError_t e = conv_launch(d, M, v, desc->n_out, X, W, bias, Y, (hipStream_t)stream);
    if (e != hipSuccess) return fail(DSATTN_EHIP, "dsattn_linear: %s", hipGetErrorString(e));
    return DSATTN_OK;
}

}  // extern "C"
