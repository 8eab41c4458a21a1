"""Clips longer than 16 frames on the matrix-core kernel (Section 4: a clip is F / N frames, on the
paper's eight devices about 288; Section 4.2: the local scope as a window around the query frame).
A clip is walked in query tiles of 16 frames; a tile sees the frames within the window's radius
that lie in its clip's local range.  Every case is compared with the oracle element by element."""
import numpy as np
import pytest
import torch

import parity_util as U
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(F, P, C, seed, gen="iid"):
    return tuple(synth.make_tensor(F, P, C, seed + t, gen, "bf16").to(DEV) for t in range(3))


def run(clip_len, n_clips, w, r, G, h, D, P, seed, out="f32", clips_per_task=None, gen="iid",
        scale=0.0, flags=0, expect_kernel=1, **opts):
    F = clip_len * n_clips
    g = synth.random_sorted_global_idx(F, G, seed=seed + 7).tolist() if G else []
    q, k, v = make(F, P, h * D, seed, gen)
    print(f"[case] long clips: {n_clips} x {clip_len} frames, w={w} r={r} G={G} {h}x{D} P={P} "
          f"out={out} tiles/chunk={clips_per_task} flags={flags} {opts}", flush=True)
    with U.planner_env(clips_per_task, None):
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype=out, window=r,
                                    scale=scale, flags=flags, **opts)
    assert info["kernel"] == expect_kernel, info
    ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, window=r, scale=scale,
                           dedup=bool(flags & B.DSATTN_FLAG_DEDUP_GLOBAL), **opts)
    U.assert_parity(o, ref, out, what=f"clip_len {clip_len} w={w} r={r} G={G} D={D}")
    return info, q, k, v, g, ref


@pytest.mark.parametrize("D,h", [(160, 2), (80, 4), (40, 8)])
@pytest.mark.parametrize("clip_len,n_clips", [(32, 5), (48, 3), (288, 2)])
@pytest.mark.parametrize("w,r,G", [
    (8, 8, 16),    # r = w: the paper's 8 + 8 neighbouring frames and 16 global ones
    (8, 3, 0),     # r < w, no global frames
    (4, 0, 64),    # r = 0: every query sees its own frame and the global set
    (2, 8, 16),    # r > w: the window is cut at the clip's local range
    (0, 5, 3),     # no context from the neighbouring clips at all
])
def test_window_inside_long_clips(D, h, clip_len, n_clips, w, r, G):
    info, *_ = run(clip_len, n_clips, w, r, G, h, D, 3, seed=100 + clip_len + D + w)
    assert info["ring_reach"] == min(r, clip_len - 16 + w)
    assert info["local_tiles"] == (16 + 2 * info["ring_reach"] + 15) // 16
    assert info["global_tiles"] == (0 if G == 0 else 1 if G <= 16 else 4)


@pytest.mark.parametrize("tiles_per_chunk", [1, 2, 5, 7, 36])
def test_chunks_need_not_end_at_clip_boundaries(tiles_per_chunk):
    # 3 clips of 48 frames = 9 query tiles; a chunk of 2, 5 or 7 tiles ends inside a clip
    run(48, 3, 3, 8, 16, 2, 160, 5, seed=300, clips_per_task=tiles_per_chunk)
    run(48, 3, 3, 8, 16, 2, 160, 5, seed=301, clips_per_task=tiles_per_chunk, out="bf16",
        gen="correlated")


def test_long_clips_without_a_window_where_the_clip_fits_the_ring():
    # 32-frame clips, no context frames, no window: a tile sees its whole clip (16 frames beyond
    # the tile on one side), and nothing of the neighbouring clips
    info, *_ = run(32, 4, 0, None, 16, 2, 160, 4, seed=400)
    assert info["ring_reach"] == 16 and info["local_tiles"] == 3
    # a longer reach than the ring holds runs the vector kernel
    run(32, 4, 2, None, 16, 2, 160, 2, seed=401, expect_kernel=0)
    run(288, 2, 8, 17, 0, 2, 160, 2, seed=402, expect_kernel=0)
    run(24, 4, 2, 2, 4, 2, 160, 2, seed=403, expect_kernel=0)       # not whole tiles


def test_long_clips_with_scope_biases_union_and_peaked_softmax():
    run(32, 4, 8, 6, 16, 2, 160, 3, seed=500, bias_local=0.4, bias_global=-0.9)
    run(48, 3, 8, 8, 16, 8, 40, 3, seed=501, scale=4.0 / np.sqrt(40.0))
    run(32, 4, 8, 6, 16, 2, 160, 3, seed=502, flags=B.DSATTN_FLAG_DEDUP_GLOBAL)
    run(32, 4, 4, 8, 64, 2, 160, 3, seed=503, flags=B.DSATTN_FLAG_DEDUP_GLOBAL)


def test_window_wider_than_context_is_partition_dependent_and_matches_per_partition():
    # with r <= w the result cannot depend on the clip partition; with r > w it does, and the
    # kernel follows the partition it was given
    F, P, h, D, r = 192, 2, 2, 160, 8
    q, k, v = make(F, P, h * D, 600)
    whole = U.oracle_forward(q, k, v, F, 1, 0, h, [], window=r)
    for clip_len, n_clips in ((16, 12), (32, 6), (48, 4), (96, 2)):
        o, info = U.library_forward(q, k, v, clip_len, n_clips, 8, h, [], out_dtype="f32", window=r)
        assert info["kernel"] == 1
        U.assert_parity(o, whole, "f32", what=f"partition {clip_len}")
    cut = U.oracle_forward(q, k, v, 96, 2, 2, h, [], window=r)
    assert np.abs(cut - whole).max() > 1e-2
    o, _ = U.library_forward(q, k, v, 96, 2, 2, h, [], out_dtype="f32", window=r)
    U.assert_parity(o, cut, "f32", what="r > w")


@pytest.mark.parametrize("clip_len,n_clips,w,r,G", [(32, 4, 8, 8, 16), (48, 3, 2, 8, 64),
                                                    (288, 2, 8, 8, 16)])
def test_materialised_context_of_long_clips(clip_len, n_clips, w, r, G):
    # dsattn_forward_ctx walks one clip per chunk through the clip's slab of the gathered context
    F, P, h, D = clip_len * n_clips, 3, 2, 160
    g = synth.random_sorted_global_idx(F, G, seed=5).tolist()
    q, k, v = make(F, P, h * D, 700 + clip_len)
    print(f"[case] long clips forward_ctx {n_clips} x {clip_len} w={w} r={r} G={G}", flush=True)
    plan = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, io_dtype=B.DSATTN_BF16,
                         out_dtype=B.DSATTN_F32, device=0, window=r)
    assert B.dsattn_plan_launch_info(plan)["kernel"] == 1
    lk = B.dsattn_plan_ctx_max(plan)
    kc = torch.empty((n_clips, lk, P, h * D), dtype=k.dtype, device=DEV)
    vc = torch.empty_like(kc)
    B.dsattn_gather_context(plan, k, v, kc, vc)
    o1 = torch.full((F, P, h * D), float("nan"), dtype=torch.float32, device=DEV)
    o2 = torch.full_like(o1, float("nan"))
    B.dsattn_forward(plan, q, k, v, o1)
    B.dsattn_forward_ctx(plan, q, kc, vc, o2)
    torch.cuda.synchronize()
    plan.close()
    assert torch.equal(o1, o2)
    ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, window=r)
    U.assert_parity(o2, ref, "f32", what="forward_ctx long clips")


def test_paper_sized_clips_on_a_slice_of_the_headline_tensor():
    # 8 clips of 288 frames (the paper's eight devices), 8 + 8 neighbouring frames, 16 global:
    # the headline level's row shape on a few positions
    info, *_ = run(288, 8, 8, 8, 16, 8, 160, 4, seed=800, out="bf16", gen="correlated")
    assert info["local_tiles"] == 2 and info["global_tiles"] == 1 and info["heads_per_wave"] == 1


def test_randomised_options_against_oracle():
    """Seeded sweep over the options together: clip lengths of one to four tiles, windows, both
    scope biases, the set union, up to 128 global frames with repeats, both output types, and the
    materialised-context path beside the fused one (identical bits expected)."""
    rng = np.random.default_rng(77)
    ran = {0: 0, 1: 0}
    for case in range(40):
        D = int(rng.choice([40, 80, 160, 64, 96]))
        h = int(rng.choice([1, 2, 3, 4, 8]))
        clip_len = int(rng.choice([16, 32, 48, 64]))
        n_clips = int(rng.integers(1, 5))
        F = clip_len * n_clips
        w = int(rng.integers(0, 17))
        G = int(rng.choice([0, 3, 16, 30, 64, 65, 128]))
        g = rng.integers(0, F, size=G).tolist()
        P = int(rng.integers(1, 5))
        window = None if (clip_len == 16 and rng.random() < 0.5) else int(rng.integers(0, 17))
        bl, bg = (0.0, 0.0) if rng.random() < 0.5 else (float(rng.normal()), float(rng.normal()))
        dedup = bool(rng.random() < 0.3)
        od = "f32" if rng.random() < 0.6 else "bf16"
        scale = 0.0 if rng.random() < 0.7 else float(2.5 / np.sqrt(D))
        print(f"[case] random options {case}: D={D} h={h} Fc={clip_len} N={n_clips} w={w} G={G} P={P} "
              f"window={window} biases=({bl:.2f},{bg:.2f}) dedup={dedup} out={od} scale={scale:.3f}",
              flush=True)
        q, k, v = make(F, P, h * D, 2000 + case)
        flags = B.DSATTN_FLAG_DEDUP_GLOBAL if dedup else 0
        ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, scale=scale, window=window,
                               bias_local=bl, bias_global=bg, dedup=dedup)
        plan = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, io_dtype=B.DSATTN_BF16,
                             out_dtype=U.dt_code(od), scale=scale, flags=flags, device=0,
                             bias_local=bl, bias_global=bg, window=window)
        info = B.dsattn_plan_launch_info(plan)
        ran[info["kernel"]] += 1
        o1 = torch.full((F, P, h * D), float("nan"), dtype=synth.torch_dtype(od), device=DEV)
        o2 = torch.full_like(o1, float("nan"))
        B.dsattn_forward(plan, q, k, v, o1)
        lk = B.dsattn_plan_ctx_max(plan)
        kc = torch.empty((n_clips, lk, P, h * D), dtype=k.dtype, device=DEV)
        vc = torch.empty_like(kc)
        B.dsattn_gather_context(plan, k, v, kc, vc)
        B.dsattn_forward_ctx(plan, q, kc, vc, o2)
        torch.cuda.synchronize()
        plan.close()
        U.assert_parity(o1, ref, od, what=f"random options {case} (kernel {info['kernel']})")
        assert torch.equal(o1.view(torch.int32 if od == "f32" else torch.int16),
                           o2.view(torch.int32 if od == "f32" else torch.int16)), case
    assert ran[0] >= 3 and ran[1] >= 15, ran   # the sweep reaches both kernels
