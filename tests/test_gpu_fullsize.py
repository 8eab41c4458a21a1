"""Parity at the full sizes of the five workloads, in the launch configuration bench.py times:
the planner's own choices, inputs generated on the device, and the oracle evaluated on a sample
of spatial positions (rows are independent, so every sampled output is exact)."""
import numpy as np
import pytest
import torch

import parity_util as U
from oracle import oracle
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sample_positions(P, n, info, heads):
    """At least n positions spread over the level, plus the ones where the launch has its seams:
    the first and last position of the level (the first and last row group of every chunk: the
    oracle covers all frames, hence every chunk, of a sampled position) and the positions on both
    sides of workgroup boundaries (a workgroup spans block_threads / 64 wavefronts of
    heads_per_wave heads each)."""
    pos = set(((np.arange(n) * P) // n).tolist())
    pos.update({0, P - 1, P // 2})
    if info["kernel"] == 1:
        pos_per_wg = max(1, (info["block_threads"] // 64) * info["heads_per_wave"] // heads)
        n_wg = max(1, P // pos_per_wg)
        for j in sorted({1, 2, n_wg // 3, n_wg // 2, n_wg - 1}):
            if 0 < j < n_wg:
                pos.update({j * pos_per_wg - 1, j * pos_per_wg})
    return sorted(p for p in pos if 0 <= p < P)


def run_level(wl, lv, out_dtype, n_pos):
    g = synth.global_idx_for(wl)
    print(f"[case] full size {wl.name} {lv.name} {lv.spatial} {lv.heads}x{lv.head_dim} "
          f"out={out_dtype}", flush=True)
    q, k, v = synth.make_qkv(wl, lv, device=DEV)
    o, info = U.library_forward(q, k, v, wl.clip_len, wl.n_clips, wl.local_ctx, lv.heads, g,
                                out_dtype=out_dtype)
    pos = sample_positions(lv.P, n_pos, info, lv.heads)
    assert len(pos) >= min(n_pos, lv.P)
    ref = U.oracle_forward(q, k, v, wl.clip_len, wl.n_clips, wl.local_ctx, lv.heads, g,
                           positions=pos)
    mx = U.assert_parity(o, ref, out_dtype, positions=pos, what=f"{wl.name}/{lv.name}")
    # nothing outside the sample is left unwritten
    assert torch.isfinite(o.float()).all()
    del q, k, v, o
    torch.cuda.empty_cache()
    return info, mx


@pytest.mark.parametrize("name,n_pos", [("C1", 32), ("C2", 32), ("C3", 160)])
def test_single_level_workloads_full_size(name, n_pos):
    # the headline level is compared on every one of its 160 positions
    wl = synth.WORKLOADS[name]
    info, _ = run_level(wl, wl.levels[0], "bf16", n_pos)
    assert info["kernel"] == 1


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_single_level_workloads_full_size_fp32_output_strict(name):
    # bf16 inputs, fp32 accumulation, fp32 output: the 1e-2 bar holds outright
    wl = synth.WORKLOADS[name]
    info, mx = run_level(wl, wl.levels[0], "f32", 32)
    assert info["kernel"] == 1 and mx <= 1e-2


@pytest.mark.parametrize("level", [0, 1, 2, 3])
def test_c4_levels_full_size(level):
    wl = synth.WORKLOADS["C4"]
    info, _ = run_level(wl, wl.levels[level], "bf16", 32)
    assert info["kernel"] == 1 and info["global_tiles"] == 4


@pytest.mark.parametrize("level", [0, 1, 2, 3])
def test_c4_levels_full_size_fp32_output_strict(level):
    wl = synth.WORKLOADS["C4"]
    info, mx = run_level(wl, wl.levels[level], "f32", 32)
    assert info["kernel"] == 1 and info["global_tiles"] == 4 and mx <= 1e-2


def test_paper_sized_clips_full_size():
    # the headline tensors cut into the paper's eight 288-frame clips, 8 + 8 context frames,
    # window radius 8, 16 global frames: the launch bench.py times as C3_8x288_w8_r8_G16
    wl = synth.WORKLOADS["C3"]
    lv = wl.levels[0]
    g = synth.stride_global_idx(wl.F, 16)
    print("[case] full size 8 x 288 frames w=8 r=8 G=16 on the C3 tensors", flush=True)
    q, k, v = synth.make_qkv(wl, lv, device=DEV)
    for od in ("bf16", "f32"):
        o, info = U.library_forward(q, k, v, 288, 8, 8, lv.heads, g, out_dtype=od, window=8)
        assert info["kernel"] == 1 and info["ring_reach"] == 8
        pos = sample_positions(lv.P, 32, info, lv.heads)
        ref = U.oracle_forward(q, k, v, 288, 8, 8, lv.heads, g, positions=pos, window=8)
        U.assert_parity(o, ref, od, positions=pos, what=f"8x288 {od}")


def test_c1_gather_full_size_bit_exact():
    wl = synth.WORKLOADS["C1"]
    lv = wl.levels[0]
    g = synth.global_idx_for(wl)
    print("[case] full size gather C1", flush=True)
    _, k, v = synth.make_qkv(wl, lv, device=DEV)
    plan = B.dsattn_plan(wl.clip_len, wl.n_clips, wl.local_ctx, lv.P, lv.heads, lv.head_dim, g,
                         io_dtype=B.DSATTN_BF16, device=0)
    lk = B.dsattn_plan_ctx_max(plan)
    kc = torch.empty((wl.n_clips, lk, lv.P, lv.C), dtype=k.dtype, device=DEV)
    vc = torch.empty_like(kc)
    B.dsattn_gather_context(plan, k, v, kc, vc)
    torch.cuda.synchronize()
    idx, ln = oracle.ctx_indices(wl.clip_len, wl.n_clips, wl.local_ctx, g)
    for i in range(wl.n_clips):
        rows = torch.as_tensor(idx[i, :ln[i]].astype(np.int64), device=DEV)
        assert torch.equal(kc[i, :ln[i]].view(torch.int16), k.index_select(0, rows).view(torch.int16))
        assert torch.equal(vc[i, :ln[i]].view(torch.int16), v.index_select(0, rows).view(torch.int16))
        assert (kc[i, ln[i]:].view(torch.int16) == 0).all() and (vc[i, ln[i]:].view(torch.int16) == 0).all()
    plan.close()
