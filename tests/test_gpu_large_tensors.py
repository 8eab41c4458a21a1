"""Tensors of more than 4 GiB (and more than 2^31 elements): every kernel addresses them with
64-bit arithmetic somewhere, and none of the five workloads' tensors is large enough to show a
32-bit slip (the largest, 2,304 x 2,560 x 320 bf16, is 3.5 GiB).  Inputs are generated on the
device; the oracle runs on sampled spatial positions (every module here treats positions
independently, group normalisation aside), chosen so that the sample includes rows whose byte
offsets lie beyond 4 GiB."""
import numpy as np
import pytest
import torch

import parity_util as U
from oracle import oracle
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth
from test_tconv import check_conv

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GIB4 = 1 << 32


def f64(t):
    return t.to("cpu").to(torch.float64).numpy()


def test_attention_on_tensors_beyond_4_gib():
    # the largest level's shape with twice the frames: 4,608 x 2,560 x 320 bf16 = 7.0 GiB per tensor
    clip_len, n_clips, w, P, h, D, G = 16, 288, 4, 2560, 8, 40, 64
    F, C = clip_len * n_clips, h * D
    assert F * P * C * 2 > GIB4 and F * P * C > (1 << 31)
    g = synth.random_sorted_global_idx(F, G, seed=11).tolist()
    print(f"[case] large attention {F} x {P} x {C} bf16", flush=True)
    q, k, v = (synth.make_tensor(F, P, C, 300 + t, "correlated", "bf16", device=DEV) for t in range(3))
    for od in ("bf16", "f32"):
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype=od)
        assert info["kernel"] == 1 and info["global_tiles"] == 4
        assert info["algorithmic_bytes"] == 4 * F * P * C * 2 + (2 if od == "f32" else 0) * F * P * C
        pos = sorted({0, 1, P // 3, P // 2, P - 2, P - 1} | set(((np.arange(8) * P) // 8).tolist()))
        ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, positions=pos)
        U.assert_parity(o, ref, od, positions=pos, what=f"large attention {od}")
        # the last frames (byte offsets beyond 4 GiB) were written, not left at the NaN fill
        assert torch.isfinite(o[-clip_len:].float()).all() and torch.isfinite(o[:clip_len].float()).all()
        del o
    del q, k, v
    torch.cuda.empty_cache()


def test_gather_of_a_context_beyond_4_gib_bit_exact():
    # the largest level: the materialised context of one tensor is 144 x 88 x 2,560 x 320 bf16 = 19 GiB
    wl = synth.WORKLOADS["C4"]
    lv = wl.levels[0]
    g = synth.global_idx_for(wl)
    print("[case] large gather: the context of the largest level", flush=True)
    k = synth.make_tensor(wl.F, lv.P, lv.C, 310, "iid", "bf16", device=DEV)
    plan = B.dsattn_plan(wl.clip_len, wl.n_clips, wl.local_ctx, lv.P, lv.heads, lv.head_dim, g,
                         io_dtype=B.DSATTN_BF16, device=0)
    lk = B.dsattn_plan_ctx_max(plan)
    assert wl.n_clips * lk * lv.P * lv.C * 2 > 4 * GIB4
    kc = torch.empty((wl.n_clips, lk, lv.P, lv.C), dtype=k.dtype, device=DEV)
    B.dsattn_gather_context(plan, k, None, kc, None)
    torch.cuda.synchronize()
    plan.close()
    idx, ln = oracle.ctx_indices(wl.clip_len, wl.n_clips, wl.local_ctx, g)
    for i in range(wl.n_clips):
        rows = torch.as_tensor(idx[i, :ln[i]].astype(np.int64), device=DEV)
        assert torch.equal(kc[i, :ln[i]].view(torch.int16), k.index_select(0, rows).view(torch.int16)), i
        assert (kc[i, ln[i]:].view(torch.int16) == 0).all(), i
    del k, kc
    torch.cuda.empty_cache()


def test_group_normalisation_of_a_tensor_beyond_4_gib():
    """The statistics run over all 3.8 * 10^9 elements, more than the oracle can be handed in
    reasonable time, so the reference statistics come from torch's own fp64 reductions on the
    device (a library routine, not this library's kernels), taken in frame chunks; sampled rows
    of the output, including the last ones, are then checked against the definition in fp64."""
    F, P, C, groups, clip_len = 4608, 2560, 320, 32, 16
    print(f"[case] large group normalisation {F} x {P} x {C} bf16, {groups} groups", flush=True)
    x = synth.make_tensor(F, P, C, 320, "correlated", "bf16", device=DEV)
    gen = torch.Generator(device="cpu").manual_seed(321)
    gamma = (1.0 + 0.1 * torch.randn(C, generator=gen)).to(DEV)
    beta = (0.1 * torch.randn(C, generator=gen)).to(DEV)
    y = torch.full_like(x, float("nan"))
    nbytes = B.dsattn_groupnorm_workspace(clip_len, F // clip_len, P, C, groups)
    ws = torch.empty((nbytes + 3) // 4, dtype=torch.float32, device=DEV)
    stats = torch.full((2 * groups,), float("nan"), dtype=torch.float32, device=DEV)
    B.dsattn_groupnorm(clip_len, F // clip_len, P, C, groups, x, y, ws, nbytes, gamma=gamma, beta=beta,
                       stats=stats, eps=1e-5)
    torch.cuda.synchronize()
    cpg = C // groups
    s1 = torch.zeros(groups, dtype=torch.float64, device=DEV)
    s2 = torch.zeros(groups, dtype=torch.float64, device=DEV)
    for f0 in range(0, F, 128):
        xc = x[f0:f0 + 128].to(torch.float64).view(-1, groups, cpg)
        s1 += xc.sum(dim=(0, 2))
        s2 += (xc * xc).sum(dim=(0, 2))
        del xc
    n = F * P * cpg
    mean = s1 / n
    var = s2 / n - mean * mean          # fp64 sums of values of order 1: cancellation is harmless here
    rstd = 1.0 / torch.sqrt(var + 1e-5)
    # the statistics the library reports: (mean, 1 / sqrt(variance + eps)) per group
    assert (stats[:groups].double() - mean).abs().max().item() < 1e-5
    assert ((stats[groups:].double() / rstd) - 1).abs().max().item() < 1e-5
    rows_f = [0, 1, F // 2, F - 2, F - 1]
    rows_p = [0, P // 2, P - 1]
    for f in rows_f:
        for p in rows_p:
            xr = x[f, p].to(torch.float64).view(groups, cpg)
            ref = ((xr - mean[:, None]) * rstd[:, None]).view(C) * gamma.double() + beta.double()
            got = y[f, p].to(torch.float64)
            refn = ref.cpu().numpy()
            err = np.abs(got.cpu().numpy() - refn)
            allow = 1e-4 * np.maximum(1.0, np.abs(refn)) + U.bf16_half_ulp(np.abs(refn))
            assert (err <= allow).all(), (f, p, float(err.max()))
    assert torch.isfinite(y[-1].float()).all()
    del x, y
    torch.cuda.empty_cache()


def test_convolution_and_projections_of_a_tensor_beyond_4_gib():
    # 16,384 frames x 2,560 positions x 64 channels bf16 = 5.0 GiB: 41.9 million rows
    clip_len, n_clips, P, c = 16, 1024, 2560, 64
    F = clip_len * n_clips
    assert F * P * c * 2 > GIB4
    print(f"[case] large convolution and projections {F} x {P} x {c} bf16", flush=True)
    x = synth.make_tensor(F, P, c, 330, "correlated", "bf16", device=DEV)
    w, b = (t.to(DEV) for t in synth.make_conv_weights(3, c, c, 331, "bf16"))
    assert B.dsattn_temporal_conv_info(clip_len, n_clips, P, c, c, 1)["kernel"] == 1
    y = torch.full_like(x, float("nan"))
    B.dsattn_temporal_conv(clip_len, n_clips, P, c, c, 1, x, w, y, bias=b)
    torch.cuda.synchronize()
    pos = [0, 1, P // 2, P - 1]
    pidx = torch.as_tensor(pos, device=DEV)
    xs = f64(x.index_select(1, pidx))
    ref = oracle.temporal_conv(xs, f64(w), clip_len, n_clips, bias=f64(b))
    check_conv(y.index_select(1, pidx), ref, "bf16", "large convolution")
    assert torch.isfinite(y[-1].float()).all() and torch.isfinite(y[0].float()).all()
    # three projections of the same rows in one launch
    ws = [synth.make_conv_weights(1, c, c, 332 + t, "bf16")[0].reshape(c, c).to(DEV) for t in range(3)]
    ys = [y] + [torch.full_like(x, float("nan")) for _ in range(2)]
    y.fill_(float("nan"))
    assert B.dsattn_linear_info(F * P, c, c, 3)["kernel"] == 1
    B.dsattn_linear(F * P, c, c, x, ws, ys)
    torch.cuda.synchronize()
    for t in range(3):
        check_conv(ys[t].index_select(1, pidx), oracle.linear(xs, f64(ws[t])), "bf16",
                   f"large projection {t}")
        assert torch.isfinite(ys[t][-1].float()).all()
    del x, y, ys
    torch.cuda.empty_cache()
