"""Clip-parallel group normalisation (Section 4.2): boundary checks on the CPU, parity of the HIP
kernels against the oracle on the GPU."""
import ctypes

import numpy as np
import pytest
import torch

import parity_util as U
from oracle import oracle
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth

DEV = "cuda:0"


# ---------------------------------------------------------------- CPU: validation only

def raw_desc(**kw):
    d = dict(clip_len=4, n_clips=3, spatial=5, channels=64, groups=4, io_dtype=B.DSATTN_BF16,
             eps=1e-5)
    d.update(kw)
    return B.DsattnGnDesc(**d)


@pytest.mark.parametrize("kw,code", [
    (dict(clip_len=0), B.DSATTN_EINVAL), (dict(n_clips=0), B.DSATTN_EINVAL),
    (dict(spatial=0), B.DSATTN_EINVAL), (dict(channels=0), B.DSATTN_EINVAL),
    (dict(groups=0), B.DSATTN_EINVAL), (dict(groups=5), B.DSATTN_EINVAL),
    (dict(io_dtype=3), B.DSATTN_EINVAL), (dict(eps=-1.0), B.DSATTN_EINVAL),
    (dict(eps=float("nan")), B.DSATTN_EINVAL),
    (dict(channels=16, groups=4), B.DSATTN_EUNSUPPORTED),     # 4 channels per group < one lane
    (dict(channels=36, groups=3), B.DSATTN_EUNSUPPORTED),     # rows are not whole 16-byte lanes
    (dict(channels=16384, groups=1), B.DSATTN_EUNSUPPORTED),  # more than 1024 lanes per row
])
def test_groupnorm_rejects_bad_descriptors(kw, code):
    lib = B.load()
    out = ctypes.c_size_t()
    d = raw_desc(**kw)
    assert lib.dsattn_groupnorm_workspace(ctypes.byref(d), ctypes.byref(out)) == code
    assert lib.dsattn_groupnorm(ctypes.byref(d), 0x1000, None, None, 0x2000, None, 0x3000, 1 << 20,
                                None) == code


def test_groupnorm_argument_checks_before_launch():
    lib = B.load()
    d = raw_desc()
    out = ctypes.c_size_t()
    assert lib.dsattn_groupnorm_workspace(ctypes.byref(d), ctypes.byref(out)) == B.DSATTN_OK
    need = out.value
    assert need >= (3 * 4 + 2 * 4) * 4
    assert lib.dsattn_groupnorm_workspace(None, ctypes.byref(out)) == B.DSATTN_EINVAL
    assert lib.dsattn_groupnorm_workspace(ctypes.byref(d), None) == B.DSATTN_EINVAL
    ok = (0x1000, None, None, 0x2000, None, 0x3000, need, None)
    assert lib.dsattn_groupnorm(ctypes.byref(d), None, *ok[1:]) == B.DSATTN_EINVAL
    assert lib.dsattn_groupnorm(ctypes.byref(d), 0x1004, *ok[1:]) == B.DSATTN_EINVAL   # misaligned
    assert lib.dsattn_groupnorm(ctypes.byref(d), 0x1000, None, None, 0x2000, None, None, need,
                                None) == B.DSATTN_EINVAL                                # no workspace
    assert lib.dsattn_groupnorm(ctypes.byref(d), 0x1000, None, None, 0x2000, None, 0x3000,
                                need - 1, None) == B.DSATTN_EINVAL                      # too small
    assert "workspace" in B.dsattn_last_error()


# ---------------------------------------------------------------- GPU: parity

def run_gn(x, clip_len, n_clips, groups, gamma=None, beta=None, eps=1e-5, in_place=False):
    F, P, C = x.shape
    dt = U.dt_code("f32" if x.dtype == torch.float32 else "bf16")
    nbytes = B.dsattn_groupnorm_workspace(clip_len, n_clips, P, C, groups, io_dtype=dt, eps=eps)
    ws = torch.empty((nbytes + 3) // 4, dtype=torch.float32, device=x.device)
    y = x if in_place else torch.full_like(x, float("nan"))
    stats = torch.full((2 * groups,), float("nan"), dtype=torch.float32, device=x.device)
    B.dsattn_groupnorm(clip_len, n_clips, P, C, groups, x, y, ws, nbytes, gamma=gamma, beta=beta,
                       stats=stats, io_dtype=dt, eps=eps)
    torch.cuda.synchronize()
    return y, stats


GN_SHAPES = [
    # clip_len, n_clips, P, C, groups, dtype
    (4, 3, 5, 64, 4, "bf16"),
    (16, 4, 7, 320, 8, "bf16"),
    (16, 4, 7, 320, 32, "bf16"),      # 10 channels per group: lanes straddle group boundaries
    (4, 6, 5, 640, 32, "bf16"),       # 20 channels per group
    (2, 3, 9, 48, 4, "bf16"),         # 12 channels per group
    (3, 4, 6, 36, 6, "f32"),          # 6 channels per group, 4-channel lanes
    (1, 9, 3, 1280, 32, "bf16"),      # one frame per clip
    (5, 1, 2, 8192, 1, "bf16"),       # 1024 lanes per row, one workgroup row
    (3, 4, 6, 24, 3, "f32"),
    (2, 2, 1, 4, 1, "f32"),           # a single lane per row
    (8, 3, 11, 640, 32, "f32"),
]


@pytest.mark.gpu
@pytest.mark.parametrize("shape", GN_SHAPES)
def test_groupnorm_matches_oracle(shape):
    clip_len, n_clips, P, C, groups, dtype = shape
    print(f"[case] groupnorm {shape}", flush=True)
    F = clip_len * n_clips
    x = synth.make_tensor(F, P, C, 5, "iid", dtype)
    # clips with different means and scales
    x = (x.float() * (1.0 + torch.arange(F)[:, None, None] / F) +
         0.5 * torch.sin(torch.arange(F, dtype=torch.float32))[:, None, None]).to(x.dtype).to(DEV)
    gen = torch.Generator().manual_seed(3)
    gamma = torch.randn(C, generator=gen).to(DEV)
    beta = torch.randn(C, generator=gen).to(DEV)
    xs = x.to("cpu").to(torch.float64).numpy()
    ref, mean, var = oracle.groupnorm(xs, clip_len, n_clips, groups, eps=1e-5,
                                      gamma=gamma.cpu().double().numpy(),
                                      beta=beta.cpu().double().numpy())
    y, stats = run_gn(x, clip_len, n_clips, groups, gamma, beta)
    st = stats.cpu().double().numpy()
    np.testing.assert_allclose(st[:groups], mean, rtol=0, atol=2e-6)
    np.testing.assert_allclose(st[groups:], 1.0 / np.sqrt(var + 1e-5), rtol=3e-6, atol=0)
    U.assert_parity(y, ref, "f32_strict" if dtype == "f32" else "bf16", what=f"groupnorm {shape}")
    # no affine parameters, in place
    ref2, _, _ = oracle.groupnorm(xs, clip_len, n_clips, groups, eps=1e-5)
    y2, _ = run_gn(x.clone(), clip_len, n_clips, groups, in_place=True)
    U.assert_parity(y2, ref2, "f32_strict" if dtype == "f32" else "bf16", what="groupnorm in place")


@pytest.mark.gpu
def test_groupnorm_partition_independent_and_deterministic():
    F, P, C, groups = 48, 9, 320, 8
    x = synth.make_tensor(F, P, C, 7, "correlated", "bf16").to(DEV)
    ys = [run_gn(x, cl, F // cl, groups)[0] for cl in (16, 4, 48, 1)]
    ref, _, _ = oracle.groupnorm(x.cpu().double().numpy(), 16, 3, groups)
    for y in ys:
        U.assert_parity(y, ref, "bf16", what="groupnorm partition")
    again = run_gn(x, 16, 3, groups)[0]
    assert torch.equal(again, ys[0])


@pytest.mark.gpu
def test_groupnorm_full_size_level():
    # the headline level's tensor: 2,304 frames x 160 positions x 1,280 channels, 32 groups
    wl = synth.WORKLOADS["C3"]
    lv = wl.levels[0]
    x = synth.make_tensor(wl.F, lv.P, lv.C, 11, "correlated", "bf16", device=DEV)
    y, stats = run_gn(x, wl.clip_len, wl.n_clips, 32)
    # statistics against a library reduction on the device (fp64), outputs on sampled positions
    xg = x.view(wl.F, lv.P, 32, lv.C // 32).double()
    mean = xg.mean(dim=(0, 1, 3))
    var = xg.var(dim=(0, 1, 3), unbiased=False)
    assert (stats[:32].double() - mean).abs().max().item() < 2e-6
    assert ((stats[32:].double() * torch.sqrt(var + 1e-5)) - 1).abs().max().item() < 3e-6
    pos = [0, 53, 159]
    ref = ((xg[:, pos] - mean[None, None, :, None]) / torch.sqrt(var + 1e-5)[None, None, :, None])
    ref = ref.reshape(wl.F, len(pos), lv.C).cpu().numpy()
    U.assert_parity(y, ref, "bf16", positions=pos, what="groupnorm full size")


@pytest.mark.gpu
def test_groupnorm_level_sized_tensor_against_the_oracle():
    # a whole level-sized tensor (the 64-frame workload's level: 64 x 2,560 x 320, 32 groups)
    # checked element by element against the oracle itself, statistics included
    wl = synth.WORKLOADS["C1"]
    lv = wl.levels[0]
    print(f"[case] groupnorm {wl.F} x {lv.P} x {lv.C} vs oracle", flush=True)
    x = synth.make_tensor(wl.F, lv.P, lv.C, 13, "correlated", "bf16", device=DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(14)
    gamma = 1.0 + 0.1 * torch.randn(lv.C, generator=gen, device=DEV)
    beta = 0.1 * torch.randn(lv.C, generator=gen, device=DEV)
    y, stats = run_gn(x, wl.clip_len, wl.n_clips, 32, gamma=gamma, beta=beta)
    ref, mean, var = oracle.groupnorm(x.cpu().double().numpy(), wl.clip_len, wl.n_clips, 32,
                                      gamma=gamma.cpu().double().numpy(),
                                      beta=beta.cpu().double().numpy())
    st = stats.cpu().double().numpy()
    np.testing.assert_allclose(st[:32], mean, rtol=0, atol=2e-6)
    np.testing.assert_allclose(st[32:], 1.0 / np.sqrt(var + 1e-5), rtol=3e-6, atol=0)
    U.assert_parity(y, ref, "bf16", what="groupnorm level-sized vs oracle")


@pytest.mark.gpu
@pytest.mark.parametrize("offset", [100.0, -3000.0])
def test_groupnorm_large_means_do_not_cancel(offset):
    """Means far larger than the deviations (fp32 tensors, |mean| / std up to 3,000): the one-pass
    statistics keep their accuracy because every partial sum is taken about a nearby pilot."""
    clip_len, n_clips, P, C, groups = 4, 5, 33, 64, 8
    F = clip_len * n_clips
    gen = torch.Generator().manual_seed(4)
    x = (torch.randn(F, P, C, generator=gen) + offset +
         0.25 * torch.arange(F, dtype=torch.float32)[:, None, None]).to(DEV)
    ref, mean, var = oracle.groupnorm(x.cpu().double().numpy(), clip_len, n_clips, groups, eps=1e-5)
    y, stats = run_gn(x, clip_len, n_clips, groups)
    st = stats.cpu().double().numpy()
    # the mean is held to fp32 resolution at its own size, the variance to a few 1e-6 relative
    np.testing.assert_allclose(st[:groups], mean, rtol=2e-7, atol=0)
    np.testing.assert_allclose(st[groups:], 1.0 / np.sqrt(var + 1e-5), rtol=1e-5, atol=0)
    # y = (x - mean) * rstd: the subtraction of two fp32 numbers of size |offset| costs up to
    # one ulp of them, relative to a spread of order one
    err = np.abs(y.cpu().double().numpy() - ref).max()
    assert err <= 4 * abs(offset) * 2.0 ** -24 + 1e-5, err
