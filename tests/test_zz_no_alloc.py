"""dsattn_groupnorm_static, the entry point that allocates nothing: the per-workgroup moments go to
a static device array instead of a caller's workspace.  Its output must equal that of
dsattn_groupnorm (same kernels, so bit for bit) and meet the oracle's bar, on two calls in a row
that share the array, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import parity_util as U
from oracle import oracle
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth

DEV = "cuda:0"


def test_static_scratch_limit_is_stated_and_enforced_on_the_host():
    lib = B.load()
    assert B.dsattn_groupnorm_static_max_bytes() == 4 << 20
    # 2,048 workgroups x 128 groups x 16 bytes = 4 MiB of moments, plus the statistics: one
    # kilobyte too many.  The check comes before any device call, so it runs without a GPU.
    big = B.DsattnGnDesc(16, 2048, 64, 1024, 128, B.DSATTN_BF16, 1e-5)
    need = ctypes.c_size_t()
    assert lib.dsattn_groupnorm_workspace(ctypes.byref(big), ctypes.byref(need)) == B.DSATTN_OK
    assert need.value > B.dsattn_groupnorm_static_max_bytes()
    rc = lib.dsattn_groupnorm_static(ctypes.byref(big), 0x1000, None, None, 0x2000, None, None)
    assert rc == B.DSATTN_EUNSUPPORTED and "scratch" in B.dsattn_last_error()
    ok = B.DsattnGnDesc(4, 3, 5, 64, 4, B.DSATTN_BF16, 1e-5)
    assert lib.dsattn_groupnorm_static(ctypes.byref(ok), None, None, None, 0x2000, None,
                                       None) == B.DSATTN_EINVAL
    assert lib.dsattn_groupnorm_static(ctypes.byref(ok), 0x1004, None, None, 0x2000, None,
                                       None) == B.DSATTN_EINVAL
    bad = B.DsattnGnDesc(4, 3, 5, 64, 5, B.DSATTN_BF16, 1e-5)
    assert lib.dsattn_groupnorm_static(ctypes.byref(bad), 0x1000, None, None, 0x2000, None,
                                       None) == B.DSATTN_EINVAL


def _both_ways(clip_len, n_clips, P, C, groups, dtype, seed):
    F = clip_len * n_clips
    dt = B.DSATTN_F32 if dtype == "f32" else B.DSATTN_BF16
    x = synth.make_tensor(F, P, C, seed, "correlated", dtype, device=DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed + 1)
    gamma = 1.0 + 0.1 * torch.randn(C, generator=gen, device=DEV)
    beta = 0.1 * torch.randn(C, generator=gen, device=DEV)
    print(f"[case] groupnorm static vs workspace: {n_clips}x{clip_len} frames, P={P}, C={C}, "
          f"groups={groups}, {dtype}", flush=True)
    # the existing entry point, with a workspace of its own
    nbytes = B.dsattn_groupnorm_workspace(clip_len, n_clips, P, C, groups, io_dtype=dt)
    ws = torch.empty((nbytes + 3) // 4, dtype=torch.float32, device=DEV)
    y_ref = torch.full_like(x, float("nan"))
    st_ref = torch.full((2 * groups,), float("nan"), dtype=torch.float32, device=DEV)
    B.dsattn_groupnorm(clip_len, n_clips, P, C, groups, x, y_ref, ws, nbytes, gamma=gamma,
                       beta=beta, stats=st_ref, io_dtype=dt)
    # the entry point under test
    y = torch.full_like(x, float("nan"))
    st = torch.full((2 * groups,), float("nan"), dtype=torch.float32, device=DEV)
    B.dsattn_groupnorm_static(clip_len, n_clips, P, C, groups, x, y, gamma=gamma, beta=beta,
                              stats=st, io_dtype=dt)
    torch.cuda.synchronize()
    assert nbytes <= B.dsattn_groupnorm_static_max_bytes()
    same = torch.equal(y.view(torch.int16 if dtype == "bf16" else torch.int32),
                       y_ref.view(torch.int16 if dtype == "bf16" else torch.int32))
    assert same, "static-scratch output differs from the workspace entry point's"
    assert torch.equal(st.view(torch.int32), st_ref.view(torch.int32))
    # and against the oracle, to the group-norm tests' bar
    xn = x.to("cpu").to(torch.float64).numpy()
    ref, mean, var = oracle.groupnorm(xn, clip_len, n_clips, groups, eps=1e-5,
                                      gamma=gamma.cpu().double().numpy(),
                                      beta=beta.cpu().double().numpy())
    U.assert_parity(y, ref, "f32_strict" if dtype == "f32" else "bf16",
                    what="groupnorm static scratch")
    np.testing.assert_allclose(st[:groups].cpu().numpy(), mean, rtol=0, atol=2e-6)
    np.testing.assert_allclose(st[groups:].cpu().numpy(), 1.0 / np.sqrt(var + 1e-5), rtol=1e-5,
                               atol=0)


@pytest.mark.gpu
def test_static_scratch_matches_workspace_entry_point_twice_in_a_row():
    # a C1-level-like tensor first (its moments fill about a fifth of the array), then a smaller
    # one that reuses the array while it still holds the first call's contents
    _both_ways(16, 12, 640, 320, 32, "bf16", 4100)
    _both_ways(8, 3, 37, 64, 4, "bf16", 4200)
    _both_ways(4, 2, 19, 48, 6, "f32", 4300)
