"""Helpers of the GPU parity tests: run the library through its C ABI (via the thin binding)
and the CPU oracle on the same seeded tensors, and compare element by element."""
import numpy as np
import torch

from oracle import oracle
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth

TOL_BF16 = 1e-2   # max-abs bar for bf16 I/O with fp32 accumulation
TOL_F32 = 1e-5    # max-abs bar for the fp32 path


def bf16_half_ulp(x):
    """Half a bf16 unit in the last place at |x| (8 significant bits)."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 8)


def bf16_allowance(ref):
    """Per-element bar for bf16 OUTPUT against the unrounded oracle: 1e-2 wherever |ref| < 4;
    beyond, where half a bf16 ulp alone exceeds 1e-2, the rounding's half ulp plus 2e-3 for the
    kernel's own error."""
    return np.where(np.abs(ref) < 4.0, TOL_BF16, bf16_half_ulp(ref) + 2e-3)


def dt_code(name):
    return B.DSATTN_F32 if name == "f32" else B.DSATTN_BF16


def library_forward(q, k, v, clip_len, n_clips, w, heads, gidx, out_dtype=None, scale=0.0,
                    flags=0, bias_local=0.0, bias_global=0.0, window=None):
    """q, k, v: CUDA tensors [F, P, C]. Returns (O tensor on device, launch info dict)."""
    F, P, C = q.shape
    io = "f32" if q.dtype == torch.float32 else "bf16"
    out_dtype = out_dtype or io
    plan = B.dsattn_plan(clip_len, n_clips, w, P, heads, C // heads, gidx, io_dtype=dt_code(io),
                         out_dtype=dt_code(out_dtype), scale=scale, flags=flags,
                         device=q.device.index or 0, bias_local=bias_local,
                         bias_global=bias_global, window=window)
    o = torch.full((F, P, C), float("nan"), dtype=synth.torch_dtype(out_dtype), device=q.device)
    B.dsattn_forward(plan, q, k, v, o)
    torch.cuda.synchronize()
    info = B.dsattn_plan_launch_info(plan)
    plan.close()
    return o, info


def oracle_forward(q, k, v, clip_len, n_clips, w, heads, gidx, scale=0.0, positions=None,
                   bias_local=0.0, bias_global=0.0, window=None, dedup=False):
    """Oracle on the exact upcast of the same tensors; optionally on a subset of positions.
    Returns O as [F, P', C] float64."""
    if positions is not None:
        idx = torch.as_tensor(positions, device=q.device)
        q, k, v = (t.index_select(1, idx) for t in (q, k, v))
    qn, kn, vn = (synth.to_f64_numpy(t, heads) for t in (q, k, v))
    o = oracle.forward(qn, kn, vn, clip_len, n_clips, w, gidx, scale=scale,
                       bias_local=bias_local, bias_global=bias_global,
                       window=-1 if window is None else window, dedup=dedup)
    return o.reshape(o.shape[0], o.shape[1], -1)


def compare(o_dev, ref, out_dtype, positions=None):
    """Returns max-abs error; for bf16 output also the worst error in units of the rounding
    allowance (half a bf16 ulp of the reference) so that output quantisation is visible."""
    got = o_dev
    if positions is not None:
        got = got.index_select(1, torch.as_tensor(positions, device=o_dev.device))
    got = got.to("cpu").to(torch.float64).numpy()
    assert np.isfinite(got).all(), "library output has non-finite values"
    err = np.abs(got - ref)
    return float(err.max()), err


def assert_parity(o_dev, ref, out_dtype, positions=None, what=""):
    """The bar: max-abs <= 1e-5 (fp32) / 1e-2 (bf16 in, fp32 out).  With bf16 OUTPUT the final
    rounding alone costs up to half a bf16 ulp of the result (2^-7 = 0.0078 for |O| in [2,4),
    2^-6 = 0.0156 for [4,8)), so there the bar is 1e-2 wherever |ref| < 4 and
    half-ulp(ref) + 2e-3 beyond: the kernel's own error (before the final rounding) is
    held to a few 1e-3 everywhere, and the fp32-output variant is held to 1e-2 outright."""
    mx, err = compare(o_dev, ref, out_dtype, positions)
    if out_dtype == "f32_strict":
        assert mx <= TOL_F32, f"{what}: max-abs {mx:.3e} > {TOL_F32}"
    elif out_dtype == "f32":
        assert mx <= TOL_BF16, f"{what}: max-abs {mx:.3e} > {TOL_BF16}"
    else:
        allow = bf16_allowance(ref)
        bad = err > allow
        assert not bad.any(), (f"{what}: {int(bad.sum())} elements beyond the bf16 bar; "
                               f"max-abs {mx:.3e}, worst |ref| {np.abs(ref[bad]).max():.3f}")
    return mx


class planner_env:
    """Pins planner choices (clips per chunk, wavefronts per workgroup) for one case."""

    def __init__(self, clips_per_task=None, waves_per_block=None):
        self.vals = {"DSATTN_CLIPS_PER_TASK": clips_per_task,
                     "DSATTN_WAVES_PER_BLOCK": waves_per_block}

    def __enter__(self):
        import os
        self.old = {k: os.environ.get(k) for k in self.vals}
        for k, v in self.vals.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = str(v)

    def __exit__(self, *exc):
        import os
        for k, v in self.old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
