"""CPU-side tests of the C-ABI boundary: exported symbols, argument validation,
host-only plans and bit-exact context tables against the oracle.  No kernel is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from conftest import ROOT, read_golden_ctx_lists
from oracle import oracle
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dsattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dsattn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def raw_plan(desc_kwargs, gidx, device=-1):
    lib = B.load()
    d = dict(clip_len=4, n_clips=2, local_ctx=1, spatial=16, heads=1, head_dim=8,
             io_dtype=B.DSATTN_F32, out_dtype=B.DSATTN_F32, scale=0.0, flags=0, bias_local=0.0,
             bias_global=0.0, window=0)
    d.update(desc_kwargs)
    desc = B.DsattnDesc(**d)
    g = np.asarray(gidx, dtype=np.int32)
    h = ctypes.c_void_p()
    rc = lib.dsattn_plan(ctypes.byref(desc), g.ctypes.data if g.size else None, g.size, device,
                         ctypes.byref(h))
    return rc, h


@pytest.mark.parametrize("kw,g", [
    (dict(clip_len=0), [0]), (dict(n_clips=0), [0]), (dict(local_ctx=-1), [0]),
    (dict(spatial=0), [0]), (dict(heads=0), [0]), (dict(head_dim=0), [0]),
    (dict(io_dtype=7), [0]), (dict(out_dtype=-1), [0]),
    (dict(io_dtype=B.DSATTN_F32, out_dtype=B.DSATTN_BF16), [0]),
    (dict(scale=float("nan")), [0]), (dict(scale=float("inf")), [0]),
    (dict(bias_local=float("nan")), [0]), (dict(bias_global=float("-inf")), [0]),
    (dict(flags=B.DSATTN_FLAG_SLIDING_WINDOW, window=-1), [0]),
    (dict(), [8]), (dict(), [-1]), (dict(), [0, 3, 99]),
])
def test_plan_rejects_bad_arguments(kw, g):
    rc, h = raw_plan(kw, g)
    assert rc == B.DSATTN_EINVAL
    assert not h.value
    assert B.dsattn_last_error() != ""


def test_plan_null_pointers_and_bad_device():
    lib = B.load()
    h = ctypes.c_void_p()
    assert lib.dsattn_plan(None, None, 0, -1, ctypes.byref(h)) == B.DSATTN_EINVAL
    desc = B.DsattnDesc(4, 2, 1, 16, 1, 8, 0, 0, 0.0, 0)
    assert lib.dsattn_plan(ctypes.byref(desc), None, 0, -1, None) == B.DSATTN_EINVAL
    assert lib.dsattn_plan(ctypes.byref(desc), None, 2, -1, ctypes.byref(h)) == B.DSATTN_EINVAL
    assert lib.dsattn_plan(ctypes.byref(desc), None, -1, -1, ctypes.byref(h)) == B.DSATTN_EINVAL
    assert lib.dsattn_plan(ctypes.byref(desc), None, 0, -2, ctypes.byref(h)) == B.DSATTN_EINVAL
    lib.dsattn_plan_destroy(None)  # must be a no-op
    out = ctypes.c_int32()
    assert lib.dsattn_plan_ctx_max(None, ctypes.byref(out)) == B.DSATTN_EINVAL
    assert lib.dsattn_plan_ctx_indices(None, None, None) == B.DSATTN_EINVAL
    assert lib.dsattn_plan_launch_info(None, None) == B.DSATTN_EINVAL


def test_host_only_plan_refuses_device_work():
    lib = B.load()
    rc, h = raw_plan({}, [0, 4])
    assert rc == B.DSATTN_OK and h.value
    fake = 0x1000  # never dereferenced: validation stops first
    assert lib.dsattn_forward(h, fake, fake, fake, fake, None) == B.DSATTN_ENODEVICE
    assert lib.dsattn_forward_ctx(h, fake, fake, fake, fake, None) == B.DSATTN_ENODEVICE
    assert lib.dsattn_gather_context(h, fake, fake, fake, fake, None) == B.DSATTN_ENODEVICE
    assert lib.dsattn_forward(h, None, fake, fake, fake, None) == B.DSATTN_EINVAL
    assert lib.dsattn_forward(None, fake, fake, fake, fake, None) == B.DSATTN_EINVAL
    lib.dsattn_plan_destroy(h)


def test_copy_probe_validates_before_launch():
    lib = B.load()
    assert lib.dsattn_copy_probe(None, 0x1000, 64, None) == B.DSATTN_EINVAL
    assert lib.dsattn_copy_probe(0x1000, 0x2000, 0, None) == B.DSATTN_EINVAL
    assert lib.dsattn_copy_probe(0x1000, 0x2000, 24, None) == B.DSATTN_EINVAL   # not x16
    assert lib.dsattn_copy_probe(0x1004, 0x2000, 64, None) == B.DSATTN_EINVAL   # misaligned
    assert lib.dsattn_copy_probe(0x1000, 0x1010, 64, None) == B.DSATTN_EINVAL   # overlap


def test_strerror_is_total():
    for code in (0, -1, -2, -3, -4, -5, -77, 5):
        s = B.dsattn_strerror(code)
        assert isinstance(s, str) and s
    assert B.dsattn_strerror(0) == "ok"


@pytest.mark.parametrize("case", read_golden_ctx_lists())
def test_plan_ctx_table_matches_hand_derived(case):
    clip_len, n_clips, w, g, clip, expected = case
    plan = B.dsattn_plan(clip_len, n_clips, w, 1, 1, 8, g, io_dtype=B.DSATTN_F32, device=-1)
    idx, ln = B.dsattn_plan_ctx_indices(plan)
    assert idx[clip, :ln[clip]].tolist() == expected
    plan.close()


@pytest.mark.parametrize("name", ["C0", "C1", "C2", "C3", "C4"])
def test_plan_ctx_table_bit_exact_vs_oracle_on_workloads(name):
    wl = synth.WORKLOADS[name]
    g = synth.global_idx_for(wl)
    assert len(g) == wl.n_global
    lv = wl.levels[0]
    dt = B.DSATTN_F32 if wl.dtype == "f32" else B.DSATTN_BF16
    plan = B.dsattn_plan(wl.clip_len, wl.n_clips, wl.local_ctx, lv.P, lv.heads, lv.head_dim, g,
                         io_dtype=dt, device=-1)
    idx, ln = B.dsattn_plan_ctx_indices(plan)
    ridx, rln = oracle.ctx_indices(wl.clip_len, wl.n_clips, wl.local_ctx, g)
    assert B.dsattn_plan_ctx_max(plan) == ridx.shape[1]
    assert np.array_equal(idx, ridx) and np.array_equal(ln, rln)
    info = B.dsattn_plan_launch_info(plan)
    esz = 4 if wl.dtype == "f32" else 2
    assert info["algorithmic_bytes"] == 4 * wl.F * lv.P * lv.C * esz
    plan.close()


def test_plan_ctx_table_random_shapes_vs_oracle():
    rng = np.random.default_rng(0)
    for _ in range(200):
        clip_len = int(rng.integers(1, 20))
        n_clips = int(rng.integers(1, 12))
        w = int(rng.integers(0, 3 * clip_len + 2))
        F = clip_len * n_clips
        g = rng.integers(0, F, size=int(rng.integers(0, 9))).astype(np.int32)
        plan = B.dsattn_plan(clip_len, n_clips, w, 2, 2, 4, g, io_dtype=B.DSATTN_F32, device=-1)
        idx, ln = B.dsattn_plan_ctx_indices(plan)
        ridx, rln = oracle.ctx_indices(clip_len, n_clips, w, g)
        assert np.array_equal(idx, ridx) and np.array_equal(ln, rln)
        plan.close()


def test_workload_recipes():
    assert synth.stride_global_idx(8, 2).tolist() == [0, 4]
    assert synth.stride_global_idx(64, 16).tolist() == list(range(0, 64, 4))
    assert synth.stride_global_idx(2304, 16).tolist() == list(range(0, 2304, 144))
    g = synth.global_idx_for(synth.WORKLOADS["C4"])
    assert len(g) == 64 and len(set(g.tolist())) == 64 and (np.diff(g) > 0).all()
    assert g.min() >= 0 and g.max() < 2304
    q1 = synth.make_tensor(8, 4, 16, 5, "correlated", "bf16")
    q2 = synth.make_tensor(8, 4, 16, 5, "correlated", "bf16")
    assert (q1 == q2).all()
    # frames are strongly correlated, positions are not
    x = q1.float()
    assert (x[0] - x[7]).abs().mean() < 0.3 and (x[:, 0] - x[:, 1]).abs().mean() > 0.5


# ---------------------------------------------------------------- launch planner (host logic)

def plan_info(wl, lv, **kw):
    g = synth.global_idx_for(wl)
    plan = B.dsattn_plan(wl.clip_len, wl.n_clips, wl.local_ctx, lv.P, lv.heads, lv.head_dim, g,
                         io_dtype=B.DSATTN_F32 if wl.dtype == "f32" else B.DSATTN_BF16, device=-1,
                         **kw)
    info = B.dsattn_plan_launch_info(plan)
    plan.close()
    return info


def test_planner_choices_per_level():
    W = synth.WORKLOADS
    assert plan_info(W["C0"], W["C0"].levels[0])["kernel"] == 0          # fp32: vector-ALU kernel
    c3 = plan_info(W["C3"], W["C3"].levels[0])
    assert (c3["kernel"], c3["heads_per_wave"], c3["local_tiles"], c3["global_tiles"]) == (1, 1, 2, 1)
    assert c3["block_threads"] == 512 and c3["lds_bytes"] <= 160 * 1024
    assert plan_info(W["C2"], W["C2"].levels[0])["heads_per_wave"] == 2   # 2 x 80 channels per row
    assert plan_info(W["C1"], W["C1"].levels[0])["heads_per_wave"] == 4   # 4 x 40
    for lv in W["C4"].levels:                                             # 64 global frames
        i = plan_info(W["C4"], lv)
        assert i["kernel"] == 1 and i["global_tiles"] == 4 and i["local_tiles"] == 2
        assert i["heads_per_wave"] * lv.head_dim <= 160
    for name in ("C1", "C2", "C3", "C4"):
        for lv in W[name].levels:
            i = plan_info(W[name], lv)
            waves = i["block_threads"] // 64
            row_groups = lv.P * lv.heads // i["heads_per_wave"]
            chunks = -(-W[name].n_clips // i["clips_per_task"])
            assert row_groups % waves == 0
            assert i["n_tasks"] == row_groups * chunks
            assert 1 <= i["clips_per_task"] <= W[name].n_clips


def test_planner_fallbacks_and_overrides(monkeypatch):
    W = synth.WORKLOADS
    lv = W["C3"].levels[0]
    assert plan_info(W["C3"], lv, flags=B.DSATTN_FLAG_FORCE_GENERIC)["kernel"] == 0
    monkeypatch.setenv("DSATTN_FORCE_GENERIC", "1")
    assert plan_info(W["C3"], lv)["kernel"] == 0
    monkeypatch.delenv("DSATTN_FORCE_GENERIC")
    monkeypatch.setenv("DSATTN_CLIPS_PER_TASK", "7")
    monkeypatch.setenv("DSATTN_WAVES_PER_BLOCK", "2")
    i = plan_info(W["C3"], lv)
    assert i["clips_per_task"] == 7 and i["block_threads"] == 128
    assert i["n_tasks"] == 1280 * 21
    monkeypatch.delenv("DSATTN_CLIPS_PER_TASK")
    monkeypatch.delenv("DSATTN_WAVES_PER_BLOCK")
    # shapes without an MFMA variant run the generic kernel
    for kw in (dict(clip_len=8), dict(head_dim=48), dict(local_ctx=17), dict(n_global=65)):
        clip_len = kw.get("clip_len", 16)
        g = list(range(kw.get("n_global", 4)))
        plan = B.dsattn_plan(clip_len, 8, kw.get("local_ctx", 2), 4, 2, kw.get("head_dim", 160), g,
                             device=-1)
        assert B.dsattn_plan_launch_info(plan)["kernel"] == 0, kw
        plan.close()


def test_flags_are_validated_and_dedup_limits_the_planner():
    lib = B.load()
    d = B.DsattnDesc(16, 4, 2, 4, 2, 160, B.DSATTN_BF16, B.DSATTN_BF16, 0.0, 8, 0.0, 0.0, 0)
    out = ctypes.c_void_p()
    assert lib.dsattn_plan(ctypes.byref(d), None, 0, -1, ctypes.byref(out)) == B.DSATTN_EINVAL
    assert "flag" in B.dsattn_last_error()
    # the set-union option runs on the matrix-core kernel with up to 16 global frames, and with
    # up to 64 where the variant has a whole SIMD's registers (head_dim 160 and 128)
    for D, G, kernel in ((160, 16, 1), (160, 17, 1), (160, 64, 1), (160, 0, 1), (128, 40, 1),
                         (80, 16, 1), (80, 17, 0), (40, 64, 0), (96, 33, 0)):
        plan = B.dsattn_plan(16, 8, 2, 4, 2, D, list(range(G)), flags=B.DSATTN_FLAG_DEDUP_GLOBAL,
                             device=-1)
        assert B.dsattn_plan_launch_info(plan)["kernel"] == kernel, (D, G)
        plan.close()


@pytest.mark.parametrize("D,h,G,hpw", [
    (128, 8, 16, 1), (96, 8, 16, 2), (96, 5, 16, 1), (64, 8, 16, 2), (64, 3, 0, 1), (32, 8, 16, 4),
    (32, 6, 16, 2), (32, 7, 3, 1), (40, 6, 16, 2), (40, 5, 16, 1), (80, 3, 16, 1),
    # 17..64 global frames: fewer heads per wavefront so that the global context fits in registers
    (128, 4, 64, 1), (96, 4, 33, 1), (64, 4, 64, 1), (32, 8, 64, 2), (32, 3, 64, 1), (40, 7, 17, 1),
])
def test_planner_head_dims_and_heads_per_wave(D, h, G, hpw):
    """Every supported head_dim has an MFMA variant for any head count: the planner takes the
    widest rows (most heads per wavefront) that divide the head count."""
    plan = B.dsattn_plan(16, 8, 4, 6, h, D, list(range(0, 2 * G, 2)), device=-1)
    i = B.dsattn_plan_launch_info(plan)
    plan.close()
    assert i["kernel"] == 1 and i["heads_per_wave"] == hpw, i
    assert i["global_tiles"] == (0 if G == 0 else 1 if G <= 16 else 4)
    assert i["n_tasks"] % (i["block_threads"] // 64) == 0
    assert i["lds_bytes"] <= 160 * 1024


def test_header_is_plain_c_and_usable_from_c(tmp_path):
    """include/dsattn.h compiles as C99 with warnings as errors, and a C program linked against
    libdsattn.so drives the host-side entry points."""
    import subprocess
    exe = tmp_path / "host_only_plan"
    src = os.path.join(ROOT, "tests", "c_abi", "host_only_plan.c")
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                    "-I", os.path.join(ROOT, "include"), src, "-o", str(exe),
                    "-L", libdir, "-l:libdsattn.so", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.startswith("ok lk_max=7")


# ---------------------------------------------------------------- binding: tensor checks
# The C ABI takes bare pointers, so the Python wrappers refuse tensors whose size, element type or
# device does not fit the plan or descriptor before anything reaches a kernel.  Driven here with
# host-only plans (device = -1) and CPU tensors: no GPU is needed to reach the checks.

def _host_plan(**kw):
    args = dict(clip_len=4, n_clips=3, local_ctx=1, spatial=5, heads=2, head_dim=8,
                global_idx=[0, 7], io_dtype=B.DSATTN_BF16, device=-1)
    args.update(kw)
    return B.dsattn_plan(**args)


def test_binding_refuses_wrong_sized_or_typed_tensors_for_a_plan():
    import torch
    plan = _host_plan()
    n = 12 * 5 * 16
    good = lambda: torch.zeros(12, 5, 16, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="elements"):
        B.dsattn_forward(plan, torch.zeros(n - 16, dtype=torch.bfloat16), good(), good(), good())
    with pytest.raises(ValueError, match="elements"):
        B.dsattn_forward(plan, good(), good(), good(), torch.zeros(n + 1, dtype=torch.bfloat16))
    with pytest.raises(ValueError, match="dtype"):
        B.dsattn_forward(plan, good(), torch.zeros(12, 5, 16, dtype=torch.float32), good(), good())
    with pytest.raises(ValueError, match="dtype"):   # O follows out_dtype (bf16 here)
        B.dsattn_forward(plan, good(), good(), good(), torch.zeros(12, 5, 16, dtype=torch.float32))
    with pytest.raises(ValueError, match="contiguous"):
        B.dsattn_forward(plan, torch.zeros(12, 16, 5, dtype=torch.bfloat16).transpose(1, 2), good(),
                         good(), good())
    # well-formed tensors pass the wrapper; the library then refuses the host-only plan
    with pytest.raises(B.DsattnError) as ei:
        B.dsattn_forward(plan, good(), good(), good(), good(), stream=0)
    assert ei.value.code == B.DSATTN_ENODEVICE
    # materialised contexts are [N, lk_max, P, C]
    lk = B.dsattn_plan_ctx_max(plan)
    assert lk == 4 + 2 + 2
    ctx = lambda k=lk: torch.zeros(3, k, 5, 16, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="Kctx"):
        B.dsattn_gather_context(plan, good(), good(), ctx(lk - 1), ctx(), stream=0)
    with pytest.raises(ValueError, match="Vctx"):
        B.dsattn_forward_ctx(plan, good(), ctx(), ctx(lk + 1), good(), stream=0)
    with pytest.raises(B.DsattnError):
        B.dsattn_forward_ctx(plan, good(), ctx(), ctx(), good(), stream=0)
    plan.close()
    # fp32 output of a bf16 plan
    plan = _host_plan(out_dtype=B.DSATTN_F32)
    with pytest.raises(ValueError, match="dtype"):
        B.dsattn_forward(plan, good(), good(), good(), good(), stream=0)
    plan.close()


def test_binding_refuses_tensors_on_the_wrong_device():
    import torch
    plan = B.Plan(None, B.DsattnDesc(4, 3, 1, 5, 2, 8, B.DSATTN_BF16, B.DSATTN_BF16, 0.0, 0, 0.0,
                                     0.0, 0), 0, device=0)   # a device plan's bookkeeping only
    t = torch.zeros(12, 5, 16, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="device memory expected"):
        plan.check("dsattn_forward", [plan.frames(t, "Q")])
    with pytest.raises(ValueError, match="device memory expected"):
        B.dsattn_copy_probe(t, t.clone(), t.numel() * 2, stream=0)
    with pytest.raises(ValueError, match="at least"):
        B.dsattn_copy_probe(t, t.clone(), t.numel() * 2 + 16, stream=0)


def test_binding_checks_groupnorm_conv_and_linear_tensors():
    import torch
    bf = lambda *s: torch.zeros(*s, dtype=torch.bfloat16)
    f32 = lambda *s: torch.zeros(*s, dtype=torch.float32)
    # group normalisation: X, Y [F, P, C]; gamma, beta [C] fp32; stats [2 groups] fp32
    gn = dict(clip_len=4, n_clips=3, spatial=5, channels=64, groups=4)
    with pytest.raises(ValueError, match="X"):
        B.dsattn_groupnorm(**gn, X=bf(12, 5, 32), Y=bf(12, 5, 64), workspace=f32(1024),
                           workspace_bytes=4096, stream=0)
    with pytest.raises(ValueError, match="gamma"):
        B.dsattn_groupnorm(**gn, X=bf(12, 5, 64), Y=bf(12, 5, 64), workspace=f32(1024),
                           workspace_bytes=4096, gamma=bf(64), stream=0)
    with pytest.raises(ValueError, match="stats"):
        B.dsattn_groupnorm_static(**gn, X=bf(12, 5, 64), Y=bf(12, 5, 64), stats=f32(4), stream=0)
    with pytest.raises(ValueError, match="device memory expected"):
        B.dsattn_groupnorm_static(**gn, X=bf(12, 5, 64), Y=bf(12, 5, 64), stream=0)
    # temporal convolution: W [2n + 1, c_out, c_in], Y [F, P, c_out]
    cv = dict(clip_len=4, n_clips=3, spatial=5, c_in=16, c_out=24, reach=1)
    with pytest.raises(ValueError, match="W"):
        B.dsattn_temporal_conv(**cv, X=bf(12, 5, 16), W=bf(1, 24, 16), Y=bf(12, 5, 24), stream=0)
    with pytest.raises(ValueError, match="Y"):
        B.dsattn_temporal_conv(**cv, X=bf(12, 5, 16), W=bf(3, 24, 16), Y=bf(12, 5, 16), stream=0)
    with pytest.raises(ValueError, match="bias"):
        B.dsattn_temporal_conv(**cv, X=bf(12, 5, 16), W=bf(3, 24, 16), Y=bf(12, 5, 24),
                               bias=bf(24), stream=0)
    # projections: every W [c_out, c_in], every Y [rows, c_out]
    with pytest.raises(ValueError, match=r"W\[1\]"):
        B.dsattn_linear(60, 16, 24, bf(60, 16), [bf(24, 16), bf(16, 16)], [bf(60, 24), bf(60, 24)],
                        stream=0)
    with pytest.raises(ValueError, match=r"Y\[0\]"):
        B.dsattn_linear(60, 16, 24, bf(60, 16), [bf(24, 16)], [bf(59, 24)], stream=0)
    with pytest.raises(ValueError, match="dtype"):
        B.dsattn_linear(60, 16, 24, bf(60, 16), [bf(24, 16)], [f32(60, 24)], stream=0)


# ---------------------------------------------------------------- planner: long clips, resolved variant

@pytest.mark.parametrize("D,h", [(160, 8), (80, 8), (40, 8)])
@pytest.mark.parametrize("clip_len,n_clips", [(32, 72), (48, 48), (288, 8)])
def test_long_clips_with_a_window_run_the_matrix_core_kernel(D, h, clip_len, n_clips):
    for w, r, G, reach in ((8, 8, 16, 8), (8, 3, 0, 3), (2, 8, 64, 8), (4, 0, 16, 0), (8, 16, 16, 16)):
        plan = B.dsattn_plan(clip_len, n_clips, w, 160, h, D, list(range(0, 4 * G, 4)), device=-1,
                             window=r)
        i = B.dsattn_plan_launch_info(plan)
        plan.close()
        assert i["kernel"] == 1 and i["ring_reach"] == reach, (w, r, G, i)
        assert i["local_tiles"] == (16 + 2 * reach + 15) // 16
        # chunks are counted in 16-frame query tiles and cover the video exactly
        tiles = clip_len * n_clips // 16
        row_groups = 160 * h // i["heads_per_wave"]
        assert i["n_tasks"] == row_groups * -(-tiles // i["clips_per_task"])
    # the window radius (or, with none, the rest of the clip) must fit the on-chip ring
    for kw in (dict(window=17), dict(window=None), dict(window=9, n_global=129)):
        g = list(range(kw.get("n_global", 4)))
        plan = B.dsattn_plan(clip_len, n_clips, 8, 160, h, D, g, device=-1, window=kw["window"])
        assert B.dsattn_plan_launch_info(plan)["kernel"] == 0, kw
        plan.close()


def test_launch_info_carries_the_resolved_variant():
    # the kernel variant is looked up once, by dsattn_plan; dsattn_forward launches what the plan
    # holds.  Distinct shapes resolve to distinct variants, equal shapes to the same one.
    seen = {}
    for D, h, w, G, od in ((160, 8, 2, 16, B.DSATTN_BF16), (160, 8, 2, 16, B.DSATTN_F32),
                           (160, 8, 4, 64, B.DSATTN_BF16), (80, 8, 2, 16, B.DSATTN_BF16),
                           (40, 8, 2, 16, B.DSATTN_BF16), (40, 8, 4, 64, B.DSATTN_BF16)):
        ids = []
        for n_clips in (8, 144):
            plan = B.dsattn_plan(16, n_clips, w, 12, h, D, list(range(G)), out_dtype=od, device=-1)
            i = B.dsattn_plan_launch_info(plan)
            plan.close()
            assert i["kernel"] == 1 and i["variant"] >= 0
            ids.append(i["variant"])
        assert ids[0] == ids[1]
        assert ids[0] not in seen.values()
        seen[(D, h, w, G, od)] = ids[0]
    plan = B.dsattn_plan(16, 8, 2, 12, 8, 48, [0], device=-1)     # no variant for head_dim 48
    assert B.dsattn_plan_launch_info(plan)["variant"] == -1
    plan.close()


def test_planning_a_very_long_video_is_quick():
    import time
    t0 = time.perf_counter()
    plan = B.dsattn_plan(16, 1 << 20, 2, 1, 8, 160, [0, 5, 9], device=-1)   # 16.8 M frames
    i = B.dsattn_plan_launch_info(plan)
    plan.close()
    assert i["kernel"] == 1 and time.perf_counter() - t0 < 2.0


def test_wide_contexts_reach_the_matrix_core_kernel():
    # 16 context frames per side together with up to 64 global frames; 65 to 128 global frames
    # where eight global key tiles fit a wavefront's registers (not at head_dim 160 and 128)
    for D, h, w, G, kernel, tiles in (
            (160, 8, 16, 64, 1, (3, 4)), (80, 8, 16, 17, 1, (3, 4)), (40, 8, 9, 64, 1, (3, 4)),
            (80, 8, 4, 128, 1, (2, 8)), (40, 8, 16, 65, 1, (3, 8)), (40, 5, 4, 128, 1, (2, 8)),
            (96, 4, 16, 128, 1, (3, 8)), (64, 4, 8, 100, 1, (2, 8)), (32, 4, 16, 128, 1, (3, 8)),
            (128, 4, 0, 128, 0, None), (128, 4, 2, 64, 1, (2, 4)), (160, 8, 4, 65, 0, None),
            (40, 5, 16, 128, 0, None), (80, 8, 4, 129, 0, None)):
        plan = B.dsattn_plan(16, 12, w, 6, h, D, [j % 192 for j in range(G)], device=-1)
        i = B.dsattn_plan_launch_info(plan)
        plan.close()
        assert i["kernel"] == kernel, (D, h, w, G, i)
        if tiles:
            assert (i["local_tiles"], i["global_tiles"]) == tiles, (D, h, w, G, i)


def test_layer_entry_point_checks_its_arguments_on_the_host():
    lib = B.load()
    plan = B.dsattn_plan(16, 4, 2, 5, 8, 40, [0, 9], device=-1)
    need = B.dsattn_temporal_layer_workspace(plan)
    one = 64 * 5 * 320 * 2                                  # one [F, P, C] bf16 tensor
    assert need == 4 * ((one + 255) // 256 * 256)
    n = ctypes.c_size_t(0)
    assert lib.dsattn_temporal_layer_workspace(None, ctypes.byref(n)) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_layer_workspace(plan.handle, None) == B.DSATTN_EINVAL
    w = (ctypes.c_void_p * 4)(0x100000, 0x200000, 0x300000, 0x400000)
    args = lambda **kw: [kw.get("plan", plan.handle), kw.get("x", 0x1000000), kw.get("w", w), None,
                         kw.get("ws", 0x8000000), kw.get("n", need), kw.get("y", 0x4000000), None]
    assert lib.dsattn_temporal_layer(*args(plan=None)) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_layer(*args(x=None)) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_layer(*args(w=None)) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_layer(*args(ws=None)) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_layer(*args(y=None)) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_layer(*args()) == B.DSATTN_ENODEVICE      # host-only plan
    plan.close()
    # fp32 output of bf16 attention cannot feed the output projection
    plan = B.dsattn_plan(16, 4, 2, 5, 8, 40, [0, 9], out_dtype=B.DSATTN_F32, device=-1)
    assert lib.dsattn_temporal_layer(*args(plan=plan.handle)) == B.DSATTN_ENODEVICE
    plan.close()
