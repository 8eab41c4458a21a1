"""Clip-parallel temporal convolution (Section 4.2, "Convolution module"): boundary checks and the
tile chooser on the CPU, parity of the HIP kernels against the oracle on the GPU."""
import ctypes

import numpy as np
import pytest
import torch

import parity_util as U
from oracle import oracle
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth

DEV = "cuda:0"

# fp32 accumulation of up to a few thousand bf16 x bf16 products (exact in fp32) into outputs of
# unit variance: observed errors are ~1e-5; the bar leaves a factor of ten
TOL_ACC = 1e-4


# ---------------------------------------------------------------- CPU: validation and tile choice

def raw_desc(**kw):
    d = dict(clip_len=16, n_clips=3, spatial=5, c_in=64, c_out=64, reach=1, io_dtype=B.DSATTN_BF16,
             out_dtype=B.DSATTN_BF16, flags=0)
    d.update(kw)
    return B.DsattnConvDesc(**d)


@pytest.mark.parametrize("kw", [
    dict(clip_len=0), dict(n_clips=0), dict(spatial=0), dict(c_in=0), dict(c_out=0),
    dict(reach=-1), dict(reach=17), dict(io_dtype=2), dict(out_dtype=7), dict(flags=4),
    dict(io_dtype=B.DSATTN_F32, out_dtype=B.DSATTN_BF16),
])
def test_conv_rejects_bad_descriptors(kw):
    lib = B.load()
    d = raw_desc(**kw)
    info = B.DsattnConvInfo()
    assert lib.dsattn_temporal_conv_info(ctypes.byref(d), ctypes.byref(info)) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_conv(ctypes.byref(d), 0x1000, 0x2000, None, 0x100000, None) == \
        B.DSATTN_EINVAL


def test_conv_argument_checks_before_launch():
    lib = B.load()
    d = raw_desc()
    info = B.DsattnConvInfo()
    assert lib.dsattn_temporal_conv_info(None, ctypes.byref(info)) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_conv_info(ctypes.byref(d), None) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_conv(ctypes.byref(d), None, 0x2000, None, 0x100000, None) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_conv(ctypes.byref(d), 0x1000, None, None, 0x100000, None) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_conv(ctypes.byref(d), 0x1000, 0x2000, None, None, None) == B.DSATTN_EINVAL
    assert lib.dsattn_temporal_conv(ctypes.byref(d), 0x1008, 0x2000, None, 0x100000, None) == B.DSATTN_EINVAL
    assert "aligned" in B.dsattn_last_error()
    assert lib.dsattn_temporal_conv(ctypes.byref(d), 0x1000, 0x2000, 0x3002, 0x100000, None) == B.DSATTN_EINVAL
    # X is 48 * 5 * 64 * 2 = 30,720 bytes: an output starting inside it is refused
    assert lib.dsattn_temporal_conv(ctypes.byref(d), 0x10000, 0x2000, None, 0x10000 + 30704, None) == \
        B.DSATTN_EINVAL
    assert "overlaps" in B.dsattn_last_error()
    assert lib.dsattn_temporal_conv(ctypes.byref(d), 0x10000, 0x2000, None, 0x10000, None) == B.DSATTN_EINVAL


def test_conv_info_tiles_and_counts():
    # the headline level's shape: 2,304 frames x 160 positions, 1,280 -> 1,280 channels, 3 taps
    i = B.dsattn_temporal_conv_info(16, 144, 160, 1280, 1280, 1)
    M = 2304 * 160
    assert i["kernel"] == 1 and i["block_threads"] in (256, 512) and i["tile_k"] == 64
    assert 1280 % i["tile_n"] == 0 and M % i["tile_m"] == 0          # no padded area at this shape
    tiles = (M // i["tile_m"]) * (1280 // i["tile_n"])
    assert tiles <= i["n_blocks"] < tiles + 8 and i["n_blocks"] % 8 == 0
    assert 2 * (i["tile_m"] + i["tile_n"]) * 128 <= i["lds_bytes"] <= 160 * 1024
    # frames 0 and F-1 each lose one tap
    assert i["useful_flops"] == 2 * (3 * 2304 - 2) * 160 * 1280 * 1280
    assert i["algorithmic_bytes"] == 2 * (M * 1280 * 2) + 3 * 1280 * 1280 * 2
    # 320 and 640 output channels take the 320-wide tile (no wasted columns)
    assert B.dsattn_temporal_conv_info(16, 4, 2560, 320, 320, 1)["tile_n"] == 320
    assert B.dsattn_temporal_conv_info(16, 24, 640, 640, 640, 1)["tile_n"] == 320
    assert B.dsattn_temporal_conv_info(16, 24, 640, 640, 512, 1)["tile_n"] == 256
    # no taps beyond the centre: one tap, nothing lost at the ends
    assert B.dsattn_temporal_conv_info(4, 2, 3, 8, 8, 0)["useful_flops"] == 2 * 8 * 3 * 8 * 8
    assert B.dsattn_temporal_conv_info(4, 2, 3, 8, 8, 2)["useful_flops"] == 2 * (5 * 8 - 6) * 3 * 8 * 8
    # fp32 tensors, channel counts that are not whole 16-byte lanes, and the flag: vector kernel
    assert B.dsattn_temporal_conv_info(16, 4, 5, 64, 64, 1, io_dtype=B.DSATTN_F32)["kernel"] == 0
    assert B.dsattn_temporal_conv_info(16, 4, 5, 36, 64, 1)["kernel"] == 0
    assert B.dsattn_temporal_conv_info(16, 4, 5, 64, 64, 1,
                                       flags=B.DSATTN_FLAG_FORCE_GENERIC)["kernel"] == 0
    assert B.dsattn_temporal_conv_info(16, 4, 5, 40, 7, 1)["kernel"] == 1


# ---------------------------------------------------------------- GPU: parity

def announce(msg):
    print(f"[case] {msg}", flush=True)


def run_conv(x, w, b, clip_len, n_clips, out_dtype, flags=0):
    F, P, c_in = x.shape
    taps, c_out, _ = w.shape
    io = "f32" if x.dtype == torch.float32 else "bf16"
    y = torch.full((F, P, c_out), float("nan"), dtype=synth.torch_dtype(out_dtype), device=x.device)
    B.dsattn_temporal_conv(clip_len, n_clips, P, c_in, c_out, taps // 2, x, w, y, bias=b,
                           io_dtype=U.dt_code(io), out_dtype=U.dt_code(out_dtype), flags=flags)
    torch.cuda.synchronize()
    return y


def check_conv(y, ref, out_dtype, what):
    got = y.to("cpu").to(torch.float64).numpy()
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    scale = np.maximum(1.0, np.abs(ref))
    if out_dtype == "f32":
        allow = TOL_ACC * scale
    else:  # the result within TOL_ACC, then one rounding to bf16
        allow = TOL_ACC * scale + U.bf16_half_ulp(np.maximum(np.abs(ref), np.abs(got)))
    bad = err > allow
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements beyond the bar, max-abs {err.max():.3e} "
                           f"at |ref| {np.abs(ref[bad]).max():.3f}")
    return float(err.max())


def conv_case(clip_len, n_clips, P, c_in, c_out, n, dtype="bf16", out_dtypes=("f32", "bf16"),
              bias=True, gen="correlated", seed=70, flags=0, expect_kernel=None):
    F = clip_len * n_clips
    x = synth.make_tensor(F, P, c_in, seed, gen, dtype).to(DEV)
    w, b = synth.make_conv_weights(2 * n + 1, c_out, c_in, seed + 1, dtype)
    w, b = w.to(DEV), (b.to(DEV) if bias else None)
    ref = oracle.temporal_conv(x.to("cpu").to(torch.float64).numpy(),
                               w.to("cpu").to(torch.float64).numpy(), clip_len, n_clips,
                               bias=None if b is None else b.to("cpu").to(torch.float64).numpy())
    info = B.dsattn_temporal_conv_info(clip_len, n_clips, P, c_in, c_out, n,
                                       io_dtype=U.dt_code(dtype), flags=flags)
    if expect_kernel is not None:
        assert info["kernel"] == expect_kernel, info
    for od in out_dtypes:
        if dtype == "f32" and od != "f32":
            continue
        announce(f"conv Fc={clip_len} N={n_clips} P={P} cin={c_in} cout={c_out} n={n} {dtype}->{od} "
                 f"bias={bias} kernel={info['kernel']} tile={info['tile_m']}x{info['tile_n']}")
        y = run_conv(x, w, b, clip_len, n_clips, od, flags=flags)
        check_conv(y, ref, od, f"conv {c_in}->{c_out} n={n} {od}")
    return info


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [
    # clip_len, n_clips, P, c_in, c_out, n
    (16, 3, 5, 64, 64, 1),          # one partly filled tile, one step per tap
    (16, 4, 40, 128, 320, 1),       # 2,560 rows: ten row tiles of 256 or 13.3 of 192; 320-wide tile
    (16, 3, 7, 320, 256, 1),        # row tail (336 rows), 5 steps per tap
    (8, 5, 9, 72, 200, 2),          # c_in not a multiple of 64 (zero-filled chunks), column tail, 5 taps
    (16, 2, 3, 1280, 1280, 1),      # the headline level's channels on a short video
    (4, 6, 33, 40, 7, 4),           # reach = clip length, 7 output channels
    (16, 2, 160, 64, 640, 0),       # a single tap: a plain matrix product
    (2, 40, 50, 96, 96, 1),         # many short clips, frames cross tile borders at every offset
])
def test_conv_mfma_matches_oracle(shape):
    conv_case(*shape, expect_kernel=1)


@pytest.mark.gpu
def test_conv_mfma_without_bias_and_iid_inputs():
    conv_case(16, 3, 10, 192, 128, 1, bias=False, gen="iid", expect_kernel=1)


@pytest.mark.gpu
@pytest.mark.parametrize("shape,dtype", [
    ((4, 3, 5, 6, 7, 1), "f32"), ((16, 2, 3, 36, 20, 1), "bf16"), ((3, 5, 4, 8, 8, 3), "f32"),
    ((16, 2, 4, 64, 64, 1), "bf16"),
])
def test_conv_generic_matches_oracle(shape, dtype):
    conv_case(*shape, dtype=dtype, flags=B.DSATTN_FLAG_FORCE_GENERIC, expect_kernel=0)


@pytest.mark.gpu
def test_conv_kernels_agree_and_are_deterministic():
    F, P, c = 48, 12, 256
    x = synth.make_tensor(F, P, c, 5, "iid", "bf16").to(DEV)
    w, b = (t.to(DEV) for t in synth.make_conv_weights(3, c, c, 6, "bf16"))
    y1 = run_conv(x, w, b, 16, 3, "f32")
    y2 = run_conv(x, w, b, 16, 3, "f32")
    assert torch.equal(y1, y2)
    yg = run_conv(x, w, b, 16, 3, "f32", flags=B.DSATTN_FLAG_FORCE_GENERIC)
    assert float((y1 - yg).abs().max()) <= TOL_ACC
    # the clip partition cannot matter
    y3 = run_conv(x, w, b, 4, 12, "f32")
    assert torch.equal(y1, y3)


@pytest.mark.gpu
def test_conv_on_side_stream():
    F, P, c = 32, 6, 128
    x = synth.make_tensor(F, P, c, 9, "iid", "bf16").to(DEV)
    w, b = (t.to(DEV) for t in synth.make_conv_weights(3, c, c, 10, "bf16"))
    ref = run_conv(x, w, b, 16, 2, "bf16")
    s = torch.cuda.Stream()
    y = torch.zeros_like(ref)
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        B.dsattn_temporal_conv(16, 2, P, c, c, 1, x, w, y, bias=b, stream=s)
    s.synchronize()
    assert torch.equal(y, ref)


@pytest.mark.gpu
@pytest.mark.parametrize("name,n_pos", [("C3", 2), ("C2", 3), ("C1", 4)])
def test_conv_full_size_levels_sampled(name, n_pos):
    """The level shapes bench.py times (C -> C channels, 3 taps, bias, bf16), inputs generated on
    the device; the oracle runs on a sample of spatial positions over all frames (positions are
    independent of each other, so every sampled output is exact)."""
    wl = synth.WORKLOADS[name]
    lv = wl.levels[0]
    announce(f"conv full size {name} {lv.spatial} C={lv.C}")
    x = synth.make_tensor(wl.F, lv.P, lv.C, wl.seed, wl.generator, "bf16", device=DEV)
    w, b = synth.make_conv_weights(3, lv.C, lv.C, wl.seed + 50, "bf16", device=DEV)
    info = B.dsattn_temporal_conv_info(wl.clip_len, wl.n_clips, lv.P, lv.C, lv.C, 1)
    assert info["kernel"] == 1
    y = run_conv(x, w, b, wl.clip_len, wl.n_clips, "bf16")
    assert torch.isfinite(y.float()).all()
    pos = sorted({0, lv.P - 1, *(((np.arange(n_pos) * lv.P) // n_pos).tolist())})
    pidx = torch.as_tensor(pos, device=DEV)
    ref = oracle.temporal_conv(x.index_select(1, pidx).to("cpu").to(torch.float64).numpy(),
                               w.to("cpu").to(torch.float64).numpy(), wl.clip_len, wl.n_clips,
                               bias=b.to("cpu").to(torch.float64).numpy())
    check_conv(y.index_select(1, pidx), ref, "bf16", f"conv full size {name}")


# ---------------------------------------------------------------- linear projections (dsattn_linear)

def test_linear_rejects_bad_arguments():
    lib = B.load()
    info = B.DsattnConvInfo()

    def desc(**kw):
        d = dict(rows=100, c_in=64, c_out=64, n_out=3, io_dtype=B.DSATTN_BF16,
                 out_dtype=B.DSATTN_BF16, flags=0)
        d.update(kw)
        return B.DsattnLinearDesc(**d)
    for kw in (dict(rows=0), dict(rows=1 << 31), dict(c_in=0), dict(c_out=0), dict(n_out=0),
               dict(n_out=5), dict(io_dtype=9), dict(flags=2),
               dict(io_dtype=B.DSATTN_F32, out_dtype=B.DSATTN_BF16)):
        d = desc(**kw)
        assert lib.dsattn_linear_info(ctypes.byref(d), ctypes.byref(info)) == B.DSATTN_EINVAL, kw
    d = desc()
    vp3 = ctypes.c_void_p * 3
    w, y = vp3(0x100000, 0x200000, 0x300000), vp3(0x400000, 0x500000, 0x600000)
    assert lib.dsattn_linear(ctypes.byref(d), None, w, None, y, None) == B.DSATTN_EINVAL
    assert lib.dsattn_linear(ctypes.byref(d), 0x1000, None, None, y, None) == B.DSATTN_EINVAL
    assert lib.dsattn_linear(ctypes.byref(d), 0x1008, w, None, y, None) == B.DSATTN_EINVAL
    assert lib.dsattn_linear(ctypes.byref(d), 0x1000, vp3(0x100000, None, 0x300000), None, y,
                             None) == B.DSATTN_EINVAL
    # two outputs overlapping (100 rows x 64 channels x 2 bytes = 12,800 bytes each)
    assert lib.dsattn_linear(ctypes.byref(d), 0x1000, w, None, vp3(0x400000, 0x400000 + 12784, 0x600000),
                             None) == B.DSATTN_EINVAL
    assert "overlap" in B.dsattn_last_error()
    # an output overlapping the input
    assert lib.dsattn_linear(ctypes.byref(d), 0x400000, w, None, y, None) == B.DSATTN_EINVAL


def test_linear_info_counts():
    # Q, K, V of the headline level in one launch: 15 column tiles per row tile
    i = B.dsattn_linear_info(2304 * 160, 1280, 1280, 3)
    assert i["kernel"] == 1 and i["tile_n"] in (256, 320)
    tiles = (2304 * 160 // i["tile_m"]) * (1280 // i["tile_n"]) * 3
    assert tiles <= i["n_blocks"] < tiles + 8
    assert i["useful_flops"] == 2 * 2304 * 160 * 1280 * 1280 * 3
    assert i["algorithmic_bytes"] == 2304 * 160 * 1280 * 2 * 4 + 3 * 1280 * 1280 * 2
    assert B.dsattn_linear_info(100, 64, 64, 1, io_dtype=B.DSATTN_F32)["kernel"] == 0


def linear_case(rows, c_in, c_out, n_out, dtype="bf16", out_dtype="bf16", flags=0, bias=True, seed=90):
    x = synth.make_tensor(rows, 1, c_in, seed, "iid", dtype).to(DEV).reshape(rows, c_in)
    ws, bs = [], []
    for k in range(n_out):
        w, b = synth.make_conv_weights(1, c_out, c_in, seed + 1 + k, dtype)
        ws.append(w.reshape(c_out, c_in).to(DEV))
        bs.append(b.to(DEV) if bias and k != 1 else None)   # the second set goes without a bias
    ys = [torch.full((rows, c_out), float("nan"), dtype=synth.torch_dtype(out_dtype), device=DEV)
          for _ in range(n_out)]
    info = B.dsattn_linear_info(rows, c_in, c_out, n_out, io_dtype=U.dt_code(dtype),
                                out_dtype=U.dt_code(out_dtype), flags=flags)
    announce(f"linear rows={rows} {c_in}->{c_out} x{n_out} {dtype}->{out_dtype} kernel={info['kernel']} "
             f"tile={info['tile_m']}x{info['tile_n']}")
    B.dsattn_linear(rows, c_in, c_out, x, ws, ys, biases=bs if bias else None,
                    io_dtype=U.dt_code(dtype), out_dtype=U.dt_code(out_dtype), flags=flags)
    torch.cuda.synchronize()
    xn = x.to("cpu").to(torch.float64).numpy()
    for k in range(n_out):
        ref = oracle.linear(xn, ws[k].to("cpu").to(torch.float64).numpy(),
                            bias=None if bs[k] is None else bs[k].to("cpu").to(torch.float64).numpy())
        check_conv(ys[k], ref, out_dtype, f"linear set {k}")
    return info


@pytest.mark.gpu
@pytest.mark.parametrize("rows,c_in,c_out,n_out", [
    (700, 128, 256, 3),      # Q, K, V: a row tail, one column tile per set
    (513, 320, 320, 3),      # the 320-wide tile
    (300, 72, 200, 2),       # channel and column tails
    (1000, 1280, 1280, 1),   # the output projection of the headline level
    (64, 64, 40, 4),
])
def test_linear_mfma_matches_oracle(rows, c_in, c_out, n_out):
    info = linear_case(rows, c_in, c_out, n_out)
    assert info["kernel"] == 1


@pytest.mark.gpu
def test_linear_other_paths_match_oracle():
    assert linear_case(50, 12, 9, 3, dtype="f32", out_dtype="f32")["kernel"] == 0
    assert linear_case(90, 64, 64, 2, flags=B.DSATTN_FLAG_FORCE_GENERIC)["kernel"] == 0
    assert linear_case(300, 128, 128, 3, out_dtype="f32", bias=False)["kernel"] == 1


@pytest.mark.gpu
def test_projected_qkv_feed_the_attention():
    """X -> (Q, K, V) in one launch -> Dual-scope attention, each stage against the oracle on the
    values the previous stage actually produced (bf16 tensors between the stages)."""
    clip_len, n_clips, w, P, h, D = 16, 3, 2, 3, 2, 160
    F, C = clip_len * n_clips, h * D
    x = synth.make_tensor(F, P, C, 31, "correlated", "bf16").to(DEV)
    ws = [synth.make_conv_weights(1, C, C, 32 + k, "bf16")[0].reshape(C, C).to(DEV) for k in range(3)]
    q, k, v = (torch.empty_like(x) for _ in range(3))
    B.dsattn_linear(F * P, C, C, x, ws, [q, k, v])
    torch.cuda.synchronize()
    xn = x.to("cpu").to(torch.float64).numpy()
    for t, wt in zip((q, k, v), ws):
        check_conv(t, oracle.linear(xn, wt.to("cpu").to(torch.float64).numpy()), "bf16", "projection")
    g = [0, 20, 47]
    o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g)
    assert info["kernel"] == 1
    U.assert_parity(o, U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g), "bf16", what="attention")


@pytest.mark.gpu
def test_whole_temporal_attention_layer_stage_by_stage():
    """The layer around the kernel, as four launches on one stream with nothing in between:
    X -> (Q, K, V) [one launch] -> Dual-scope attention -> output projection with bias.  Every
    stage is checked against the oracle on the bf16 tensors the previous stage produced, and the
    end result against the oracle chain run on its own roundings."""
    clip_len, n_clips, w, P, h, D = 16, 5, 2, 7, 8, 40
    F, C = clip_len * n_clips, h * D
    g = synth.stride_global_idx(F, 16).tolist()
    print(f"[case] layer chain {n_clips}x{clip_len} frames P={P} {h}x{D} w={w} G=16", flush=True)
    x = synth.make_tensor(F, P, C, 41, "correlated", "bf16").to(DEV)
    ws = [synth.make_conv_weights(1, C, C, 42 + k, "bf16")[0].reshape(C, C).to(DEV) for k in range(3)]
    wo, bo = synth.make_conv_weights(1, C, C, 46, "bf16")
    wo, bo = wo.reshape(C, C).to(DEV), bo.to(DEV)
    q, k, v, o, y = (torch.full_like(x, float("nan")) for _ in range(5))
    plan = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, io_dtype=B.DSATTN_BF16, device=0)
    assert B.dsattn_plan_launch_info(plan)["kernel"] == 1
    B.dsattn_linear(F * P, C, C, x, ws, [q, k, v])
    B.dsattn_forward(plan, q, k, v, o)
    B.dsattn_linear(F * P, C, C, o, [wo], [y], biases=[bo])
    torch.cuda.synchronize()
    plan.close()
    f64 = lambda t: t.to("cpu").to(torch.float64).numpy()
    for t, wt, name in zip((q, k, v), ws, "QKV"):
        check_conv(t, oracle.linear(f64(x), f64(wt)), "bf16", f"projection {name}")
    U.assert_parity(o, U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g), "bf16", what="attention")
    check_conv(y, oracle.linear(f64(o), f64(wo), bias=f64(bo)), "bf16", "output projection")
    # the oracle chained with itself, rounding to bf16 between its stages as the tensors do
    rb = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    qo, ko, vo = (rb(oracle.linear(f64(x), f64(wt))).reshape(F, P, h, D) for wt in ws)
    oo = rb(oracle.forward(qo, ko, vo, clip_len, n_clips, w, g).reshape(F, P, C))
    yo = oracle.linear(oo, f64(wo), bias=f64(bo))
    err = np.abs(f64(y) - yo)
    # three bf16 roundings along the way: a few bf16 ulps of the unit-scale values in between
    assert err.max() <= 4e-2, err.max()
    assert np.sqrt((err ** 2).mean()) <= 4e-3


@pytest.mark.gpu
@pytest.mark.parametrize("in_place,with_qkv_bias", [(False, False), (True, True)])
def test_layer_entry_point_equals_its_three_stages(in_place, with_qkv_bias):
    """dsattn_temporal_layer enqueues the same three launches as the separate calls: its result
    and the workspace's Q, K, V, A are bit-identical to theirs, and the result meets the oracle
    chain (with the oracle rounding to bf16 between its stages as the tensors do)."""
    clip_len, n_clips, w, P, h, D = 16, 4, 2, 9, 8, 40
    F, C = clip_len * n_clips, h * D
    g = synth.stride_global_idx(F, 16).tolist()
    print(f"[case] layer entry {n_clips}x{clip_len} frames P={P} {h}x{D} in_place={in_place}", flush=True)
    x = synth.make_tensor(F, P, C, 51, "correlated", "bf16").to(DEV)
    wb = [synth.make_conv_weights(1, C, C, 52 + k, "bf16") for k in range(4)]
    ws = [t[0].reshape(C, C).to(DEV) for t in wb]
    bs = [t[1].to(DEV) if (with_qkv_bias or k == 3) else None for k, t in enumerate(wb)]
    plan = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, io_dtype=B.DSATTN_BF16, device=0)
    # the separate calls
    q, k, v, o, y = (torch.full_like(x, float("nan")) for _ in range(5))
    B.dsattn_linear(F * P, C, C, x, ws[:3], [q, k, v], biases=bs[:3])
    B.dsattn_forward(plan, q, k, v, o)
    B.dsattn_linear(F * P, C, C, o, ws[3:], [y], biases=bs[3:])
    # the one call, on a workspace with a little slack in front of the needed bytes
    need = B.dsattn_temporal_layer_workspace(plan)
    assert need >= 4 * x.numel() * 2 and need % 256 == 0
    space = torch.full((need,), 0xFF, dtype=torch.uint8, device=DEV)
    x2 = x.clone()
    y2 = x2 if in_place else torch.full_like(x, float("nan"))
    B.dsattn_temporal_layer(plan, x2, ws, space, y2, biases=bs)
    torch.cuda.synchronize()
    assert torch.equal(y2, y)
    slab = need // 4
    for i, (t, name) in enumerate(zip((q, k, v, o), "QKVA")):
        got = space[i * slab: i * slab + t.numel() * 2].view(torch.bfloat16).reshape(t.shape)
        assert torch.equal(got, t), name
    # a short workspace, a misaligned one and one that overlaps Y are refused before any launch
    with pytest.raises(B.DsattnError, match="workspace"):
        B.dsattn_temporal_layer(plan, x, ws, space[: need - 256], y, biases=bs)
    big = torch.empty(need + 256, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.DsattnError, match="aligned"):
        B.dsattn_temporal_layer(plan, x, ws, big[16:], y, biases=bs)
    with pytest.raises(B.DsattnError, match="overlaps"):
        B.dsattn_temporal_layer(plan, x, ws, space, space[:x.numel() * 2].view(torch.bfloat16).reshape(x.shape),
                                biases=bs)
    plan.close()
    f64 = lambda t: None if t is None else t.to("cpu").to(torch.float64).numpy()
    rb = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    qo, ko, vo = (rb(oracle.linear(f64(x), f64(ws[i]), bias=f64(bs[i]))).reshape(F, P, h, D) for i in range(3))
    oo = rb(oracle.forward(qo, ko, vo, clip_len, n_clips, w, g).reshape(F, P, C))
    yo = oracle.linear(oo, f64(ws[3]), bias=f64(bs[3]))
    err = np.abs(f64(y2) - yo)
    assert err.max() <= 4e-2, err.max()
    assert np.sqrt((err ** 2).mean()) <= 4e-3


@pytest.mark.gpu
def test_layer_in_hip_graph_replays():
    """After one eager call the layer is three kernel launches and nothing else: captured once,
    every replay (with eager work and synchronisations in between) reproduces the eager result."""
    clip_len, n_clips, w, P, h, D = 16, 3, 2, 5, 4, 80
    F, C = clip_len * n_clips, h * D
    g = [1, 17, 40]
    print(f"[case] layer in a graph {n_clips}x{clip_len} frames P={P} {h}x{D}", flush=True)
    x = synth.make_tensor(F, P, C, 61, "correlated", "bf16").to(DEV)
    ws = [synth.make_conv_weights(1, C, C, 62 + k, "bf16")[0].reshape(C, C).to(DEV) for k in range(4)]
    plan = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, io_dtype=B.DSATTN_BF16, device=0)
    space = torch.zeros(B.dsattn_temporal_layer_workspace(plan), dtype=torch.uint8, device=DEV)
    y_eager = torch.empty_like(x)
    B.dsattn_temporal_layer(plan, x, ws, space, y_eager)
    torch.cuda.synchronize()
    y = torch.zeros_like(x)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.dsattn_temporal_layer(plan, x, ws, space, y)
    for rep in range(3):
        y.fill_(0)
        space.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager), f"replay {rep} differs from the eager result"
    plan.close()


def test_conv_falls_back_when_offsets_would_not_fit_32_bits():
    # the matrix-core kernel addresses a tile's X rows and all of W with 32-bit byte offsets
    assert B.dsattn_temporal_conv_info(16, 4, 40000, 1280, 64, 16)["kernel"] == 0   # reach x P rows x c_in
    assert B.dsattn_temporal_conv_info(16, 4, 4, 16384, 16384, 3)["kernel"] == 0    # W of 3.75 GB
    assert B.dsattn_temporal_conv_info(16, 4, 40000, 1280, 64, 1)["kernel"] == 1


@pytest.mark.gpu
def test_conv_and_linear_in_hip_graph_replays():
    """After one eager call on the device (which raises the kernel's LDS limit once), both entry
    points are a single kernel launch and can be captured and replayed."""
    F, P, c = 32, 6, 128
    x = synth.make_tensor(F, P, c, 15, "iid", "bf16").to(DEV)
    w, b = (t.to(DEV) for t in synth.make_conv_weights(3, c, c, 16, "bf16"))
    ws = [synth.make_conv_weights(1, c, c, 17 + k, "bf16")[0].reshape(c, c).to(DEV) for k in range(3)]
    y_eager = run_conv(x, w, b, 16, 2, "bf16")
    p_eager = [torch.empty_like(x) for _ in range(3)]
    B.dsattn_linear(F * P, c, c, x, ws, p_eager)
    torch.cuda.synchronize()
    y = torch.zeros_like(y_eager)
    ps = [torch.zeros_like(x) for _ in range(3)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.dsattn_temporal_conv(16, 2, P, c, c, 1, x, w, y, bias=b)
        B.dsattn_linear(F * P, c, c, x, ws, ps)
    for rep in range(3):
        y.fill_(0)                             # eager work between replays
        for t in ps:
            t.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager), f"replay {rep}: convolution differs from the eager result"
        for t, e in zip(ps, p_eager):
            assert torch.equal(t, e), f"replay {rep}: projection differs from the eager result"
