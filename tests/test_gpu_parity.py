"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Context indices and gathered context are bit-exact; attention outputs
are within 1e-5 (fp32 path) / 1e-2 (bf16 I/O, fp32 accumulation; see parity_util.assert_parity
for how bf16 output rounding is accounted)."""
import numpy as np
import pytest
import torch

import parity_util as U
from oracle import oracle
from paper_2406_16260_amd import binding as B
from paper_2406_16260_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def announce(msg):
    print(f"[case] {msg}", flush=True)


def make(F, P, C, seed, gen, dtype):
    return tuple(synth.make_tensor(F, P, C, seed + t, gen, dtype).to(DEV) for t in range(3))


# ---------------------------------------------------------------- C0: the tiny fp32 case

def test_c0_tiny_fp32():
    wl = synth.WORKLOADS["C0"]
    lv = wl.levels[0]
    g = synth.global_idx_for(wl)
    announce("C0 fp32 2x4 frames 4x4 1x8 w=1 G={0,4} scale=1/sqrt(8)")
    q, k, v = (t.to(DEV) for t in synth.make_qkv(wl, lv))
    o, info = U.library_forward(q, k, v, wl.clip_len, wl.n_clips, wl.local_ctx, lv.heads, g,
                                scale=1.0 / np.sqrt(8.0))
    ref = U.oracle_forward(q, k, v, wl.clip_len, wl.n_clips, wl.local_ctx, lv.heads, g,
                           scale=1.0 / np.sqrt(8.0))
    U.assert_parity(o, ref, "f32_strict", what="C0")
    assert info["kernel"] == 0  # fp32 runs the vector-ALU kernel


# ---------------------------------------------------------------- generic kernel, many shapes

GENERIC_SHAPES = [
    # clip_len, n_clips, w, P, heads, D, global, dtype
    (4, 3, 0, 5, 2, 5, [], "f32"),
    (3, 4, 2, 7, 2, 4, [11, 0, 5], "f32"),
    (2, 4, 5, 3, 1, 3, [7, 7, 1], "f32"),
    (5, 1, 3, 2, 1, 6, [2], "f32"),
    (16, 3, 8, 9, 2, 24, list(range(0, 48, 3)), "f32"),
    (7, 5, 3, 33, 3, 72, [0, 34, 17, 17], "f32"),       # D > 64: lanes stride over channels
    (16, 6, 2, 19, 4, 40, list(range(0, 96, 6)), "bf16"),
    (8, 10, 70, 3, 2, 16, list(range(80)), "bf16"),     # more than 64 keys: lanes stride over keys
    (2, 5, 1, 2, 2, 30, [9, 0], "f32"),                 # clip shorter than a workgroup's 4 wavefronts
    (5, 3, 2, 3, 1, 18, [1], "bf16"),                   # head_dim not a multiple of 4: scalar LDS reads
    # 112 keys x 512 channels do not fit in LDS as fp32: the plain kernel reads them from memory
    (16, 2, 16, 1, 1, 512, list(range(0, 32, 1)) + list(range(0, 32, 1)), "f32"),
    (16, 3, 4, 2, 1, 768, list(range(0, 48, 2)), "bf16"),
]


@pytest.mark.parametrize("shape", GENERIC_SHAPES)
def test_generic_kernel_matches_oracle(shape):
    clip_len, n_clips, w, P, h, D, g, dtype = shape
    announce(f"generic {shape[:6]} G={len(g)} {dtype}")
    F = clip_len * n_clips
    q, k, v = make(F, P, h * D, 17, "iid", dtype)
    for out_dtype in (["f32"] if dtype == "f32" else ["f32", "bf16"]):
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype=out_dtype,
                                    flags=B.DSATTN_FLAG_FORCE_GENERIC)
        assert info["kernel"] == 0
        ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g)
        U.assert_parity(o, ref, "f32_strict" if dtype == "f32" else out_dtype, what=str(shape))


# ---------------------------------------------------------------- gather: bit exact

@pytest.mark.parametrize("shape", [
    (4, 2, 1, 16, 8, [0, 4], "f32"),
    (16, 4, 2, 40, 320, list(range(0, 64, 4)), "bf16"),
    (3, 5, 4, 3, 5, [14, 2], "bf16"),      # slab of 30 bytes: element-wise path
    (2, 3, 0, 1, 3, [], "f32"),            # slab of 12 bytes
    (4, 3, 9, 6, 8, [], "bf16"),           # edge clips shorter than lk_max: zero-filled rows
])
def test_gather_context_bit_exact(shape):
    clip_len, n_clips, w, P, C, g, dtype = shape
    announce(f"gather {shape[:5]} G={len(g)} {dtype}")
    F = clip_len * n_clips
    k, v, _ = make(F, P, C, 3, "iid", dtype)
    plan = B.dsattn_plan(clip_len, n_clips, w, P, 1, C, g, io_dtype=U.dt_code(dtype), device=0)
    lk = B.dsattn_plan_ctx_max(plan)
    idx, ln = B.dsattn_plan_ctx_indices(plan)
    ridx, rln = oracle.ctx_indices(clip_len, n_clips, w, g)
    assert np.array_equal(idx, ridx) and np.array_equal(ln, rln)
    kc = torch.full((n_clips, lk, P, C), 7.0, dtype=k.dtype, device=DEV)
    vc = torch.full((n_clips, lk, P, C), 7.0, dtype=k.dtype, device=DEV)
    B.dsattn_gather_context(plan, k, v, kc, vc)
    torch.cuda.synchronize()
    as_bits = (lambda t: t.cpu().view(torch.int16).numpy()) if dtype == "bf16" else \
              (lambda t: t.cpu().view(torch.int32).numpy())
    for src, dst in ((k, kc), (v, vc)):
        ref = oracle.gather_context(as_bits(src), clip_len, n_clips, w, g)
        assert np.array_equal(as_bits(dst), ref)
    # one pair at a time is allowed
    kc2 = torch.zeros_like(kc)
    B.dsattn_gather_context(plan, k, None, kc2, None)
    torch.cuda.synchronize()
    assert torch.equal(kc2, kc)
    plan.close()


@pytest.mark.parametrize("D,h,P,w,G,opts", [
    (160, 2, 3, 2, 16, {}),                                   # the headline level's shape
    (160, 8, 2, 8, 16, {}),                                   # the paper's sizes
    (40, 8, 3, 4, 64, {}),                                    # four global key tiles, paired tiles
    (80, 2, 5, 0, 5, {"bias_global": 0.4}),                   # no boundary frames, partial global tile
    (64, 3, 2, 12, 0, {"window": 5}),                         # three local key tiles, no global part
    (128, 2, 2, 3, 40, {"flags": B.DSATTN_FLAG_DEDUP_GLOBAL}),  # set union needs the real indices
])
def test_forward_ctx_on_matrix_cores(D, h, P, w, G, opts):
    # the two-stage path of the paper (gather the context, then attend over it) through the MFMA
    # kernel: one clip per chunk reading its slab of the materialised context; same arithmetic
    # in the same order as the fused path, so the outputs are identical
    n_clips = 6
    F = 16 * n_clips
    g = np.random.default_rng(77 + G).integers(0, F, size=G).tolist()
    q, k, v = make(F, P, h * D, 31, "iid", "bf16")
    for od in ("f32", "bf16"):
        announce(f"forward_ctx mfma D={D} h={h} P={P} w={w} G={G} {opts} out={od}")
        with planner_env(4, None):
            plan = B.dsattn_plan(16, n_clips, w, P, h, D, g, io_dtype=B.DSATTN_BF16,
                                 out_dtype=U.dt_code(od), device=0, **opts)
        assert B.dsattn_plan_launch_info(plan)["kernel"] == 1
        lk = B.dsattn_plan_ctx_max(plan)
        kc = torch.empty((n_clips, lk, P, h * D), dtype=k.dtype, device=DEV)
        vc = torch.empty_like(kc)
        B.dsattn_gather_context(plan, k, v, kc, vc)
        o1 = torch.full((F, P, h * D), float("nan"), dtype=synth.torch_dtype(od), device=DEV)
        o2 = torch.full_like(o1, float("nan"))
        B.dsattn_forward(plan, q, k, v, o1)
        B.dsattn_forward_ctx(plan, q, kc, vc, o2)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2)
        plan.close()
    ref = U.oracle_forward(q, k, v, 16, n_clips, w, h, g, window=opts.get("window"),
                           bias_global=opts.get("bias_global", 0.0), dedup="flags" in opts)
    U.assert_parity(o2, ref, "bf16", what="forward_ctx mfma")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_ctx_equals_forward(dtype):
    clip_len, n_clips, w, P, h, D = 8, 4, 3, 11, 2, 16
    g = [31, 0, 9, 9]
    announce(f"forward_ctx {dtype}")
    F = clip_len * n_clips
    q, k, v = make(F, P, h * D, 29, "iid", dtype)
    plan = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, io_dtype=U.dt_code(dtype),
                         out_dtype=B.DSATTN_F32, flags=B.DSATTN_FLAG_FORCE_GENERIC, device=0)
    lk = B.dsattn_plan_ctx_max(plan)
    kc = torch.empty((n_clips, lk, P, h * D), dtype=k.dtype, device=DEV)
    vc = torch.empty_like(kc)
    B.dsattn_gather_context(plan, k, v, kc, vc)
    o1 = torch.empty((F, P, h * D), dtype=torch.float32, device=DEV)
    o2 = torch.empty_like(o1)
    B.dsattn_forward(plan, q, k, v, o1)
    B.dsattn_forward_ctx(plan, q, kc, vc, o2)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)   # same kernel, same order of operations
    ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g)
    U.assert_parity(o2, ref, "f32_strict" if dtype == "f32" else "f32", what="forward_ctx")
    plan.close()


def test_device_argument_checks():
    lib = B.load()
    plan = B.dsattn_plan(4, 2, 1, 16, 1, 8, [0, 4], io_dtype=B.DSATTN_F32, device=0)
    x = torch.zeros((8, 16, 8), device=DEV)
    o = torch.zeros_like(x)
    st = torch.cuda.current_stream().cuda_stream
    assert lib.dsattn_forward(plan.handle, x.data_ptr(), x.data_ptr(), x.data_ptr(),
                              x.data_ptr(), st) == B.DSATTN_EINVAL          # O aliases Q
    assert lib.dsattn_forward(plan.handle, x.data_ptr() + 4, x.data_ptr(), x.data_ptr(),
                              o.data_ptr(), st) == B.DSATTN_EINVAL          # misaligned
    assert lib.dsattn_forward(plan.handle, x.data_ptr(), x.data_ptr(), x.data_ptr(),
                              o.data_ptr(), st) == B.DSATTN_OK              # K may alias Q
    torch.cuda.synchronize()
    plan.close()


def test_copy_probe_copies():
    src = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    B.dsattn_copy_probe(dst, src, src.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


# ---------------------------------------------------------------- bf16 MFMA streaming kernel

planner_env = U.planner_env


def run_mfma_case(n_clips, w, P, h, D, g, gen="correlated", scale=0.0, clips_per_task=None,
                  waves_per_block=None, seed=41, out_dtypes=("f32", "bf16"), what=""):
    clip_len = 16
    F = clip_len * n_clips
    q, k, v = make(F, P, h * D, seed, gen, "bf16")
    ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, scale=scale)
    with planner_env(clips_per_task, waves_per_block):
        for od in out_dtypes:
            announce(f"mfma {what} N={n_clips} w={w} P={P} h={h} D={D} G={len(g)} {gen} "
                     f"scale={scale} M={clips_per_task} wpb={waves_per_block} out={od}")
            o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype=od,
                                        scale=scale)
            assert info["kernel"] == 1, f"planner did not pick the MFMA kernel: {info}"
            if clips_per_task is not None:
                assert info["clips_per_task"] == min(clips_per_task, n_clips)
            if waves_per_block is not None:
                assert info["block_threads"] == 64 * waves_per_block
            U.assert_parity(o, ref, od, what=what)
    return info


@pytest.mark.parametrize("m", [None, 1, 2, 4, 6])
def test_mfma_d160_chunking(m):
    # the headline level's shape on a short video: 6 clips, interior and both edge clips,
    # every way of cutting the clips into per-wavefront chunks
    run_mfma_case(6, 2, 5, 8, 160, synth.stride_global_idx(96, 16), clips_per_task=m,
                  what="d160 chunking")


@pytest.mark.parametrize("wpb", [1, 2, 4, 8])
def test_mfma_d160_waves_per_block(wpb):
    run_mfma_case(5, 2, 3, 8, 160, synth.stride_global_idx(80, 16), clips_per_task=2,
                  waves_per_block=wpb, what="d160 wpb")


@pytest.mark.parametrize("w,g", [
    (1, [0, 47, 20]),                       # partial global tile, unsorted
    (2, []),                                # no global context
    (8, list(range(0, 48, 3))),             # the paper's own setting: 8 + 8 neighbours, 16 global
    (5, [7, 7, 7, 30, 30, 1]),              # duplicates count twice
    (3, list(range(16))),                   # global set inside clip 0 (all duplicates of local)
    (0, [5, 40]),                           # no local context beyond the clip itself
    (0, []),                                # plain per-clip attention
    (12, [1]),                              # window of 40 frames: three local key tiles
    (16, list(range(0, 48, 4))),            # w = clip length
])
def test_mfma_d160_context_shapes(w, g):
    run_mfma_case(3, w, 3, 2, 160, g, gen="iid", clips_per_task=2, what=f"ctx w={w}")


def test_mfma_reduces_to_full_attention():
    # no global set and a window covering the whole video: every clip sees all frames
    info = run_mfma_case(2, 16, 2, 2, 160, [], gen="iid", what="full attention")
    assert info["local_tiles"] == 3


def test_mfma_d160_single_clip_and_tiny_grid():
    run_mfma_case(1, 2, 1, 1, 160, [3, 9], gen="iid", what="single clip")
    run_mfma_case(2, 4, 1, 1, 160, [31], gen="iid", clips_per_task=1, what="two clips")


def test_mfma_d160_peaked_softmax():
    # iid inputs with a 4x larger scale: near one-hot weights, large logits
    run_mfma_case(4, 2, 3, 2, 160, synth.stride_global_idx(64, 16), gen="iid",
                  scale=4.0 / np.sqrt(160.0), what="peaked")


@pytest.mark.parametrize("D,h,P", [(80, 8, 5), (80, 2, 3), (40, 8, 7), (40, 4, 2)])
@pytest.mark.parametrize("w,G", [(2, 16), (0, 0), (8, 5), (12, 16)])
def test_mfma_other_head_dims(D, h, P, w, G):
    # head_dim 80 runs two heads per wavefront, head_dim 40 four: padded contraction blocks
    g = synth.stride_global_idx(64, G) if G else []
    info = run_mfma_case(4, w, P, h, D, g, gen="iid", clips_per_task=3, what=f"D={D}")
    assert info["heads_per_wave"] == 160 // D


@pytest.mark.parametrize("D,h,P,hpw", [
    (128, 8, 3, 1), (128, 1, 2, 1), (96, 4, 3, 2), (96, 3, 2, 1), (64, 8, 5, 2), (64, 5, 2, 1),
    (32, 8, 3, 4), (32, 6, 3, 2), (32, 3, 5, 1), (40, 6, 3, 2), (40, 3, 2, 1), (80, 3, 3, 1)])
@pytest.mark.parametrize("w,G", [(2, 16), (0, 0), (8, 5), (12, 16)])
def test_mfma_head_dim_family(D, h, P, hpw, w, G):
    # head dims whose contraction blocks and output tiles are whole (32, 64, 96, 128), and head
    # counts that the widest rows do not divide: narrower rows, down to one head per wavefront
    g = synth.stride_global_idx(64, G) if G else []
    info = run_mfma_case(4, w, P, h, D, g, gen="iid", clips_per_task=3, out_dtypes=("bf16",),
                         what=f"D={D} h={h}")
    assert info["heads_per_wave"] == hpw


@pytest.mark.parametrize("D,h,P", [(128, 2, 3), (96, 2, 2), (64, 4, 3), (32, 8, 2), (32, 3, 2),
                                   (40, 3, 2)])
@pytest.mark.parametrize("w,G", [(4, 64), (0, 17)])
def test_mfma_head_dim_family_many_global_frames(D, h, P, w, G):
    g = synth.random_sorted_global_idx(80, G, seed=5)
    info = run_mfma_case(5, w, P, h, D, g, gen="iid", clips_per_task=2, what=f"G={G} D={D}")
    assert info["global_tiles"] == 4


@pytest.mark.parametrize("D,h,P", [(160, 8, 3), (80, 8, 3), (40, 8, 3), (160, 1, 2)])
@pytest.mark.parametrize("w,G", [(4, 64), (2, 33), (0, 17), (8, 48)])
def test_mfma_many_global_frames(D, h, P, w, G):
    # 17..64 global frames: four global key tiles in registers, one wavefront per SIMD
    g = synth.random_sorted_global_idx(80, G, seed=3)
    info = run_mfma_case(5, w, P, h, D, g, gen="iid", clips_per_task=2, what=f"G={G} D={D}")
    assert info["global_tiles"] == 4


@pytest.mark.parametrize("w,D,h,G", [
    (w, D, h, G)
    for (D, h, G) in [(160, 2, 16), (40, 4, 16), (80, 2, 64), (40, 2, 64), (64, 2, 0)]
    for w in [1, 3, 5, 6, 7, 8, 9, 11, 13, 16]
    if G <= 16 or w <= 8])  # 64 global frames run on the matrix cores with w <= 8 only
def test_mfma_interior_clips_every_local_width(w, D, h, G):
    # 7 clips of which 5 are interior (for w <= 16): full global key tiles and no options, so the
    # interior clips take the softmax path without per-score masks; ring rows past 16 + 2w are
    # cleared after rounding, per packed pair of keys, in every local key tile after the first
    g = synth.random_sorted_global_idx(112, G, seed=11) if G else []
    run_mfma_case(7, w, 2, h, D, g, gen="iid", clips_per_task=4, out_dtypes=("f32",),
                  what=f"interior w={w} D={D} G={G}")


def test_mfma_odd_row_group_count():
    # 3 positions x 2 heads = 6 row groups: workgroups of 2 wavefronts, not 8
    info = run_mfma_case(3, 2, 3, 2, 160, [0, 9], what="odd rows")
    assert info["block_threads"] == 128
    info = run_mfma_case(3, 2, 5, 1, 160, [0, 9], what="prime rows")
    assert info["block_threads"] == 64


def test_mfma_matches_generic_kernel_on_device():
    # two independent device kernels agree (fp32 outputs), beyond both matching the oracle
    clip_len, n_clips, w, P, h, D = 16, 5, 2, 7, 8, 160
    g = synth.stride_global_idx(80, 16)
    q, k, v = make(80, P, h * D, 5, "correlated", "bf16")
    o1, i1 = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype="f32")
    o2, i2 = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype="f32",
                               flags=B.DSATTN_FLAG_FORCE_GENERIC)
    assert i1["kernel"] == 1 and i2["kernel"] == 0
    assert (o1 - o2).abs().max().item() < 5e-3


def test_mfma_is_deterministic():
    clip_len, n_clips, w, P, h, D = 16, 4, 2, 6, 8, 160
    g = synth.stride_global_idx(64, 16)
    q, k, v = make(64, P, h * D, 9, "correlated", "bf16")
    o1, _ = U.library_forward(q, k, v, clip_len, n_clips, w, h, g)
    o2, _ = U.library_forward(q, k, v, clip_len, n_clips, w, h, g)
    assert torch.equal(o1, o2)


def test_mfma_locality_and_permutation_on_device():
    # frames outside a clip's list cannot change its output (bit for bit); permuting the
    # global set changes nothing beyond rounding order
    clip_len, n_clips, w, P, h, D = 16, 4, 2, 3, 2, 160
    g = [0, 40, 63, 17]
    q, k, v = make(64, P, h * D, 13, "iid", "bf16")
    base, _ = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype="f32")
    k2, v2 = k.clone(), v.clone()
    k2[30] += 3.0   # frame 30 belongs to clip 1 and (w = 2) to clip 2's c_pre: not to clips 0, 3
    v2[30] -= 3.0
    o, _ = U.library_forward(q, k2, v2, clip_len, n_clips, w, h, g, out_dtype="f32")
    assert torch.equal(o[:16], base[:16]) and torch.equal(o[48:], base[48:])
    assert (o[16:48] - base[16:48]).abs().max().item() > 1e-3
    operm, _ = U.library_forward(q, k, v, clip_len, n_clips, w, h, [17, 63, 0, 40], out_dtype="f32")
    assert (operm - base).abs().max().item() < 2e-3


# ---------------------------------------------------------------- scope weights (Section 5.1)

@pytest.mark.parametrize("bl,bg", [(0.0, 2.302585), (2.302585, 0.0), (1.5, 1.5), (-3.0, 4.0)])
def test_scope_biases_both_kernels(bl, bg):
    # the weight of the global or of the local scope raised, e.g. by ln 10 (a tenfold weight)
    clip_len, n_clips, w, P, h, D = 16, 4, 2, 3, 2, 160
    g = synth.stride_global_idx(64, 16)
    q, k, v = make(64, P, h * D, 23, "iid", "bf16")
    ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, bias_local=bl, bias_global=bg)
    plain = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g)
    if bl != bg:
        assert np.abs(ref - plain).max() > 1e-2   # the biases matter on these inputs
    for flags, kernel in ((0, 1), (B.DSATTN_FLAG_FORCE_GENERIC, 0)):
        announce(f"scope bias local={bl} global={bg} kernel={kernel}")
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype="f32",
                                    flags=flags, bias_local=bl, bias_global=bg)
        assert info["kernel"] == kernel
        U.assert_parity(o, ref, "f32", what=f"bias {bl},{bg} kernel {kernel}")


def test_scope_biases_fp32_and_many_globals():
    q, k, v = make(12, 5, 2 * 5, 3, "iid", "f32")
    ref = U.oracle_forward(q, k, v, 4, 3, 1, 2, [0, 7, 10], bias_local=0.4, bias_global=-1.1)
    o, _ = U.library_forward(q, k, v, 4, 3, 1, 2, [0, 7, 10], bias_local=0.4, bias_global=-1.1)
    U.assert_parity(o, ref, "f32_strict", what="bias fp32")
    g = synth.random_sorted_global_idx(80, 40, seed=5)
    q, k, v = make(80, 2, 8 * 40, 7, "iid", "bf16")
    ref = U.oracle_forward(q, k, v, 16, 5, 4, 8, g, bias_global=2.302585)
    o, info = U.library_forward(q, k, v, 16, 5, 4, 8, g, out_dtype="f32", bias_global=2.302585)
    assert info["kernel"] == 1 and info["global_tiles"] == 4
    U.assert_parity(o, ref, "f32", what="bias G=40 D=40")


# ---------------------------------------------------------------- sliding-window local scope (Section 4.2)

@pytest.mark.parametrize("w,r,G", [(8, 8, 16), (2, 1, 3), (4, 0, 0), (2, 30, 5), (3, 5, 64), (16, 12, 0)])
def test_sliding_window_both_kernels(w, r, G):
    clip_len, n_clips, P, h, D = 16, 4, 3, 2, 160
    g = synth.random_sorted_global_idx(64, G, seed=11).tolist() if G else []
    q, k, v = make(64, P, h * D, 31, "iid", "bf16")
    ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, window=r)
    if r < 16 + w - 1:
        plain = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g)
        assert np.abs(ref - plain).max() > 1e-2   # the window matters on these inputs
    for flags, kernel in ((0, 1), (B.DSATTN_FLAG_FORCE_GENERIC, 0)):
        announce(f"sliding window w={w} r={r} G={G} kernel={kernel}")
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype="f32",
                                    flags=flags, window=r, scale=2.0 / np.sqrt(160.0))
        ref2 = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, window=r,
                                scale=2.0 / np.sqrt(160.0))
        assert info["kernel"] == kernel
        U.assert_parity(o, ref2, "f32", what=f"window w={w} r={r} kernel {kernel}")


def test_sliding_window_partition_invariance_on_device():
    # with w >= r the clip partition cannot matter: 2 clips chunked differently, and the fp32
    # generic kernel with other clip lengths, all agree with banded attention over the video
    F, P, h, D, r = 64, 2, 2, 160, 5
    q, k, v = make(F, P, h * D, 37, "iid", "bf16")
    ref = U.oracle_forward(q, k, v, F, 1, 0, h, [], window=r)      # one clip = the whole video
    with planner_env(clips_per_task=1):
        o1, i1 = U.library_forward(q, k, v, 16, 4, 5, h, [], out_dtype="f32", window=r)
    with planner_env(clips_per_task=4):
        o2, i2 = U.library_forward(q, k, v, 16, 4, 8, h, [], out_dtype="f32", window=r)
    o3, i3 = U.library_forward(q, k, v, 8, 8, 6, h, [], out_dtype="f32", window=r)   # generic
    assert i1["kernel"] == 1 and i2["kernel"] == 1 and i3["kernel"] == 0
    for o in (o1, o2, o3):
        U.assert_parity(o, ref, "f32", what="window partition invariance")


def test_sliding_window_fp32_with_biases():
    q, k, v = make(24, 5, 2 * 6, 3, "iid", "f32")
    kw = dict(bias_local=0.3, bias_global=-0.7, window=2)
    ref = U.oracle_forward(q, k, v, 4, 6, 3, 2, [23, 0, 11], **kw)
    o, _ = U.library_forward(q, k, v, 4, 6, 3, 2, [23, 0, 11], **kw)
    U.assert_parity(o, ref, "f32_strict", what="window fp32")


# ---------------------------------------------------------------- streams, graphs, limits

def test_forward_on_side_stream_and_two_plans():
    clip_len, n_clips, w, P, h, D = 16, 4, 2, 6, 8, 160
    g = synth.stride_global_idx(64, 16)
    q, k, v = make(64, P, h * D, 51, "correlated", "bf16")
    ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g)
    p1 = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, device=0)
    p2 = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, out_dtype=B.DSATTN_F32, device=0)
    o1 = torch.empty_like(q)
    o2 = torch.empty(q.shape, dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.dsattn_forward(p1, q, k, v, o1, side)
    B.dsattn_forward(p2, q, k, v, o2)          # on the current stream, concurrently
    side.synchronize()
    torch.cuda.synchronize()
    U.assert_parity(o1, ref, "bf16", what="side stream")
    U.assert_parity(o2, ref, "f32", what="current stream")
    p1.close()
    p2.close()


def test_forward_in_hip_graph_replays():
    # dsattn_forward is one kernel launch and nothing else: it can be captured and replayed
    clip_len, n_clips, w, P, h, D = 16, 5, 2, 4, 8, 160
    g = synth.stride_global_idx(80, 16)
    q, k, v = make(80, P, h * D, 61, "correlated", "bf16")
    plan = B.dsattn_plan(clip_len, n_clips, w, P, h, D, g, device=0)
    eager = torch.empty_like(q)
    B.dsattn_forward(plan, q, k, v, eager)
    torch.cuda.synchronize()
    out = torch.zeros_like(q)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.dsattn_forward(plan, q, k, v, out)
    for rep in range(4):
        out.fill_(0)                           # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
    # new inputs in the same buffers are picked up by the next replay
    q2, k2, v2 = make(80, P, h * D, 62, "correlated", "bf16")
    q.copy_(q2)
    k.copy_(k2)
    v.copy_(v2)
    B.dsattn_forward(plan, q, k, v, eager)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, eager)
    plan.close()


def test_generic_kernel_limit_is_reported():
    # a context list too long for the generic kernel's LDS is refused, not launched
    lib = B.load()
    F = 20000
    plan = B.dsattn_plan(1, F, F, 1, 1, 8, [], io_dtype=B.DSATTN_F32, device=0)
    x = torch.zeros((F, 1, 8), device=DEV)
    o = torch.zeros_like(x)
    st = torch.cuda.current_stream().cuda_stream
    rc = lib.dsattn_forward(plan.handle, x.data_ptr(), x.data_ptr(), x.data_ptr(), o.data_ptr(), st)
    assert rc == B.DSATTN_EUNSUPPORTED and "generic" in B.dsattn_last_error()
    plan.close()


def test_randomised_shapes_against_oracle():
    # seeded sweep over shapes the planner sends to either kernel
    rng = np.random.default_rng(2024)
    for case in range(24):
        D = int(rng.choice([40, 80, 160, 24, 64, 128]))
        h = int(rng.choice([1, 2, 4, 8]))
        clip_len = 16 if D != 24 and rng.random() < 0.8 else int(rng.integers(1, 20))
        n_clips = int(rng.integers(1, 7))
        F = clip_len * n_clips
        w = int(rng.integers(0, 18))
        G = int(rng.choice([0, 1, 5, 16, 17, 40, 64]))
        g = rng.integers(0, F, size=G).tolist()
        P = int(rng.integers(1, 6))
        window = None if rng.random() < 0.6 else int(rng.integers(0, 12))
        bg = 0.0 if rng.random() < 0.6 else float(rng.normal())
        announce(f"random case {case}: D={D} h={h} Fc={clip_len} N={n_clips} w={w} G={G} P={P} "
                 f"window={window} bias_global={bg:.3f}")
        q, k, v = make(F, P, h * D, 1000 + case, "iid", "bf16")
        ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, window=window, bias_global=bg)
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype="f32",
                                    window=window, bias_global=bg)
        # MFMA variants: clips of whole 16-frame tiles, head_dim 32/40/64/80/96/128/160 with any
        # head count; the frames a tile's local scope reaches beyond the tile (the window radius,
        # at most the rest of the clip's local range) <= 16; up to 64 global frames (the sweep
        # draws no more)
        reach = clip_len - 16 + w
        reach = reach if window is None else min(window, reach)
        expect_mfma = clip_len % 16 == 0 and D != 24 and reach <= 16
        assert info["kernel"] == (1 if expect_mfma else 0), (info, case)
        U.assert_parity(o, ref, "f32", what=f"random case {case}")


# ---------------------------------------------------------------- set union of the two scopes (Section 4.2)

@pytest.mark.parametrize("w,window,g", [
    (2, None, [0, 20, 20, 47, 33, 0]),          # repeats inside G, entries inside several clips' ranges
    (8, None, list(range(0, 64, 4))),           # the paper's sizes: every clip holds some global frames
    (4, 2, [5, 17, 18, 40, 63]),                # per query under the sliding window
    (0, None, [3]),
    (2, 0, list(range(16))),                    # window of the query frame only
])
def test_dedup_global_both_kernels(w, window, g):
    clip_len, n_clips, P, h, D = 16, 4, 3, 2, 160
    F = clip_len * n_clips
    q, k, v = make(F, P, h * D, 88, "iid", "bf16")
    ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, window=window, dedup=True)
    cat = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, window=window)
    assert np.abs(ref - cat).max() > 1e-2        # the option matters on these inputs
    for flags, kernel in ((B.DSATTN_FLAG_DEDUP_GLOBAL, 1),
                          (B.DSATTN_FLAG_DEDUP_GLOBAL | B.DSATTN_FLAG_FORCE_GENERIC, 0)):
        announce(f"dedup w={w} window={window} G={len(g)} kernel={kernel}")
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype="f32", flags=flags,
                                    window=window)
        assert info["kernel"] == kernel
        U.assert_parity(o, ref, "f32", what=f"dedup kernel {kernel}")


def test_dedup_global_other_shapes():
    # fp32 tensors (generic kernel), head_dim 40 with four heads per wavefront, and more than 16
    # global frames (the option then runs on the generic kernel)
    q, k, v = make(12, 2, 16, 89, "iid", "f32")
    g = [1, 1, 7, 11]
    ref = U.oracle_forward(q, k, v, 4, 3, 1, 2, g, dedup=True)
    o, _ = U.library_forward(q, k, v, 4, 3, 1, 2, g, flags=B.DSATTN_FLAG_DEDUP_GLOBAL)
    U.assert_parity(o, ref, "f32_strict", what="dedup fp32")
    q, k, v = make(48, 3, 8 * 40, 90, "iid", "bf16")
    g = [0, 9, 9, 30, 47]
    ref = U.oracle_forward(q, k, v, 16, 3, 3, 8, g, dedup=True, bias_global=0.7)
    o, info = U.library_forward(q, k, v, 16, 3, 3, 8, g, out_dtype="f32", flags=B.DSATTN_FLAG_DEDUP_GLOBAL,
                                bias_global=0.7)
    assert info["kernel"] == 1 and info["heads_per_wave"] == 4
    U.assert_parity(o, ref, "f32", what="dedup D=40")
    g = sorted(set(range(0, 48, 2)))  # 24 global frames
    ref = U.oracle_forward(q, k, v, 16, 3, 3, 8, g, dedup=True)
    o, info = U.library_forward(q, k, v, 16, 3, 3, 8, g, out_dtype="f32", flags=B.DSATTN_FLAG_DEDUP_GLOBAL)
    assert info["kernel"] == 0
    U.assert_parity(o, ref, "f32", what="dedup G=24")


@pytest.mark.parametrize("D,h", [(160, 2), (128, 3)])
@pytest.mark.parametrize("w,window,G", [(4, None, 64), (2, None, 17), (8, 3, 40), (0, None, 33), (4, 0, 64)])
def test_dedup_global_many_global_frames_on_matrix_cores(D, h, w, window, G):
    # 17..64 global frames with the set union: head_dim 160 and 128 keep it on the matrix cores
    # (one wavefront per SIMD); entries repeat each other and lie inside several clips' ranges
    n_clips = 5
    rng = np.random.default_rng(100 + G)
    g = rng.integers(0, 16 * n_clips, size=G).tolist()
    q, k, v = make(16 * n_clips, 2, h * D, 93, "iid", "bf16")
    ref = U.oracle_forward(q, k, v, 16, n_clips, w, h, g, window=window, dedup=True, bias_global=-0.3)
    with planner_env(2, None):
        o, info = U.library_forward(q, k, v, 16, n_clips, w, h, g, out_dtype="f32", window=window,
                                    flags=B.DSATTN_FLAG_DEDUP_GLOBAL, bias_global=-0.3)
    assert info["kernel"] == 1 and info["global_tiles"] == 4
    U.assert_parity(o, ref, "f32", what=f"dedup D={D} G={G} w={w} window={window}")


# ---------------------------------------------------------------- accumulator chains of O^T and the denominator

@pytest.mark.parametrize("D,h", [(40, 4), (80, 2), (160, 2)])
@pytest.mark.parametrize("w,G,tiles,pairs", [
    (4, 64, (2, 4), True),     # even / even: key tiles enter in pairs (16x16x32)
    (4, 0, (2, 0), True),      # even / none
    (0, 64, (1, 4), False),    # odd local tiles with an even number of global ones: single tiles
    (12, 0, (3, 0), False),    # odd / none
    (2, 16, (2, 1), False),    # even local tiles with an odd number of global ones
    (0, 7, (1, 1), False),     # odd / odd
])
def test_accumulator_chain_families(D, h, w, G, tiles, pairs):
    """Both sides of the rule that decides whether a variant feeds its key tiles to O^T = V^T P^T
    in pairs or one by one (a chain never mixes the two instructions), at the three head sizes of
    the base model: each family against the oracle, strict fp32-output bar, peaked softmax so
    that single weights matter."""
    clip_len, n_clips, P = 16, 5, 3
    F = clip_len * n_clips
    g = synth.random_sorted_global_idx(F, G, seed=3).tolist() if G else []
    q, k, v = make(F, P, h * D, 900 + D + w + G, "iid", "bf16")
    announce(f"chain family D={D} tiles={tiles} pairs={pairs}")
    for scale in (0.0, 3.0 / np.sqrt(D)):
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype="f32",
                                    scale=scale)
        assert info["kernel"] == 1
        assert (info["local_tiles"], info["global_tiles"]) == tiles
        assert (tiles[0] % 2 == 0 and tiles[1] % 2 == 0) == pairs
        ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, scale=scale)
        U.assert_parity(o, ref, "f32", what=f"chain family D={D} {tiles}")


# ---------------------------------------------------------------- wide contexts: 16 local frames with 17..64 global, 65..128 global

@pytest.mark.parametrize("D,h,w,G,tiles", [
    (160, 2, 16, 64, (3, 4)), (160, 2, 9, 17, (3, 4)), (80, 4, 12, 40, (3, 4)), (40, 8, 16, 64, (3, 4)),
    (40, 3, 10, 33, (3, 4)), (128, 2, 16, 64, (3, 4)), (96, 2, 16, 20, (3, 4)), (64, 2, 11, 64, (3, 4)),
    (32, 4, 16, 64, (3, 4)),
    # 65 to 128 global frames: eight global key tiles
    (80, 4, 4, 128, (2, 8)), (80, 2, 16, 100, (3, 8)), (40, 8, 4, 128, (2, 8)), (40, 3, 2, 65, (2, 8)),
    (96, 2, 8, 128, (2, 8)), (64, 2, 16, 128, (3, 8)), (32, 4, 0, 90, (1, 8)),
])
def test_wide_contexts_on_matrix_cores(D, h, w, G, tiles):
    clip_len, n_clips, P = 16, 10, 3
    F = clip_len * n_clips
    g = np.random.default_rng(G + D).integers(0, F, size=G).tolist()   # repeats allowed
    q, k, v = make(F, P, h * D, 1200 + D + w + G, "iid", "bf16")
    announce(f"wide context D={D} h={h} w={w} G={G}")
    for od, scale in (("f32", 0.0), ("bf16", 2.0 / np.sqrt(D))):
        o, info = U.library_forward(q, k, v, clip_len, n_clips, w, h, g, out_dtype=od, scale=scale)
        assert info["kernel"] == 1 and (info["local_tiles"], info["global_tiles"]) == tiles, info
        ref = U.oracle_forward(q, k, v, clip_len, n_clips, w, h, g, scale=scale)
        U.assert_parity(o, ref, od, what=f"wide context D={D} w={w} G={G}")


def test_contexts_beyond_the_matrix_core_variants_run_the_generic_kernel():
    q, k, v = make(64, 2, 2 * 160, 1300, "iid", "bf16")
    for D, h, w, G in ((160, 2, 4, 65), (128, 2, 4, 70), (80, 4, 4, 129)):
        g = list(range(G % 64)) + list(range(64)) + ([5] * (G - 64 - G % 64) if G > 64 + G % 64 else [])
        g = (g + [0] * G)[:G]
        o, info = U.library_forward(q, k, v, 16, 4, w, h, g, out_dtype="f32")
        assert info["kernel"] == 0, (D, G, info)
        ref = U.oracle_forward(q, k, v, 16, 4, w, h, g)
        U.assert_parity(o, ref, "f32", what=f"generic D={D} G={G}")
    # the set union with more than 64 global frames
    g = list(range(64)) + list(range(30))
    o, info = U.library_forward(q, k, v, 16, 4, 2, 4, g, out_dtype="f32",
                                flags=B.DSATTN_FLAG_DEDUP_GLOBAL)
    assert info["kernel"] == 0
    ref = U.oracle_forward(q, k, v, 16, 4, 2, 4, g, dedup=True)
    U.assert_parity(o, ref, "f32", what="dedup G=94")
