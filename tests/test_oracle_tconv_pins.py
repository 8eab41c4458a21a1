"""Pins of the temporal-convolution oracle (Section 4.2, "Convolution module"): the library
routine on the whole video (what clip parallelism must reproduce), closed forms that fix the
orientation of the taps and of the weight matrix, brute force, independence of the clip
partition, locality, and a planted-mistake check of the pins themselves."""
import numpy as np
import pytest
import torch

from oracle import oracle


def rand_case(F, P, c_in, c_out, n, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((F, P, c_in))
    w = rng.standard_normal((2 * n + 1, c_out, c_in))
    b = rng.standard_normal(c_out)
    return x, w, b


def library_conv(x, w, b):
    """torch's conv1d over the whole video per spatial position: [P, C_in, F] -> [P, C_out, F],
    zero padding n at both ends; torch's weight is [C_out, C_in, taps]."""
    n = w.shape[0] // 2
    t = torch.from_numpy(x).permute(1, 2, 0)
    wt = torch.from_numpy(w).permute(1, 2, 0).contiguous()
    y = torch.nn.functional.conv1d(t, wt, None if b is None else torch.from_numpy(b), padding=n)
    return y.permute(2, 0, 1).numpy()


@pytest.mark.parametrize("clip_len,n_clips,P,c_in,c_out,n", [
    (4, 3, 5, 6, 7, 1), (16, 2, 3, 8, 8, 1), (3, 5, 2, 4, 9, 3), (5, 4, 3, 5, 2, 2), (2, 6, 1, 3, 3, 0),
    (6, 1, 4, 4, 4, 2),
])
def test_matches_library_convolution_over_the_whole_video(clip_len, n_clips, P, c_in, c_out, n):
    x, w, b = rand_case(clip_len * n_clips, P, c_in, c_out, n, seed=clip_len * 100 + n)
    y = oracle.temporal_conv(x, w, clip_len, n_clips, bias=b)
    np.testing.assert_allclose(y, library_conv(x, w, b), rtol=0, atol=1e-12)
    y0 = oracle.temporal_conv(x, w, clip_len, n_clips)
    np.testing.assert_allclose(y0, library_conv(x, w, None), rtol=0, atol=1e-12)


def test_closed_forms_fix_tap_order_and_weight_orientation():
    F, P, C = 8, 2, 3
    x = np.random.default_rng(0).standard_normal((F, P, C))
    eye = np.eye(C)
    # centre tap = identity: the module returns its input (plus the bias)
    w = np.zeros((3, C, C))
    w[1] = eye
    b = np.array([1.0, -2.0, 0.5])
    np.testing.assert_array_equal(oracle.temporal_conv(x, w, 4, 2, bias=b), x + b)
    # tap 0 looks one frame back: output frame f is input frame f - 1, zero at the first frame,
    # also across the clip boundary (frame 4 takes frame 3, which is c_pre of clip 1)
    w = np.zeros((3, C, C))
    w[0] = eye
    y = oracle.temporal_conv(x, w, 4, 2)
    np.testing.assert_array_equal(y[1:], x[:-1])
    assert (y[0] == 0).all()
    # tap 2 looks one frame ahead, zero at the last frame
    w = np.zeros((3, C, C))
    w[2] = eye
    y = oracle.temporal_conv(x, w, 4, 2)
    np.testing.assert_array_equal(y[:-1], x[1:])
    assert (y[-1] == 0).all()
    # W[t][co][ci]: a single 1 at (co = 2, ci = 0) routes input channel 0 to output channel 2
    w = np.zeros((1, C, C))
    w[0, 2, 0] = 1.0
    y = oracle.temporal_conv(x, w, 4, 2)
    np.testing.assert_array_equal(y[..., 2], x[..., 0])
    assert (y[..., :2] == 0).all()
    # box filter over time of a ramp: interior frames keep the ramp, the ends lose a neighbour
    ramp = np.arange(F, dtype=np.float64)[:, None, None] * np.ones((F, 1, 1))
    y = oracle.temporal_conv(ramp, np.full((3, 1, 1), 1.0 / 3.0), 2, 4)[:, 0, 0]
    np.testing.assert_allclose(y[1:-1], np.arange(1, F - 1), atol=1e-14)
    np.testing.assert_allclose([y[0], y[-1]], [1.0 / 3.0, (2 * F - 3) / 3.0], atol=1e-14)


def brute(x, w, b, n):
    F, P, c_in = x.shape
    c_out = w.shape[1]
    y = np.zeros((F, P, c_out))
    for f in range(F):
        for p in range(P):
            for co in range(c_out):
                acc = 0.0 if b is None else float(b[co])
                for t in range(2 * n + 1):
                    g = f + t - n
                    if 0 <= g < F:
                        for ci in range(c_in):
                            acc += float(w[t, co, ci]) * float(x[g, p, ci])
                y[f, p, co] = acc
    return y


@pytest.mark.parametrize("clip_len,n_clips,n", [(2, 3, 1), (3, 2, 3), (1, 5, 1), (4, 1, 2)])
def test_brute_force_on_tiny_inputs(clip_len, n_clips, n):
    x, w, b = rand_case(clip_len * n_clips, 2, 3, 4, n, seed=7 + n)
    np.testing.assert_allclose(oracle.temporal_conv(x, w, clip_len, n_clips, bias=b),
                               brute(x, w, b, n), rtol=0, atol=1e-13)


def test_partition_invariance_linearity_and_locality():
    x, w, b = rand_case(12, 3, 5, 4, 2, seed=11)
    y = oracle.temporal_conv(x, w, 12, 1, bias=b)
    # how the video is cut into clips cannot matter (n <= clip length)
    for clip_len, n_clips in ((6, 2), (4, 3), (3, 4), (2, 6)):
        np.testing.assert_allclose(oracle.temporal_conv(x, w, clip_len, n_clips, bias=b), y,
                                   rtol=0, atol=1e-13)
    # linear in x (without the bias) and in w
    x2 = np.random.default_rng(12).standard_normal(x.shape)
    np.testing.assert_allclose(oracle.temporal_conv(x + 2 * x2, w, 4, 3),
                               oracle.temporal_conv(x, w, 4, 3) + 2 * oracle.temporal_conv(x2, w, 4, 3),
                               rtol=0, atol=1e-12)
    # frame f of the output depends on frames f - n .. f + n only, and on its own position only
    xp = x.copy()
    xp[7] += 1.0
    d = oracle.temporal_conv(xp, w, 4, 3, bias=b) - oracle.temporal_conv(x, w, 4, 3, bias=b)
    touched = np.abs(d).max(axis=(1, 2)) > 0
    assert touched.tolist() == [5 <= f <= 9 for f in range(12)]
    xp = x.copy()
    xp[:, 1] += 1.0
    d = oracle.temporal_conv(xp, w, 4, 3, bias=b) - oracle.temporal_conv(x, w, 4, 3, bias=b)
    assert (d[:, 0] == 0).all() and (d[:, 2] == 0).all() and (d[:, 1] != 0).any()


def test_bad_arguments():
    x, w, b = rand_case(8, 2, 3, 3, 3, seed=1)
    with pytest.raises(ValueError):
        oracle.temporal_conv(x, w, 2, 4)        # n = 3 reaches past the neighbouring clip
    with pytest.raises(ValueError):
        oracle.temporal_conv(x, w[:2], 4, 2)    # even number of taps
    with pytest.raises(ValueError):
        oracle.temporal_conv(x, w, 3, 2)        # F != N * F_clip


def test_pins_catch_planted_mistakes():
    """Each plausible slip, planted in a copy of the definition, fails the library pin."""
    x, w, b = rand_case(8, 2, 3, 3, 1, seed=5)
    ref = library_conv(x, w, b)
    good = brute(x, w, b, 1)
    np.testing.assert_allclose(good, ref, atol=1e-12)
    flipped = brute(x, w[::-1], b, 1)                       # convolution instead of correlation
    transposed = brute(x, np.swapaxes(w, 1, 2), b, 1)       # W[t][ci][co]
    no_bias = brute(x, w, None, 1)
    for bad in (flipped, transposed, no_bias):
        assert np.abs(bad - ref).max() > 1e-3
    # replicate padding instead of zeros at the video ends
    xr = np.concatenate([x[:1], x, x[-1:]])
    rep = brute(xr, w, b, 1)[1:-1]
    assert np.abs(rep - ref).max() > 1e-3


# ---------------------------------------------------------------- linear projections (Section 4.2)

def test_linear_oracle_matches_library_matmul_and_closed_forms():
    rng = np.random.default_rng(21)
    x = rng.standard_normal((5, 3, 7))
    w = rng.standard_normal((4, 7))
    b = rng.standard_normal(4)
    y = oracle.linear(x, w, bias=b)
    np.testing.assert_allclose(y, x @ w.T + b, rtol=0, atol=1e-13)                 # numpy's matmul
    ref = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b))
    np.testing.assert_allclose(y, ref.numpy(), rtol=0, atol=1e-13)                 # the library layer
    np.testing.assert_allclose(oracle.linear(x, w), x @ w.T, rtol=0, atol=1e-13)
    # identity weights return the input; a single 1 at (co = 2, ci = 5) routes channel 5 to 2
    np.testing.assert_array_equal(oracle.linear(x, np.eye(7)), x)
    w1 = np.zeros((4, 7))
    w1[2, 5] = 1.0
    y1 = oracle.linear(x, w1)
    np.testing.assert_array_equal(y1[..., 2], x[..., 5])
    assert (np.delete(y1, 2, axis=-1) == 0).all()
    # the one-tap temporal convolution is the same map
    np.testing.assert_allclose(oracle.temporal_conv(x, w[None], 5, 1, bias=b), y, rtol=0, atol=1e-13)
    # a transposed weight or a dropped bias is caught by the library pin
    assert np.abs(oracle.linear(x, w) - ref.numpy()).max() > 1e-3
    with pytest.raises(ValueError):
        oracle.linear(x, w.T)


def test_projection_commutes_with_gathering_context():
    """Section 4.2 computes keys and values from the tokens of a clip's context; the projection is
    per token, so gathering projected K equals projecting gathered tokens (why the attention's
    inputs are projected tensors)."""
    rng = np.random.default_rng(22)
    F, P, C = 12, 2, 6
    x = rng.standard_normal((F, P, C))
    w = rng.standard_normal((C, C))
    k = oracle.linear(x, w)
    g = [0, 7, 11]
    np.testing.assert_allclose(oracle.gather_context(k, 4, 3, 1, g),
                               np.where(oracle.gather_context(np.ones((F, 1, 1)), 4, 3, 1, g) > 0,
                                        oracle.linear(oracle.gather_context(x, 4, 3, 1, g), w), 0.0),
                               rtol=0, atol=1e-13)
