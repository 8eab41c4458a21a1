"""Pins of the CPU oracle against what the paper and the mathematics fix.

The paper prints no numeric attention output, so the oracle is pinned by
  a. reduction to full temporal softmax attention (no global set, window over the whole video),
  b. a per-clip check against a library attention routine (torch SDPA, fp64, CPU),
  c. hand-derived context lists (tests/golden/ctx_lists.txt),
  d. closed forms through the whole path (Q = 0 gives the mean of the listed V frames),
  e. softmax weights summing to 1,
  f. invariance to permuting the global set,
  g. constant V giving constant output,
  h. invariance to translating every key by one vector,
  i. linearity in V,
  j. locality (frames outside a clip's list cannot change its output),
  k. a duplicated frame acting as a ln 2 logit bias,
  l. an independently written pure-Python brute force.
No test here touches the GPU library.
"""
import math

import numpy as np
import pytest
import torch

from conftest import read_golden_ctx_lists
from oracle import brute, oracle


def rand_qkv(F, P, h, D, seed):
    rng = np.random.default_rng(seed)
    return tuple(rng.standard_normal((F, P, h, D)) for _ in range(3))


SHAPES = [
    # clip_len, n_clips, w, P, h, D, global
    (4, 2, 1, 3, 1, 8, [0, 4]),
    (4, 3, 0, 2, 2, 5, []),
    (3, 4, 2, 2, 2, 4, [11, 0, 5]),
    (2, 4, 5, 1, 1, 3, [7, 7, 1]),
    (5, 1, 3, 2, 1, 6, [2]),
    (16, 3, 8, 1, 2, 8, list(range(0, 48, 3))),
]


# ---------------------------------------------------------------- c. index lists

@pytest.mark.parametrize("case", read_golden_ctx_lists())
def test_ctx_lists_match_hand_derived(case):
    clip_len, n_clips, w, g, clip, expected = case
    idx, ln = oracle.ctx_indices(clip_len, n_clips, w, g)
    assert ln[clip] == len(expected)
    assert idx[clip, :ln[clip]].tolist() == expected
    assert (idx[clip, ln[clip]:] == -1).all()
    # the brute force builds its list per query frame: every frame of the clip agrees
    for a in range(clip * clip_len, (clip + 1) * clip_len):
        assert brute.key_frames(a, clip_len, n_clips, w, g)[0] == expected


def test_ctx_rejects_bad_arguments():
    with pytest.raises(ValueError):
        oracle.ctx_indices(4, 2, 1, [8])
    with pytest.raises(ValueError):
        oracle.ctx_indices(4, 2, 1, [-1])
    with pytest.raises(ValueError):
        oracle.ctx_indices(4, 2, -1, [0])


def test_ctx_lengths_interior_and_edge():
    # interior clips see F_clip + 2w + G frames, edge clips F_clip + w + G (Section 4.2 sizes)
    idx, ln = oracle.ctx_indices(16, 144, 2, list(range(0, 2304, 144)))
    assert ln[0] == 16 + 2 + 16 and ln[-1] == 16 + 2 + 16
    assert (ln[1:-1] == 16 + 4 + 16).all()
    assert idx.shape == (144, 36)


# ---------------------------------------------------------------- l. brute force

@pytest.mark.parametrize("shape", SHAPES)
def test_matches_python_brute_force(shape):
    clip_len, n_clips, w, P, h, D, g = shape
    q, k, v = rand_qkv(clip_len * n_clips, P, h, D, seed=hash(tuple(shape[:6])) % 1000)
    for scale in (0.0, 0.37):
        o = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=scale)
        ref = np.array(brute.forward(q, k, v, clip_len, n_clips, w, g, scale=scale))
        np.testing.assert_allclose(o, ref, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- a. full attention

def sdpa_f64(q, k, v, scale):
    """q [Lq, D], k/v [Lk, D] -> library softmax attention in fp64 on the CPU."""
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x))[None, None] for x in (q, k, v))
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)[0, 0].numpy()


@pytest.mark.parametrize("clip_len,n_clips", [(4, 3), (2, 5), (16, 2)])
def test_reduces_to_full_temporal_attention(clip_len, n_clips):
    F, P, h, D = clip_len * n_clips, 2, 2, 6
    q, k, v = rand_qkv(F, P, h, D, seed=7)
    w = (n_clips - 1) * clip_len  # every clip's window covers the whole video
    o = oracle.forward(q, k, v, clip_len, n_clips, w, [])
    scale = 1.0 / math.sqrt(D)
    for p in range(P):
        for g in range(h):
            ref = sdpa_f64(q[:, p, g], k[:, p, g], v[:, p, g], scale)
            np.testing.assert_allclose(o[:, p, g], ref, rtol=0, atol=1e-13)
    # a narrower window must differ (the test would otherwise pass vacuously)
    o2 = oracle.forward(q, k, v, clip_len, n_clips, w - 1, [])
    assert np.abs(o2 - o).max() > 1e-6


# ---------------------------------------------------------------- b. per-clip library check

@pytest.mark.parametrize("shape", SHAPES)
def test_per_clip_library_attention(shape):
    clip_len, n_clips, w, P, h, D, g = shape
    q, k, v = rand_qkv(clip_len * n_clips, P, h, D, seed=11)
    scale = 0.5
    o = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=scale)
    golden = {(c[0], c[1], c[2], tuple(c[3]), c[4]): c[5] for c in read_golden_ctx_lists()}
    for i in range(n_clips):
        # the list comes from the hand-derived fixture where there is one, else from the
        # brute force's own list builder (never from the C oracle under test)
        lst = golden.get((clip_len, n_clips, w, tuple(g), i),
                         brute.key_frames(i * clip_len, clip_len, n_clips, w, g)[0])
        rows = slice(i * clip_len, (i + 1) * clip_len)
        for p in range(P):
            for hd in range(h):
                ref = sdpa_f64(q[rows, p, hd], k[lst, p, hd], v[lst, p, hd], scale)
                np.testing.assert_allclose(o[rows, p, hd], ref, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- d. closed forms

def test_zero_query_gives_mean_of_listed_frames():
    # tiny case: clip 0 lists [0,1,2,3,4,0,4] -> mean 14/7 = 2; clip 1 lists [3,4,5,6,7,0,4] -> 29/7
    clip_len, n_clips, w, g = 4, 2, 1, [0, 4]
    F, P, h, D = 8, 3, 2, 4
    q = np.zeros((F, P, h, D))
    k = np.random.default_rng(0).standard_normal((F, P, h, D))
    v = np.broadcast_to(np.arange(F, dtype=np.float64)[:, None, None, None], (F, P, h, D)).copy()
    o = oracle.forward(q, k, v, clip_len, n_clips, w, g)
    np.testing.assert_allclose(o[:4], 2.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(o[4:], 29.0 / 7.0, rtol=0, atol=1e-14)


def test_one_hot_softmax_limit_selects_a_frame():
    # keys orthogonal, one per frame; a huge scale makes the softmax a hard selector,
    # so each query returns the V row of the listed frame whose key matches it
    clip_len, n_clips, w, g = 2, 3, 1, [5]
    F, D = 6, 6
    k = np.eye(F)[:, None, None, :]            # K[f] = e_f
    v = (10.0 + np.arange(F))[:, None, None, None] * np.ones((F, 1, 1, D))
    target = [1, 2, 5, 1, 5, 3]                # a frame inside each query's list
    q = np.eye(F)[target][:, None, None, :]
    o = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=200.0)
    np.testing.assert_allclose(o[:, 0, 0, 0], 10.0 + np.array(target), rtol=0, atol=1e-12)


def test_two_key_closed_form():
    # one clip of one frame, one global frame (itself a different frame): two keys, sigmoid weights
    clip_len, n_clips, w, g = 1, 2, 0, [1]
    q = np.array([1.0, 2.0]).reshape(2, 1, 1, 1) * np.ones((2, 1, 1, 1))
    k = np.array([0.5, -1.5]).reshape(2, 1, 1, 1)
    v = np.array([3.0, 7.0]).reshape(2, 1, 1, 1)
    o = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=1.0)
    # query frame 0: keys [frame0, frame1]: logits q0*k0, q0*k1
    a0 = 1.0 / (1.0 + math.exp(1.0 * (-1.5) - 1.0 * 0.5))
    assert abs(o[0, 0, 0, 0] - (a0 * 3.0 + (1 - a0) * 7.0)) < 1e-14
    # query frame 1: keys [frame1, frame1] (local + the same frame as global): output is V[1]
    assert abs(o[1, 0, 0, 0] - 7.0) < 1e-14


# ---------------------------------------------------------------- e, g. weights / constant V

@pytest.mark.parametrize("shape", SHAPES)
def test_weights_sum_to_one_and_constant_v(shape):
    clip_len, n_clips, w, P, h, D, g = shape
    q, k, v = rand_qkv(clip_len * n_clips, P, h, D, seed=3)
    o, wts = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=1.3, return_weights=True)
    np.testing.assert_allclose(wts.sum(-1), 1.0, rtol=0, atol=1e-12)
    assert (wts >= 0).all()
    idx, ln = oracle.ctx_indices(clip_len, n_clips, w, g)
    for i in range(n_clips):
        rows = slice(i * clip_len, (i + 1) * clip_len)
        assert (wts[rows, :, :, ln[i]:] == 0).all()
        # output really is weights @ V over the clip's list
        ref = np.einsum("aphj,jphd->aphd", wts[rows][..., :ln[i]], v[idx[i, :ln[i]]])
        np.testing.assert_allclose(o[rows], ref, rtol=0, atol=1e-13)
    vc = np.full_like(v, -2.75)
    oc = oracle.forward(q, k, vc, clip_len, n_clips, w, g)
    np.testing.assert_allclose(oc, -2.75, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- f. permutation of G

def test_permuting_global_set_changes_nothing():
    clip_len, n_clips, w = 4, 4, 1
    q, k, v = rand_qkv(16, 2, 2, 5, seed=5)
    g = [0, 9, 13, 6, 6]
    base = oracle.forward(q, k, v, clip_len, n_clips, w, g)
    rng = np.random.default_rng(1)
    for _ in range(4):
        perm = rng.permutation(len(g))
        o = oracle.forward(q, k, v, clip_len, n_clips, w, [g[t] for t in perm])
        np.testing.assert_allclose(o, base, rtol=0, atol=1e-13)
    # but changing the set does change it
    o = oracle.forward(q, k, v, clip_len, n_clips, w, [0, 9, 13, 6, 7])
    assert np.abs(o - base).max() > 1e-6


# ---------------------------------------------------------------- h, i. invariances

def test_key_translation_invariance_and_linearity_in_v():
    clip_len, n_clips, w, g = 4, 3, 2, [1, 10]
    q, k, v = rand_qkv(12, 2, 2, 6, seed=9)
    base = oracle.forward(q, k, v, clip_len, n_clips, w, g)
    u = np.random.default_rng(2).standard_normal((1, 2, 2, 6))
    shifted = oracle.forward(q, k + u, v, clip_len, n_clips, w, g)
    np.testing.assert_allclose(shifted, base, rtol=0, atol=1e-12)
    v2 = np.random.default_rng(4).standard_normal(v.shape)
    lin = oracle.forward(q, k, 2.0 * v - 3.0 * v2, clip_len, n_clips, w, g)
    ref = 2.0 * base - 3.0 * oracle.forward(q, k, v2, clip_len, n_clips, w, g)
    np.testing.assert_allclose(lin, ref, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- j. locality

def test_frames_outside_the_list_do_not_matter():
    clip_len, n_clips, w, g = 4, 4, 1, [0, 12]
    q, k, v = rand_qkv(16, 2, 1, 4, seed=13)
    base = oracle.forward(q, k, v, clip_len, n_clips, w, g)
    # clip 1 lists frames 3..8 plus {0, 12}; frame 10 is outside it, frame 8 inside
    k2, v2 = k.copy(), v.copy()
    k2[10] += 5.0
    v2[10] -= 5.0
    o = oracle.forward(q, k2, v2, clip_len, n_clips, w, g)
    assert np.array_equal(o[4:8], base[4:8])          # clip 1 untouched, bit for bit
    assert np.abs(o[8:12] - base[8:12]).max() > 1e-6  # clip 2 owns frame 10
    k3 = k.copy()
    k3[8] += 5.0
    o = oracle.forward(q, k3, v, clip_len, n_clips, w, g)
    assert np.abs(o[4:8] - base[4:8]).max() > 1e-6    # frame 8 is clip 1's c_post


# ---------------------------------------------------------------- k. duplicates

def test_duplicate_frame_counts_twice():
    # listing every global frame twice equals adding ln 2 to the global logits; emulate the bias
    # by hand: weights of a doubled key are 2 e^s / Z
    clip_len, n_clips, w = 2, 3, 0
    q, k, v = rand_qkv(6, 1, 1, 3, seed=21)
    g = [5]
    o2 = oracle.forward(q, k, v, clip_len, n_clips, w, g + g, scale=1.0)
    for a in range(6):
        clip = a // clip_len
        loc = list(range(clip * clip_len, (clip + 1) * clip_len))
        logits = np.array([q[a, 0, 0] @ k[f, 0, 0] for f in loc] + [q[a, 0, 0] @ k[5, 0, 0] + math.log(2.0)])
        wts = np.exp(logits - logits.max())
        wts /= wts.sum()
        ref = wts[:-1] @ v[loc, 0, 0] + wts[-1] * v[5, 0, 0]
        np.testing.assert_allclose(o2[a, 0, 0], ref, rtol=0, atol=1e-13)
    # a global frame that is also local is NOT deduplicated (Concat, not set union)
    o_dup = oracle.forward(q, k, v, clip_len, n_clips, w, [4], scale=1.0)
    o_nodup = oracle.forward(q, k, v, clip_len, n_clips, w, [], scale=1.0)
    assert np.abs(o_dup[4:6] - o_nodup[4:6]).max() > 1e-6


# ---------------------------------------------------------------- scope weights (Section 5.1)

def test_scope_bias_pins():
    clip_len, n_clips, w = 4, 3, 1
    g = [0, 7, 10]
    q, k, v = rand_qkv(12, 2, 2, 5, seed=31)
    base = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7)
    # equal biases on both scopes cancel in the softmax
    same = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7, bias_local=3.5,
                          bias_global=3.5)
    np.testing.assert_allclose(same, base, rtol=0, atol=1e-12)
    # only the difference matters
    a = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7, bias_local=1.0, bias_global=3.0)
    b = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7, bias_local=0.0, bias_global=2.0)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
    assert np.abs(a - base).max() > 1e-3
    # a global bias of ln 2 equals listing every global frame twice (weights count twice)
    dbl = oracle.forward(q, k, v, clip_len, n_clips, w, g + g, scale=0.7)
    ln2 = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7, bias_global=math.log(2.0))
    np.testing.assert_allclose(ln2, dbl, rtol=0, atol=1e-12)
    # a very negative global bias removes the global scope, a very negative local bias leaves
    # plain attention over the global frames only (library routine)
    no_g = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7, bias_global=-800.0)
    np.testing.assert_allclose(no_g, oracle.forward(q, k, v, clip_len, n_clips, w, [], scale=0.7),
                               rtol=0, atol=1e-12)
    only_g = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7, bias_local=-800.0)
    for p in range(2):
        for hd in range(2):
            ref = sdpa_f64(q[:, p, hd], k[g, p, hd], v[g, p, hd], 0.7)
            np.testing.assert_allclose(only_g[:, p, hd], ref, rtol=0, atol=1e-12)
    # hand-computed two-key case: one local key, one global key, bias b on the global one
    q1 = np.array([1.0, 1.0]).reshape(2, 1, 1, 1)
    k1 = np.array([0.25, -0.5]).reshape(2, 1, 1, 1)
    v1 = np.array([2.0, 6.0]).reshape(2, 1, 1, 1)
    o = oracle.forward(q1, k1, v1, 1, 2, 0, [1], scale=1.0, bias_global=1.5)
    wl, wg = math.exp(0.25), math.exp(-0.5 + 1.5)
    assert abs(o[0, 0, 0, 0] - (wl * 2.0 + wg * 6.0) / (wl + wg)) < 1e-14
    # the brute force agrees
    bf = np.array(brute.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7, bias_local=-0.3,
                                bias_global=2.2))
    np.testing.assert_allclose(
        oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=0.7, bias_local=-0.3,
                       bias_global=2.2), bf, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- sliding-window local scope (Section 4.2)

def banded_sdpa_f64(q, k, v, scale, radius):
    """Library attention over the whole sequence with a band mask |f - a| <= radius."""
    n = q.shape[0]
    idx = torch.arange(n)
    mask = (idx[None, :] - idx[:, None]).abs() <= radius
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x))[None, None] for x in (q, k, v))
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask,
                                                            scale=scale)[0, 0].numpy()


def test_sliding_window_pins():
    F, P, h, D = 24, 2, 2, 5
    q, k, v = rand_qkv(F, P, h, D, seed=17)
    scale = 0.6
    # (1) a window that covers every clip's whole list changes nothing
    base = oracle.forward(q, k, v, 4, 6, 2, [0, 13], scale=scale)
    wide = oracle.forward(q, k, v, 4, 6, 2, [0, 13], scale=scale, window=4 + 2)
    assert np.array_equal(wide, base)
    # (2) radius 0 and no global frames: the only visible key is the frame itself
    self_only = oracle.forward(q, k, v, 4, 6, 2, [], scale=scale, window=0)
    np.testing.assert_allclose(self_only, v, rtol=0, atol=1e-15)
    # (3) with boundary context at least as wide as the window (w >= r) the result cannot
    # depend on how the frames are cut into clips, and equals banded attention over the
    # whole video computed by the library routine
    r = 3
    outs = [oracle.forward(q, k, v, clip_len, F // clip_len, w, [], scale=scale, window=r)
            for clip_len, w in ((4, 3), (8, 3), (24, 0), (2, 5), (6, 4))]
    for o in outs[1:]:
        np.testing.assert_allclose(o, outs[0], rtol=0, atol=1e-13)
    for p in range(P):
        for hd in range(h):
            ref = banded_sdpa_f64(q[:, p, hd], k[:, p, hd], v[:, p, hd], scale, r)
            np.testing.assert_allclose(outs[0][:, p, hd], ref, rtol=0, atol=1e-13)
    # (4) w < r truncates the window at the clip's local range: differs from the full band
    trunc = oracle.forward(q, k, v, 4, 6, 1, [], scale=scale, window=r)
    assert np.abs(trunc - outs[0]).max() > 1e-6
    # (5) global frames stay visible whatever their distance; the brute force agrees,
    # also together with scope biases
    g = [23, 0, 11]
    o = oracle.forward(q, k, v, 4, 6, 2, g, scale=scale, window=1, bias_global=0.8)
    bf = np.array(brute.forward(q, k, v, 4, 6, 2, g, scale=scale, window=1, bias_global=0.8))
    np.testing.assert_allclose(o, bf, rtol=0, atol=1e-13)
    o_nog = oracle.forward(q, k, v, 4, 6, 2, [], scale=scale, window=1)
    assert np.abs(o - o_nog).max() > 1e-3
    # (6) weights of hidden keys are exactly zero and the rest still sums to one
    _, wts = oracle.forward(q, k, v, 4, 6, 2, g, scale=scale, window=1, return_weights=True)
    np.testing.assert_allclose(wts.sum(-1), 1.0, rtol=0, atol=1e-12)
    idx, ln = oracle.ctx_indices(4, 6, 2, g)
    for a in range(F):
        i = a // 4
        nloc = ln[i] - len(g)
        hidden = np.abs(idx[i, :nloc] - a) > 1
        assert (wts[a][..., :nloc][..., hidden] == 0).all()
        assert (wts[a][..., :nloc][..., ~hidden] > 0).all()


# ---------------------------------------------------------------- gather by definition

def test_gather_context_is_index_select():
    clip_len, n_clips, w, g = 4, 3, 2, [11, 0]
    x = np.random.default_rng(0).integers(0, 2 ** 16, size=(12, 5, 6), dtype=np.uint16)
    out = oracle.gather_context(x, clip_len, n_clips, w, g)
    golden_clip0 = [0, 1, 2, 3, 4, 5, 11, 0]          # hand-derived: [0,6) then globals
    golden_clip1 = [2, 3, 4, 5, 6, 7, 8, 9, 11, 0]    # [2,10) then globals
    assert out.shape == (3, 10, 5, 6)
    assert np.array_equal(out[0, :8], x[golden_clip0])
    assert (out[0, 8:] == 0).all()
    assert np.array_equal(out[1], x[golden_clip1])


# ---------------------------------------------------------------- set union instead of Concat (Section 4.2)

def test_dedup_global_pins():
    """With dedup the key set of a query is the union of Section 4.2's formula: no frame twice."""
    rng = np.random.default_rng(77)
    clip_len, n_clips, w, P, h, D = 4, 5, 1, 2, 2, 3
    F = clip_len * n_clips
    q, k, v = (rng.standard_normal((F, P, h, D)) for _ in range(3))
    scale = 0.9
    g = [0, 4, 4, 17, 9, 0]          # repeats inside G, and frames inside some clips' local range
    got = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=scale, dedup=True)
    # (1) the separately written brute force over explicit union lists
    np.testing.assert_allclose(got, np.array(brute.forward(q, k, v, clip_len, n_clips, w, g, scale=scale,
                                                           dedup=True)), rtol=0, atol=1e-12)
    # (2) per clip it is plain attention over the deduplicated list: library routine
    for i in range(n_clips):
        lo, hi = max(0, i * clip_len - w), min(F, (i + 1) * clip_len + w)
        frames = list(range(lo, hi))
        for f in g:
            if f not in frames:
                frames.append(f)
        idx = torch.as_tensor(frames)
        qt = torch.from_numpy(q[i * clip_len:(i + 1) * clip_len]).permute(1, 2, 0, 3)   # [P, h, Fc, D]
        kt = torch.from_numpy(k).index_select(0, idx).permute(1, 2, 0, 3)
        vt = torch.from_numpy(v).index_select(0, idx).permute(1, 2, 0, 3)
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=scale)
        np.testing.assert_allclose(got[i * clip_len:(i + 1) * clip_len], ref.permute(2, 0, 1, 3).numpy(),
                                   rtol=0, atol=1e-12)
    # (3) it differs from the concatenation exactly where a frame is listed twice
    cat = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=scale)
    assert np.abs(cat - got).max() > 1e-3
    # (4) a global set that repeats nothing and overlaps no clip's range: the flag changes nothing
    wide = oracle.forward(q, k, v, 4, 5, 0, [], scale=scale, dedup=True)
    np.testing.assert_array_equal(wide, oracle.forward(q, k, v, 4, 5, 0, [], scale=scale))
    g1 = [19]
    a_ = oracle.forward(q, k, v, clip_len, n_clips, w, g1, scale=scale, dedup=True)
    b_ = oracle.forward(q, k, v, clip_len, n_clips, w, g1, scale=scale)
    np.testing.assert_array_equal(a_[:14], b_[:14])          # clips 0..2 and frames 12, 13 of clip 3 ...
    assert np.abs(a_[16:] - b_[16:]).max() > 1e-6            # ... but clip 4 holds frame 19 itself
    # (5) a global set inside clip 0's range: clip 0 attends as if there were no global set
    g0 = [0, 2, 4]
    d0 = oracle.forward(q, k, v, clip_len, n_clips, w, g0, scale=scale, dedup=True)
    none = oracle.forward(q, k, v, clip_len, n_clips, w, [], scale=scale)
    np.testing.assert_allclose(d0[:clip_len], none[:clip_len], rtol=0, atol=1e-14)
    # (6) weights: the dropped entries get exactly 0, the rest still sum to 1
    _, wts = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=scale, dedup=True, return_weights=True)
    np.testing.assert_allclose(wts.sum(axis=-1), 1.0, rtol=0, atol=1e-12)
    idx, ln = oracle.ctx_indices(clip_len, n_clips, w, g)
    for i in range(n_clips):
        row = idx[i, :ln[i]].tolist()
        for j, f in enumerate(row):
            dropped = j >= ln[i] - len(g) and f in row[:j]
            zero = (wts[i * clip_len:(i + 1) * clip_len, :, :, j] == 0).all()
            assert zero == dropped, (i, j, f)


def test_dedup_with_sliding_window_is_per_query():
    """Under the window a local copy the query cannot see does not shadow the global copy."""
    rng = np.random.default_rng(78)
    clip_len, n_clips, w, P, h, D = 4, 3, 2, 1, 1, 2
    q, k, v = (rng.standard_normal((12, P, h, D)) for _ in range(3))
    g = [5, 1]
    got = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=1.0, window=1, dedup=True)
    np.testing.assert_allclose(got, np.array(brute.forward(q, k, v, clip_len, n_clips, w, g, scale=1.0,
                                                           window=1, dedup=True)), rtol=0, atol=1e-12)
    _, wts = oracle.forward(q, k, v, clip_len, n_clips, w, g, scale=1.0, window=1, dedup=True,
                            return_weights=True)
    idx, ln = oracle.ctx_indices(clip_len, n_clips, w, g)
    jg5 = ln[1] - 2   # position of global frame 5 in clip 1's list (frames 2..9, then 5, 1)
    # query frame 4 sees local 3..5: global 5 is dropped; query frame 7 sees 6..8: global 5 stays
    assert wts[4, 0, 0, jg5] == 0 and wts[5, 0, 0, jg5] == 0 and wts[6, 0, 0, jg5] == 0
    assert wts[7, 0, 0, jg5] > 0
