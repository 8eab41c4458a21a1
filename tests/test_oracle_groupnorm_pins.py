"""Pins of the group-normalisation oracle (Section 4.2, "Group normalization"): the library
routine on the whole video as one sample, numpy statistics, closed forms, independence of the
clip partition, and the paper's footnote (averaging per-clip deviations is a different thing)."""
import numpy as np
import pytest
import torch

from oracle import oracle


def rand_x(F, P, C, seed, spread=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((F, P, C))
    if spread:  # clips with different means and scales, so that per-clip statistics differ
        x = x * (1.0 + 0.5 * np.arange(F)[:, None, None] / F) + 0.3 * np.sin(np.arange(F))[:, None, None]
    return x


@pytest.mark.parametrize("clip_len,n_clips,P,C,groups", [(4, 3, 5, 12, 3), (2, 5, 3, 8, 8), (16, 2, 2, 40, 1),
                                                         (1, 7, 4, 6, 2)])
def test_matches_library_group_norm_over_the_whole_video(clip_len, n_clips, P, C, groups):
    F = clip_len * n_clips
    x = rand_x(F, P, C, seed=F + C)
    rng = np.random.default_rng(1)
    gamma, beta = rng.standard_normal(C), rng.standard_normal(C)
    y, mean, var = oracle.groupnorm(x, clip_len, n_clips, groups, eps=1e-5, gamma=gamma, beta=beta)
    # one sample [1, C, F, P]: torch normalises over (C/groups, F, P) per group
    t = torch.from_numpy(x).permute(2, 0, 1)[None]
    ref = torch.nn.functional.group_norm(t, groups, torch.from_numpy(gamma), torch.from_numpy(beta),
                                         eps=1e-5)[0].permute(1, 2, 0).numpy()
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)
    xg = x.reshape(F, P, groups, C // groups)
    np.testing.assert_allclose(mean, xg.mean(axis=(0, 1, 3)), rtol=0, atol=1e-13)
    np.testing.assert_allclose(var, xg.var(axis=(0, 1, 3)), rtol=0, atol=1e-13)


def test_closed_forms_and_invariances():
    x = rand_x(12, 3, 8, seed=3)
    beta = np.linspace(-1, 1, 8)
    # constant input: every deviation is zero, the output is beta
    y, mean, var = oracle.groupnorm(np.full((12, 3, 8), 2.5), 4, 3, 2, eps=1e-5, beta=beta)
    np.testing.assert_allclose(y, np.broadcast_to(beta, y.shape), rtol=0, atol=1e-15)
    np.testing.assert_allclose(mean, 2.5, rtol=0, atol=1e-15)
    assert (var == 0).all()
    # output has zero mean and unit variance per group (eps = 0, no affine)
    y, _, _ = oracle.groupnorm(x, 4, 3, 2, eps=0.0)
    yg = y.reshape(12, 3, 2, 4)
    np.testing.assert_allclose(yg.mean(axis=(0, 1, 3)), 0.0, atol=1e-13)
    np.testing.assert_allclose(yg.var(axis=(0, 1, 3)), 1.0, atol=1e-12)
    # x -> a x + b leaves the normalised output unchanged (eps = 0)
    y2, _, _ = oracle.groupnorm(3.0 * x - 7.0, 4, 3, 2, eps=0.0)
    np.testing.assert_allclose(y2, y, rtol=0, atol=1e-12)
    # the clip partition cannot matter: the statistics are those of the whole video
    for clip_len, n_clips in ((12, 1), (1, 12), (6, 2), (3, 4)):
        y3, _, _ = oracle.groupnorm(x, clip_len, n_clips, 2, eps=0.0)
        np.testing.assert_allclose(y3, y, rtol=0, atol=1e-12)


def test_footnote_averaging_per_clip_deviations_is_wrong():
    # clips with different means: the mean of per-clip variances (about per-clip means) misses the
    # between-clip part, and the mean of per-clip standard deviations is different again
    x = rand_x(12, 4, 6, seed=9)
    _, _, var = oracle.groupnorm(x, 4, 3, 1, eps=0.0)
    clips = x.reshape(3, 4 * 4 * 6)
    var_within = clips.var(axis=1).mean()
    between = clips.mean(axis=1).var()
    assert abs(var[0] - (var_within + between)) < 1e-13      # law of total variance
    assert var[0] - var_within > 1e-3
    assert abs(np.sqrt(var[0]) - clips.std(axis=1).mean()) > 1e-3


def test_rejects_bad_arguments():
    x = np.zeros((4, 2, 6))
    with pytest.raises(ValueError):
        oracle.groupnorm(x, 2, 2, 4)       # 6 channels do not split into 4 groups
    with pytest.raises(ValueError):
        oracle.groupnorm(x, 3, 2, 2)       # F != N * clip_len
