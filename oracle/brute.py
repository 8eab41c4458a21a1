"""Pure-Python brute force of Dual-scope attention for tiny inputs.

TEST INFRASTRUCTURE ONLY.  Written separately from the C oracle and in a
different shape on purpose (per query, explicit key list, Python floats and
math.exp), so that the two can be checked against each other.

Definition followed: Section 4.2 (key/value frames of a query = local
neighbours plus global frames, concatenated) with the per-clip local scope of
Section 4.1 (own clip plus c_pre / c_post boundary frames).
"""
import math


def key_frames(a, clip_len, n_clips, w, global_idx, window=-1, dedup=False):
    """Frame list seen by a query in frame `a` and the number of local entries in it: local
    part then global part.  With window >= 0 only local frames within `window` of `a` are kept
    (Section 4.2).  With dedup the list is the set union of Section 4.2: a global frame that is
    already in the list is not added again."""
    F = clip_len * n_clips
    clip = a // clip_len
    first = clip * clip_len - w
    last = clip * clip_len + clip_len - 1 + w
    local = [f for f in range(first, last + 1) if 0 <= f < F]
    if window >= 0:
        local = [f for f in local if abs(f - a) <= window]
    frames = list(local)
    for g in global_idx:
        if not (dedup and int(g) in frames):
            frames.append(int(g))
    return frames, len(local)


def forward(q, k, v, clip_len, n_clips, w, global_idx, scale=None, bias_local=0.0,
            bias_global=0.0, window=-1, dedup=False):
    """q, k, v: nested lists / arrays indexed [f][p][g][d]. Returns nested lists."""
    F = clip_len * n_clips
    P = len(q[0])
    H = len(q[0][0])
    D = len(q[0][0][0])
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(D)
    out = [[[[0.0] * D for _ in range(H)] for _ in range(P)] for _ in range(F)]
    for a in range(F):
        frames, n_local = key_frames(a, clip_len, n_clips, w, global_idx, window, dedup)
        # scope weights (Section 5.1) as logit biases: local keys first, then global keys
        bias = [bias_local] * n_local + [bias_global] * (len(frames) - n_local)
        for p in range(P):
            for g in range(H):
                logits = []
                for f, b in zip(frames, bias):
                    logits.append(scale * sum(float(q[a][p][g][d]) * float(k[f][p][g][d])
                                              for d in range(D)) + b)
                top = max(logits)
                ex = [math.exp(x - top) for x in logits]
                tot = sum(ex)
                for d in range(D):
                    out[a][p][g][d] = sum(e * float(v[f][p][g][d])
                                          for e, f in zip(ex, frames)) / tot
    return out
