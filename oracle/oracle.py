"""ctypes front end of the C oracle (oracle/dsattn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.

Functions mirror the paper's statement of Dual-scope attention (Section 4.2)
under the clip split of Section 4 / 4.1; see the header of the C file for the
exact definition and the readings taken where the paper is silent.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        i64 = ctypes.c_int64
        p = ctypes.c_void_p
        lib.oracle_ctx_max.restype = i64
        lib.oracle_ctx_max.argtypes = [i64, i64, i64, i64]
        lib.oracle_ctx_indices.restype = ctypes.c_int
        lib.oracle_ctx_indices.argtypes = [i64, i64, i64, p, i64, i64, p, p]
        lib.oracle_forward.restype = ctypes.c_int
        lib.oracle_forward.argtypes = [i64, i64, i64, i64, i64, i64, p, i64, ctypes.c_double,
                                       ctypes.c_double, ctypes.c_double, i64, ctypes.c_int, p, p, p, p, p]
        lib.oracle_gather_context.restype = ctypes.c_int
        lib.oracle_gather_context.argtypes = [i64, i64, i64, p, i64, i64, p, p]
        lib.oracle_groupnorm.restype = ctypes.c_int
        lib.oracle_groupnorm.argtypes = [i64, i64, i64, i64, i64, ctypes.c_double, p, p, p, p, p, p]
        lib.oracle_temporal_conv.restype = ctypes.c_int
        lib.oracle_temporal_conv.argtypes = [i64, i64, i64, i64, i64, i64, p, p, p, p]
        lib.oracle_linear.restype = ctypes.c_int
        lib.oracle_linear.argtypes = [i64, i64, i64, p, p, p, p]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _gidx(global_idx):
    g = np.ascontiguousarray(np.asarray(global_idx, dtype=np.int32).reshape(-1))
    return g, (g.ctypes.data if g.size else None)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def ctx_max(clip_len, n_clips, w, n_global) -> int:
    return int(_load().oracle_ctx_max(clip_len, n_clips, w, n_global))


def ctx_indices(clip_len, n_clips, w, global_idx):
    """Returns (ctx_idx [N, lk_max] int32 with -1 padding, ctx_len [N] int32)."""
    lib = _load()
    g, gp = _gidx(global_idx)
    lk = ctx_max(clip_len, n_clips, w, g.size)
    idx = np.empty((n_clips, lk), dtype=np.int32)
    ln = np.empty((n_clips,), dtype=np.int32)
    rc = lib.oracle_ctx_indices(clip_len, n_clips, w, gp, g.size, lk, idx.ctypes.data,
                                ln.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_ctx_indices: bad arguments")
    return idx, ln


def forward(q, k, v, clip_len, n_clips, w, global_idx, scale=0.0, return_weights=False,
            bias_local=0.0, bias_global=0.0, window=-1, dedup=False):
    """q, k, v: arrays [F, P, h, D] (any float dtype; converted exactly to float64).

    bias_local / bias_global: scope weights of Section 5.1 as additive logit biases.
    window: sliding-window radius for local keys (Section 4.2), < 0 for none.
    dedup: set union instead of concatenation (Section 4.2): no frame counts twice.
    Returns O [F, P, h, D] float64, and the weights [F, P, h, lk_max] if asked.
    """
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    F, P, h, D = q.shape
    if F != clip_len * n_clips or k.shape != q.shape or v.shape != q.shape:
        raise ValueError("shape mismatch")
    g, gp = _gidx(global_idx)
    o = np.empty_like(q)
    wts = None
    wp = None
    if return_weights:
        lk = ctx_max(clip_len, n_clips, w, g.size)
        wts = np.empty((F, P, h, lk), dtype=np.float64)
        wp = wts.ctypes.data
    rc = lib.oracle_forward(clip_len, n_clips, w, P, h, D, gp, g.size, float(scale),
                            float(bias_local), float(bias_global), int(window), int(bool(dedup)),
                            q.ctypes.data,
                            k.ctypes.data, v.ctypes.data, o.ctypes.data, wp)
    if rc != 0:
        raise ValueError(f"oracle_forward failed with {rc}")
    return (o, wts) if return_weights else o


def gather_context(x, clip_len, n_clips, w, global_idx):
    """x: [F, ...] any dtype. Returns [N, lk_max, ...] with zero rows past each list."""
    lib = _load()
    x = np.ascontiguousarray(x)
    F = x.shape[0]
    if F != clip_len * n_clips:
        raise ValueError("shape mismatch")
    g, gp = _gidx(global_idx)
    lk = ctx_max(clip_len, n_clips, w, g.size)
    row_bytes = x.nbytes // F
    out = np.empty((n_clips, lk) + x.shape[1:], dtype=x.dtype)
    rc = lib.oracle_gather_context(clip_len, n_clips, w, gp, g.size, row_bytes,
                                   x.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_gather_context failed with {rc}")
    return out


def groupnorm(x, clip_len, n_clips, groups, eps=1e-5, gamma=None, beta=None):
    """Clip-parallel group normalisation (Section 4.2): x [F, P, C] -> (y, mean[groups], var[groups]),
    statistics over the whole video per channel group, computed clip by clip as the paper orders it."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    F, P, C = x.shape
    if F != clip_len * n_clips:
        raise ValueError("shape mismatch")
    ga = None if gamma is None else np.ascontiguousarray(gamma, dtype=np.float64)
    be = None if beta is None else np.ascontiguousarray(beta, dtype=np.float64)
    y = np.empty_like(x)
    mean = np.empty((groups,), dtype=np.float64)
    var = np.empty((groups,), dtype=np.float64)
    rc = lib.oracle_groupnorm(clip_len, n_clips, P, C, groups, float(eps), x.ctypes.data,
                              None if ga is None else ga.ctypes.data,
                              None if be is None else be.ctypes.data, y.ctypes.data,
                              mean.ctypes.data, var.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_groupnorm failed with {rc}")
    return y, mean, var


def temporal_conv(x, w, clip_len, n_clips, bias=None):
    """Clip-parallel temporal convolution (Section 4.2): x [F, P, C_in], w [2n+1, C_out, C_in]
    (tap t looks at frame a + t - n), bias [C_out] or None -> y [F, P, C_out] float64.  Every clip
    is convolved on its own, padded with n frames of each neighbouring clip (zeros at the ends)."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    F, P, c_in = x.shape
    taps, c_out, c_in_w = w.shape
    if F != clip_len * n_clips or c_in_w != c_in or taps % 2 != 1:
        raise ValueError("shape mismatch")
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    if b is not None and b.shape != (c_out,):
        raise ValueError("bias shape")
    y = np.empty((F, P, c_out), dtype=np.float64)
    rc = lib.oracle_temporal_conv(clip_len, n_clips, P, c_in, c_out, taps // 2, x.ctypes.data,
                                  w.ctypes.data, None if b is None else b.ctypes.data,
                                  y.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_temporal_conv failed with {rc}")
    return y


def linear(x, w, bias=None):
    """Token-wise projection (Section 4.2): x [..., C_in], w [C_out, C_in], bias [C_out] or None
    -> y [..., C_out] float64."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    c_out, c_in = w.shape
    if x.shape[-1] != c_in:
        raise ValueError("shape mismatch")
    rows = x.size // c_in
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    if b is not None and b.shape != (c_out,):
        raise ValueError("bias shape")
    y = np.empty(x.shape[:-1] + (c_out,), dtype=np.float64)
    rc = lib.oracle_linear(rows, c_in, c_out, x.ctypes.data, w.ctypes.data,
                           None if b is None else b.ctypes.data, y.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle_linear failed with {rc}")
    return y
