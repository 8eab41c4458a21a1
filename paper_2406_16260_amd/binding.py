"""Thin ctypes binding of libdsattn.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/dsattn.h).
PyTorch supplies device memory (`tensor.data_ptr()`) and the stream handle; all
arithmetic runs in the library's HIP kernels.  There is no CPU fallback: if the
library is missing, loading fails with an error.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdsattn.so")

DSATTN_OK = 0
DSATTN_EINVAL = -1
DSATTN_EUNSUPPORTED = -2
DSATTN_ENOMEM = -3
DSATTN_EHIP = -4
DSATTN_ENODEVICE = -5

DSATTN_F32 = 0
DSATTN_BF16 = 1
DSATTN_FLAG_FORCE_GENERIC = 1
DSATTN_FLAG_SLIDING_WINDOW = 2
DSATTN_FLAG_DEDUP_GLOBAL = 4

EXPORTS = (
    "dsattn_plan", "dsattn_plan_destroy", "dsattn_plan_ctx_max", "dsattn_plan_ctx_indices",
    "dsattn_plan_launch_info", "dsattn_gather_context", "dsattn_forward", "dsattn_forward_ctx",
    "dsattn_copy_probe", "dsattn_strerror", "dsattn_last_error", "dsattn_groupnorm_workspace",
    "dsattn_groupnorm", "dsattn_temporal_conv_info", "dsattn_temporal_conv", "dsattn_linear_info",
    "dsattn_linear", "dsattn_groupnorm_static", "dsattn_groupnorm_static_max_bytes",
)


class DsattnDesc(ctypes.Structure):
    _fields_ = [
        ("clip_len", ctypes.c_int32), ("n_clips", ctypes.c_int32), ("local_ctx", ctypes.c_int32),
        ("spatial", ctypes.c_int32), ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("io_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32), ("scale", ctypes.c_float),
        ("flags", ctypes.c_uint32), ("bias_local", ctypes.c_float), ("bias_global", ctypes.c_float),
        ("window", ctypes.c_int32),
    ]


class DsattnGnDesc(ctypes.Structure):
    _fields_ = [
        ("clip_len", ctypes.c_int32), ("n_clips", ctypes.c_int32), ("spatial", ctypes.c_int32),
        ("channels", ctypes.c_int32), ("groups", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
        ("eps", ctypes.c_float),
    ]


class DsattnConvDesc(ctypes.Structure):
    _fields_ = [
        ("clip_len", ctypes.c_int32), ("n_clips", ctypes.c_int32), ("spatial", ctypes.c_int32),
        ("c_in", ctypes.c_int32), ("c_out", ctypes.c_int32), ("reach", ctypes.c_int32),
        ("io_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
    ]


class DsattnLinearDesc(ctypes.Structure):
    _fields_ = [
        ("rows", ctypes.c_int64), ("c_in", ctypes.c_int32), ("c_out", ctypes.c_int32),
        ("n_out", ctypes.c_int32), ("io_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
    ]


class DsattnConvInfo(ctypes.Structure):
    _fields_ = [
        ("kernel", ctypes.c_int32), ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32),
        ("tile_k", ctypes.c_int32), ("n_blocks", ctypes.c_int32), ("block_threads", ctypes.c_int32),
        ("lds_bytes", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("useful_flops", ctypes.c_int64), ("algorithmic_bytes", ctypes.c_int64),
    ]

    def as_dict(self):
        return {name: int(getattr(self, name)) for name, _ in self._fields_ if name != "reserved"}


class DsattnLaunchInfo(ctypes.Structure):
    _fields_ = [
        ("kernel", ctypes.c_int32), ("heads_per_wave", ctypes.c_int32),
        ("local_tiles", ctypes.c_int32), ("global_tiles", ctypes.c_int32),
        ("clips_per_task", ctypes.c_int32), ("n_tasks", ctypes.c_int32),
        ("block_threads", ctypes.c_int32), ("lds_bytes", ctypes.c_int32),
        ("algorithmic_bytes", ctypes.c_int64),
    ]

    def as_dict(self):
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


class DsattnError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        lib = load()
        detail = lib.dsattn_last_error().decode()
        super().__init__(f"{where}: {lib.dsattn_strerror(self.code).decode()} ({self.code})"
                         + (f": {detail}" if detail else ""))


_lib = None


def load():
    """Load libdsattn.so (built in-tree by paper_2406_16260_amd.build). Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2406_16260_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
    lib.dsattn_plan.restype = ctypes.c_int
    lib.dsattn_plan.argtypes = [ctypes.POINTER(DsattnDesc), vp, ctypes.c_int32, ctypes.c_int,
                                ctypes.POINTER(vp)]
    lib.dsattn_plan_destroy.restype = None
    lib.dsattn_plan_destroy.argtypes = [vp]
    lib.dsattn_plan_ctx_max.restype = ctypes.c_int
    lib.dsattn_plan_ctx_max.argtypes = [vp, i32p]
    lib.dsattn_plan_ctx_indices.restype = ctypes.c_int
    lib.dsattn_plan_ctx_indices.argtypes = [vp, vp, vp]
    lib.dsattn_plan_launch_info.restype = ctypes.c_int
    lib.dsattn_plan_launch_info.argtypes = [vp, ctypes.POINTER(DsattnLaunchInfo)]
    lib.dsattn_gather_context.restype = ctypes.c_int
    lib.dsattn_gather_context.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.dsattn_forward.restype = ctypes.c_int
    lib.dsattn_forward.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.dsattn_forward_ctx.restype = ctypes.c_int
    lib.dsattn_forward_ctx.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.dsattn_copy_probe.restype = ctypes.c_int
    lib.dsattn_copy_probe.argtypes = [vp, vp, ctypes.c_int64, vp]
    lib.dsattn_groupnorm_workspace.restype = ctypes.c_int
    lib.dsattn_groupnorm_workspace.argtypes = [ctypes.POINTER(DsattnGnDesc),
                                               ctypes.POINTER(ctypes.c_size_t)]
    lib.dsattn_temporal_conv_info.restype = ctypes.c_int
    lib.dsattn_temporal_conv_info.argtypes = [ctypes.POINTER(DsattnConvDesc),
                                              ctypes.POINTER(DsattnConvInfo)]
    lib.dsattn_temporal_conv.restype = ctypes.c_int
    lib.dsattn_temporal_conv.argtypes = [ctypes.POINTER(DsattnConvDesc), vp, vp, vp, vp, vp]
    lib.dsattn_linear_info.restype = ctypes.c_int
    lib.dsattn_linear_info.argtypes = [ctypes.POINTER(DsattnLinearDesc),
                                       ctypes.POINTER(DsattnConvInfo)]
    lib.dsattn_linear.restype = ctypes.c_int
    lib.dsattn_linear.argtypes = [ctypes.POINTER(DsattnLinearDesc), vp, ctypes.POINTER(vp),
                                  ctypes.POINTER(vp), ctypes.POINTER(vp), vp]
    lib.dsattn_groupnorm.restype = ctypes.c_int
    lib.dsattn_groupnorm.argtypes = [ctypes.POINTER(DsattnGnDesc), vp, vp, vp, vp, vp, vp,
                                     ctypes.c_size_t, vp]
    lib.dsattn_groupnorm_static.restype = ctypes.c_int
    lib.dsattn_groupnorm_static.argtypes = [ctypes.POINTER(DsattnGnDesc), vp, vp, vp, vp, vp, vp]
    lib.dsattn_groupnorm_static_max_bytes.restype = ctypes.c_size_t
    lib.dsattn_groupnorm_static_max_bytes.argtypes = []
    lib.dsattn_strerror.restype = ctypes.c_char_p
    lib.dsattn_strerror.argtypes = [ctypes.c_int]
    lib.dsattn_last_error.restype = ctypes.c_char_p
    lib.dsattn_last_error.argtypes = []
    _lib = lib
    return lib


def _check(rc, where):
    if rc != DSATTN_OK:
        raise DsattnError(rc, where)


def _ptr(t):
    """Device/host address of a torch tensor, numpy array, int or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        if not t.is_contiguous():
            raise ValueError("tensor must be contiguous")
        return t.data_ptr()
    if isinstance(t, np.ndarray):
        if not t.flags["C_CONTIGUOUS"]:
            raise ValueError("array must be contiguous")
        return t.ctypes.data
    raise TypeError(f"cannot take the address of {type(t)}")


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream  # a hipStream_t on ROCm builds
    if hasattr(stream, "cuda_stream"):
        return stream.cuda_stream
    return int(stream)


class Plan:
    """Owns one dsattn_plan_t handle."""

    def __init__(self, handle, desc, n_global):
        self.handle = handle
        self.desc = desc
        self.n_global = n_global

    def close(self):
        if self.handle:
            load().dsattn_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def F(self):
        return self.desc.clip_len * self.desc.n_clips

    @property
    def C(self):
        return self.desc.heads * self.desc.head_dim


def dsattn_plan(clip_len, n_clips, local_ctx, spatial, heads, head_dim, global_idx,
                io_dtype=DSATTN_BF16, out_dtype=None, scale=0.0, flags=0, device=0,
                bias_local=0.0, bias_global=0.0, window=None) -> Plan:
    """window: sliding-window radius of the local scope (sets DSATTN_FLAG_SLIDING_WINDOW), or None."""
    lib = load()
    if out_dtype is None:
        out_dtype = io_dtype
    desc = DsattnDesc(clip_len, n_clips, local_ctx, spatial, heads, head_dim, io_dtype, out_dtype,
                      float(scale), flags | (DSATTN_FLAG_SLIDING_WINDOW if window is not None else 0),
                      float(bias_local), float(bias_global), int(window) if window is not None else 0)
    g = np.ascontiguousarray(np.asarray(global_idx, dtype=np.int32).reshape(-1))
    handle = ctypes.c_void_p()
    rc = lib.dsattn_plan(ctypes.byref(desc), g.ctypes.data if g.size else None, int(g.size),
                         int(device), ctypes.byref(handle))
    _check(rc, "dsattn_plan")
    return Plan(handle, desc, int(g.size))


def dsattn_plan_destroy(plan: Plan):
    plan.close()


def dsattn_plan_ctx_max(plan: Plan) -> int:
    out = ctypes.c_int32()
    _check(load().dsattn_plan_ctx_max(plan.handle, ctypes.byref(out)), "dsattn_plan_ctx_max")
    return int(out.value)


def dsattn_plan_ctx_indices(plan: Plan):
    lk = dsattn_plan_ctx_max(plan)
    idx = np.empty((plan.desc.n_clips, lk), dtype=np.int32)
    ln = np.empty((plan.desc.n_clips,), dtype=np.int32)
    _check(load().dsattn_plan_ctx_indices(plan.handle, idx.ctypes.data, ln.ctypes.data),
           "dsattn_plan_ctx_indices")
    return idx, ln


def dsattn_plan_launch_info(plan: Plan) -> dict:
    info = DsattnLaunchInfo()
    _check(load().dsattn_plan_launch_info(plan.handle, ctypes.byref(info)),
           "dsattn_plan_launch_info")
    return info.as_dict()


def dsattn_gather_context(plan: Plan, K, V, Kctx, Vctx, stream=None):
    _check(load().dsattn_gather_context(plan.handle, _ptr(K), _ptr(V), _ptr(Kctx), _ptr(Vctx),
                                        _stream(stream)), "dsattn_gather_context")


def dsattn_forward(plan: Plan, Q, K, V, O, stream=None):
    _check(load().dsattn_forward(plan.handle, _ptr(Q), _ptr(K), _ptr(V), _ptr(O),
                                 _stream(stream)), "dsattn_forward")


def dsattn_forward_ctx(plan: Plan, Q, Kctx, Vctx, O, stream=None):
    _check(load().dsattn_forward_ctx(plan.handle, _ptr(Q), _ptr(Kctx), _ptr(Vctx), _ptr(O),
                                     _stream(stream)), "dsattn_forward_ctx")


def dsattn_copy_probe(dst, src, nbytes, stream=None):
    _check(load().dsattn_copy_probe(_ptr(dst), _ptr(src), int(nbytes), _stream(stream)),
           "dsattn_copy_probe")


def dsattn_strerror(code: int) -> str:
    return load().dsattn_strerror(int(code)).decode()


def dsattn_last_error() -> str:
    return load().dsattn_last_error().decode()


def dsattn_groupnorm_workspace(clip_len, n_clips, spatial, channels, groups, io_dtype=DSATTN_BF16,
                               eps=1e-5) -> int:
    desc = DsattnGnDesc(clip_len, n_clips, spatial, channels, groups, io_dtype, float(eps))
    out = ctypes.c_size_t()
    _check(load().dsattn_groupnorm_workspace(ctypes.byref(desc), ctypes.byref(out)),
           "dsattn_groupnorm_workspace")
    return int(out.value)


def dsattn_groupnorm(clip_len, n_clips, spatial, channels, groups, X, Y, workspace,
                     workspace_bytes, gamma=None, beta=None, stats=None, io_dtype=DSATTN_BF16,
                     eps=1e-5, stream=None):
    desc = DsattnGnDesc(clip_len, n_clips, spatial, channels, groups, io_dtype, float(eps))
    _check(load().dsattn_groupnorm(ctypes.byref(desc), _ptr(X), _ptr(gamma), _ptr(beta), _ptr(Y),
                                   _ptr(stats), _ptr(workspace), int(workspace_bytes),
                                   _stream(stream)), "dsattn_groupnorm")


def dsattn_groupnorm_static_max_bytes() -> int:
    return int(load().dsattn_groupnorm_static_max_bytes())


def dsattn_groupnorm_static(clip_len, n_clips, spatial, channels, groups, X, Y, gamma=None,
                            beta=None, stats=None, io_dtype=DSATTN_BF16, eps=1e-5, stream=None):
    desc = DsattnGnDesc(clip_len, n_clips, spatial, channels, groups, io_dtype, float(eps))
    _check(load().dsattn_groupnorm_static(ctypes.byref(desc), _ptr(X), _ptr(gamma), _ptr(beta),
                                          _ptr(Y), _ptr(stats), _stream(stream)),
           "dsattn_groupnorm_static")


def dsattn_temporal_conv_info(clip_len, n_clips, spatial, c_in, c_out, reach,
                              io_dtype=DSATTN_BF16, out_dtype=None, flags=0) -> dict:
    desc = DsattnConvDesc(clip_len, n_clips, spatial, c_in, c_out, reach, io_dtype,
                          io_dtype if out_dtype is None else out_dtype, flags)
    info = DsattnConvInfo()
    _check(load().dsattn_temporal_conv_info(ctypes.byref(desc), ctypes.byref(info)),
           "dsattn_temporal_conv_info")
    return info.as_dict()


def dsattn_temporal_conv(clip_len, n_clips, spatial, c_in, c_out, reach, X, W, Y, bias=None,
                         io_dtype=DSATTN_BF16, out_dtype=None, flags=0, stream=None):
    desc = DsattnConvDesc(clip_len, n_clips, spatial, c_in, c_out, reach, io_dtype,
                          io_dtype if out_dtype is None else out_dtype, flags)
    _check(load().dsattn_temporal_conv(ctypes.byref(desc), _ptr(X), _ptr(W), _ptr(bias), _ptr(Y),
                                       _stream(stream)), "dsattn_temporal_conv")


def dsattn_linear_info(rows, c_in, c_out, n_out, io_dtype=DSATTN_BF16, out_dtype=None, flags=0) -> dict:
    desc = DsattnLinearDesc(rows, c_in, c_out, n_out, io_dtype,
                            io_dtype if out_dtype is None else out_dtype, flags)
    info = DsattnConvInfo()
    _check(load().dsattn_linear_info(ctypes.byref(desc), ctypes.byref(info)), "dsattn_linear_info")
    return info.as_dict()


def _ptr_array(items, n):
    arr = (ctypes.c_void_p * n)()
    for i in range(n):
        arr[i] = _ptr(items[i])
    return arr


def dsattn_linear(rows, c_in, c_out, X, Ws, Ys, biases=None, io_dtype=DSATTN_BF16, out_dtype=None,
                  flags=0, stream=None):
    """Ws, Ys (and biases, entries may be None): sequences of n_out tensors."""
    n = len(Ws)
    if len(Ys) != n or (biases is not None and len(biases) != n):
        raise ValueError("Ws, Ys and biases must have the same length")
    desc = DsattnLinearDesc(rows, c_in, c_out, n, io_dtype,
                            io_dtype if out_dtype is None else out_dtype, flags)
    _check(load().dsattn_linear(ctypes.byref(desc), _ptr(X), _ptr_array(Ws, n),
                                None if biases is None else _ptr_array(biases, n),
                                _ptr_array(Ys, n), _stream(stream)), "dsattn_linear")
