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
    "dsattn_temporal_layer_workspace", "dsattn_temporal_layer",
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
        ("algorithmic_bytes", ctypes.c_int64), ("variant", ctypes.c_int32),
        ("ring_reach", ctypes.c_int32),
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
    lib.dsattn_temporal_layer_workspace.restype = ctypes.c_int
    lib.dsattn_temporal_layer_workspace.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
    lib.dsattn_temporal_layer.restype = ctypes.c_int
    lib.dsattn_temporal_layer.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                          ctypes.c_size_t, vp, vp]
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


def _dtype_name(code):
    return "float32" if code == DSATTN_F32 else "bfloat16"


def _check_tensors(who, items, device):
    """Refuse torch tensors that the kernels would read or write out of bounds: wrong element
    count, element type or device.  The C ABI takes bare pointers and cannot know any of these.
    items: (tensor, name, numel, dtype code or None); numel is exact unless given as ("min", n).
    device: the HIP ordinal the call runs on, "current" for entry points that run on the current
    device, or None to skip the device check (a host-only plan: the library itself refuses the
    call).  Sizes and types of all tensors are checked before any device.  Raw addresses (int) and
    None pass through: they are the C-level tests' business."""
    import torch
    tensors = [it for it in items if it[0] is not None and hasattr(it[0], "data_ptr")]
    for t, name, numel, dtype_code in tensors:
        if not t.is_contiguous():
            raise ValueError(f"{who}: {name}: tensor must be contiguous")
        if isinstance(numel, tuple):
            if t.numel() < numel[1]:
                raise ValueError(f"{who}: {name}: {t.numel()} elements, at least {numel[1]} needed")
        elif t.numel() != numel:
            raise ValueError(f"{who}: {name}: {t.numel()} elements, {numel} expected")
        if dtype_code is not None:
            want = torch.float32 if dtype_code == DSATTN_F32 else torch.bfloat16
            if t.dtype != want:
                raise ValueError(f"{who}: {name}: dtype {t.dtype}, {_dtype_name(dtype_code)} expected")
    if device is None:
        return
    for t, name, _, _ in tensors:
        if t.device.type != "cuda":
            raise ValueError(f"{who}: {name}: tensor is on {t.device}, device memory expected")
        dev = torch.cuda.current_device() if device == "current" else device
        if t.device.index != dev:
            raise ValueError(f"{who}: {name}: tensor is on {t.device}, the call runs on device {dev}")


class Plan:
    """Owns one dsattn_plan_t handle."""

    def __init__(self, handle, desc, n_global, device=0):
        self.handle = handle
        self.desc = desc
        self.n_global = n_global
        self.device = device
        self._lk_max = None

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

    @property
    def lk_max(self):
        if self._lk_max is None:
            self._lk_max = dsattn_plan_ctx_max(self)
        return self._lk_max

    def frames(self, t, name, out=False):
        """Check item for an [F, P, C] tensor of this plan (Q, K, V or O)."""
        return (t, name, self.F * self.desc.spatial * self.C,
                self.desc.out_dtype if out else self.desc.io_dtype)

    def ctx(self, t, name):
        """Check item for a materialised context [N, lk_max, P, C] of this plan."""
        return (t, name, self.desc.n_clips * self.lk_max * self.desc.spatial * self.C,
                self.desc.io_dtype)

    def check(self, who, items):
        _check_tensors(who, items, self.device if self.device >= 0 else None)


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
    return Plan(handle, desc, int(g.size), int(device))


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
    plan.check("dsattn_gather_context", [plan.frames(K, "K"), plan.frames(V, "V"),
                                         plan.ctx(Kctx, "Kctx"), plan.ctx(Vctx, "Vctx")])
    _check(load().dsattn_gather_context(plan.handle, _ptr(K), _ptr(V), _ptr(Kctx), _ptr(Vctx),
                                        _stream(stream)), "dsattn_gather_context")


def dsattn_forward(plan: Plan, Q, K, V, O, stream=None):
    plan.check("dsattn_forward", [plan.frames(Q, "Q"), plan.frames(K, "K"), plan.frames(V, "V"),
                                  plan.frames(O, "O", out=True)])
    _check(load().dsattn_forward(plan.handle, _ptr(Q), _ptr(K), _ptr(V), _ptr(O),
                                 _stream(stream)), "dsattn_forward")


def dsattn_forward_ctx(plan: Plan, Q, Kctx, Vctx, O, stream=None):
    plan.check("dsattn_forward_ctx", [plan.frames(Q, "Q"), plan.ctx(Kctx, "Kctx"),
                                      plan.ctx(Vctx, "Vctx"), plan.frames(O, "O", out=True)])
    _check(load().dsattn_forward_ctx(plan.handle, _ptr(Q), _ptr(Kctx), _ptr(Vctx), _ptr(O),
                                     _stream(stream)), "dsattn_forward_ctx")


def dsattn_copy_probe(dst, src, nbytes, stream=None):
    _check_tensors("dsattn_copy_probe",
                   [(t, name, ("min", -(-int(nbytes) // t.element_size())), None)
                    for t, name in ((dst, "dst"), (src, "src")) if hasattr(t, "element_size")],
                   "current")
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


def _gn_items(desc, X, Y, gamma, beta, stats):
    n = desc.clip_len * desc.n_clips * desc.spatial * desc.channels
    return [(X, "X", n, desc.io_dtype), (Y, "Y", n, desc.io_dtype),
            (gamma, "gamma", desc.channels, DSATTN_F32), (beta, "beta", desc.channels, DSATTN_F32),
            (stats, "stats", 2 * desc.groups, DSATTN_F32)]


def dsattn_groupnorm(clip_len, n_clips, spatial, channels, groups, X, Y, workspace,
                     workspace_bytes, gamma=None, beta=None, stats=None, io_dtype=DSATTN_BF16,
                     eps=1e-5, stream=None):
    desc = DsattnGnDesc(clip_len, n_clips, spatial, channels, groups, io_dtype, float(eps))
    items = _gn_items(desc, X, Y, gamma, beta, stats)
    if hasattr(workspace, "element_size"):
        items.append((workspace, "workspace",
                      ("min", -(-int(workspace_bytes) // workspace.element_size())), None))
    _check_tensors("dsattn_groupnorm", items, "current")
    _check(load().dsattn_groupnorm(ctypes.byref(desc), _ptr(X), _ptr(gamma), _ptr(beta), _ptr(Y),
                                   _ptr(stats), _ptr(workspace), int(workspace_bytes),
                                   _stream(stream)), "dsattn_groupnorm")


def dsattn_groupnorm_static_max_bytes() -> int:
    return int(load().dsattn_groupnorm_static_max_bytes())


def dsattn_groupnorm_static(clip_len, n_clips, spatial, channels, groups, X, Y, gamma=None,
                            beta=None, stats=None, io_dtype=DSATTN_BF16, eps=1e-5, stream=None):
    desc = DsattnGnDesc(clip_len, n_clips, spatial, channels, groups, io_dtype, float(eps))
    _check_tensors("dsattn_groupnorm_static", _gn_items(desc, X, Y, gamma, beta, stats), "current")
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
    rows = clip_len * n_clips * spatial
    _check_tensors("dsattn_temporal_conv",
                   [(X, "X", rows * c_in, desc.io_dtype),
                    (W, "W", (2 * reach + 1) * c_out * c_in, desc.io_dtype),
                    (bias, "bias", c_out, DSATTN_F32), (Y, "Y", rows * c_out, desc.out_dtype)],
                   "current")
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
    items = [(X, "X", rows * c_in, desc.io_dtype)]
    for g in range(n):
        items.append((Ws[g], f"W[{g}]", c_out * c_in, desc.io_dtype))
        items.append((Ys[g], f"Y[{g}]", rows * c_out, desc.out_dtype))
        if biases is not None:
            items.append((biases[g], f"bias[{g}]", c_out, DSATTN_F32))
    _check_tensors("dsattn_linear", items, "current")
    _check(load().dsattn_linear(ctypes.byref(desc), _ptr(X), _ptr_array(Ws, n),
                                None if biases is None else _ptr_array(biases, n),
                                _ptr_array(Ys, n), _stream(stream)), "dsattn_linear")


def dsattn_temporal_layer_workspace(plan):
    """Bytes of device workspace dsattn_temporal_layer needs for this plan."""
    n = ctypes.c_size_t(0)
    _check(load().dsattn_temporal_layer_workspace(plan.handle, ctypes.byref(n)),
           "dsattn_temporal_layer_workspace")
    return int(n.value)


def dsattn_temporal_layer(plan, X, Ws, workspace, Y, biases=None, stream=None):
    """Ws = (Wq, Wk, Wv, Wo), biases = None or four entries (each a tensor or None); workspace: a
    uint8 device tensor of at least dsattn_temporal_layer_workspace(plan) bytes."""
    if len(Ws) != 4 or (biases is not None and len(biases) != 4):
        raise ValueError("dsattn_temporal_layer: four weight sets (and four bias entries) expected")
    C = plan.C
    items = [plan.frames(X, "X"), plan.frames(Y, "Y")]
    for g in range(4):
        items.append((Ws[g], f"W[{g}]", C * C, plan.desc.io_dtype))
        if biases is not None:
            items.append((biases[g], f"bias[{g}]", C, DSATTN_F32))
    nbytes = 0
    if hasattr(workspace, "data_ptr"):
        if workspace.element_size() != 1:
            raise ValueError("dsattn_temporal_layer: workspace: a byte tensor (uint8) expected")
        nbytes = workspace.numel()
        items.append((workspace, "workspace", ("min", 0), None))
    plan.check("dsattn_temporal_layer", items)
    _check(load().dsattn_temporal_layer(plan.handle, _ptr(X), _ptr_array(Ws, 4),
                                        None if biases is None else _ptr_array(biases, 4),
                                        _ptr(workspace), nbytes, _ptr(Y), _stream(stream)),
           "dsattn_temporal_layer")
