"""dsattn: Dual-scope temporal self-attention (Video-Infinity, arXiv 2406.16260, Section 4.2)
as hand-written HIP kernels for gfx950 behind a C ABI (include/dsattn.h).

`binding` mirrors the C entry points; `synth` holds the seeded synthetic workloads;
`build` compiles libdsattn.so in-tree.  Attribute access is lazy so that importing the
package (e.g. for `synth`) does not require the built library.
"""
import importlib

_BINDING_NAMES = (
    "dsattn_plan", "dsattn_plan_destroy", "dsattn_plan_ctx_max", "dsattn_plan_ctx_indices",
    "dsattn_plan_launch_info", "dsattn_gather_context", "dsattn_forward", "dsattn_forward_ctx",
    "dsattn_copy_probe", "dsattn_strerror", "dsattn_last_error", "dsattn_groupnorm",
    "dsattn_groupnorm_workspace", "Plan", "DsattnError",
    "DSATTN_F32", "DSATTN_BF16", "DSATTN_FLAG_FORCE_GENERIC", "DSATTN_FLAG_SLIDING_WINDOW",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        return getattr(importlib.import_module(".binding", __name__), name)
    if name in ("binding", "synth", "build"):
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
