"""Seeded synthetic workloads: shapes, global-frame recipes and Q/K/V generators.

This module holds no attention arithmetic.  It is the one piece shared by the
library's tests/benchmark and by the CPU oracle's tests: both sides receive the
same tensors from here.

The tensors stand in for the per-level temporal-attention inputs of a
VideoCrafter2-style U-Net at 512x320 (the paper's base model and resolution,
Section 5.1): projected Q, K, V of shape [F, P, C] with P = H'*W', C = heads*D.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class Level:
    """One U-Net level's temporal-attention shape."""
    name: str
    spatial: Tuple[int, int]
    heads: int
    head_dim: int

    @property
    def P(self):
        return self.spatial[0] * self.spatial[1]

    @property
    def C(self):
        return self.heads * self.head_dim


@dataclass(frozen=True)
class Workload:
    name: str
    n_clips: int
    clip_len: int
    local_ctx: int           # w: frames from each neighbouring side
    n_global: int
    global_recipe: str       # "stride" | "random_sorted" | "explicit"
    dtype: str               # "f32" | "bf16"
    generator: str           # "iid" | "correlated"
    levels: Tuple[Level, ...]
    seed: int
    explicit_global: Tuple[int, ...] = field(default=())

    @property
    def F(self):
        return self.n_clips * self.clip_len


WORKLOADS = {
    # tiny fp32 case: 2 clips x 4 frames, 4x4, 1 head x 8, w = 1, G = {0, 4}
    "C0": Workload("C0", 2, 4, 1, 2, "explicit", "f32", "iid",
                   (Level("tiny", (4, 4), 1, 8),), seed=1000, explicit_global=(0, 4)),
    # 64 frames, 40x64, 8 x 40
    "C1": Workload("C1", 4, 16, 2, 16, "stride", "bf16", "correlated",
                   (Level("L1", (40, 64), 8, 40),), seed=1100),
    # 384 frames, 20x32, 8 x 80
    "C2": Workload("C2", 24, 16, 2, 16, "stride", "bf16", "correlated",
                   (Level("L2", (20, 32), 8, 80),), seed=1200),
    # 2,304 frames, 10x16, 8 x 160  (the configuration the headline metric is quoted on)
    "C3": Workload("C3", 144, 16, 2, 16, "stride", "bf16", "correlated",
                   (Level("L3", (10, 16), 8, 160),), seed=1300),
    # 2,304 frames, four U-Net levels in sequence, w = 4, 64 random sorted global frames
    "C4": Workload("C4", 144, 16, 4, 64, "random_sorted", "bf16", "correlated",
                   (Level("L1", (40, 64), 8, 40), Level("L2", (20, 32), 8, 80),
                    Level("L3", (10, 16), 8, 160), Level("L4", (5, 8), 8, 160)), seed=1400),
}


def stride_global_idx(F: int, G: int) -> np.ndarray:
    """G frames at uniform stride over the video: floor(j * F / G)."""
    return np.array([(j * F) // G for j in range(G)], dtype=np.int32)


def random_sorted_global_idx(F: int, G: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(F, size=G, replace=False)).astype(np.int32)


def global_idx_for(wl: Workload) -> np.ndarray:
    if wl.global_recipe == "explicit":
        return np.array(wl.explicit_global, dtype=np.int32)
    if wl.global_recipe == "stride":
        return stride_global_idx(wl.F, wl.n_global)
    if wl.global_recipe == "random_sorted":
        return random_sorted_global_idx(wl.F, wl.n_global, wl.seed + 3)
    raise ValueError(wl.global_recipe)


def torch_dtype(name: str):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def make_tensor(F: int, P: int, C: int, seed: int, generator: str, dtype: str, device="cpu",
                frame_noise: float = 0.1):
    """One [F, P, C] tensor.

    "iid":        N(0,1) per element.
    "correlated": a per-(position, channel) base N(0,1) shared by all frames plus
                  frame_noise * N(0,1) per element (slowly varying video latents).
    Drawn in fp32 on `device` with a generator seeded by `seed`, then rounded to `dtype`.
    """
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    out = torch.empty((F, P, C), dtype=torch_dtype(dtype), device=device)
    if generator == "iid":
        base = None
    elif generator == "correlated":
        base = torch.randn((P, C), generator=gen, device=device, dtype=torch.float32)
    else:
        raise ValueError(generator)
    # frame chunks bound the fp32 temporary
    chunk = max(1, min(F, (1 << 27) // max(1, P * C)))
    for f0 in range(0, F, chunk):
        f1 = min(F, f0 + chunk)
        x = torch.randn((f1 - f0, P, C), generator=gen, device=device, dtype=torch.float32)
        if base is not None:
            x = base.unsqueeze(0) + frame_noise * x
        out[f0:f1] = x.to(out.dtype)
    return out


def make_qkv(wl: Workload, level: Level, device="cpu", seed_offset: int = 0):
    """(Q, K, V) for one level of a workload; seeds: wl.seed + 10*level_index + {0,1,2}."""
    li = wl.levels.index(level)
    s = wl.seed + 10 * li + seed_offset
    return tuple(make_tensor(wl.F, level.P, level.C, s + t, wl.generator, wl.dtype, device)
                 for t in range(3))


def to_f64_numpy(t, heads: int):
    """Exact upcast of a [F, P, C] torch tensor to a [F, P, h, D] float64 numpy array."""
    import torch
    x = t.detach().to("cpu").to(torch.float64).numpy()
    F, P, C = x.shape
    return x.reshape(F, P, heads, C // heads)


def make_conv_weights(taps: int, c_out: int, c_in: int, seed: int, dtype: str, device="cpu"):
    """Weights [taps, c_out, c_in] ~ N(0, 1 / (taps * c_in)) (unit-variance outputs for unit-variance
    inputs) rounded to `dtype`, and an fp32 bias [c_out] ~ 0.1 * N(0, 1)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    w = torch.randn((taps, c_out, c_in), generator=gen, device=device, dtype=torch.float32)
    w = (w / float(taps * c_in) ** 0.5).to(torch_dtype(dtype))
    b = 0.1 * torch.randn((c_out,), generator=gen, device=device, dtype=torch.float32)
    return w, b
