"""Seeded synthetic inputs for the activation path -- shared by tests, smoke and bench.

This module holds NO arithmetic of the method (no GELU, no quantizer, no
table): it only draws random activations and gradients with the shapes and
value distributions of ViT / Swin MLP hidden layers, and converts between
float32 and bf16 storage.  Both the GPU library and the CPU oracle are fed the
bit patterns produced here.

The tensors stand in for the post-fc1 activations of the paper's fine-tuning
runs (Sec. 4.1: ViT-B/16, Swin-B on VTAB-1k / FGVC); the datasets and the
pre-trained weights are not needed for an element-wise path and are not used.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np

F32 = 0
BF16 = 1

_SEED_BASE = 25030815400


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration.

    shapes  one entry per launch of a layer pass (ragged for Swin stages)
    layers  how many times the whole shape list runs back to back
    dist    "normal", "normal_outliers" or "student_t"
    scale   standard deviation (or scale of the t distribution) of x
    """
    name: str
    index: int
    dtype: int
    shapes: Tuple[Tuple[int, ...], ...]
    layers: int
    dist: str
    scale: float
    dy_scale: float

    def sizes(self):
        return [int(np.prod(s)) for s in self.shapes]


WORKLOADS = {
    w.name: w
    for w in (
        Workload("tiny", 0, F32, ((2, 197, 768),), 1, "normal", 1.0, 1.0),
        Workload("vit_b16", 1, BF16, ((64, 197, 3072),), 12, "normal_outliers", 1.5, 1e-2),
        Workload("vit_l16", 2, BF16, ((64, 197, 4096),), 24, "normal_outliers", 1.5, 1e-2),
        Workload("swin_b", 3, BF16,
                 ((64, 3136, 512), (64, 784, 1024), (64, 196, 2048), (64, 49, 4096)),
                 1, "normal", 1.0, 1e-2),
        Workload("vit_g14", 4, BF16, ((32, 257, 8192),), 1, "student_t", 2.0, 1e-2),
        Workload("vit_g14_f32", 4, F32, ((32, 257, 8192),), 1, "student_t", 2.0, 1e-2),
    )
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns.

    NaN keeps a quiet-NaN pattern; values that round past the largest bf16
    become infinity, as IEEE rounding prescribes.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    r = np.where(np.isnan(a), (u >> np.uint32(16)) | np.uint32(0x0040), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a64: np.ndarray, dtype: int) -> np.ndarray:
    """float64 samples -> storage array: float32, or uint16 bf16 bits."""
    a32 = a64.astype(np.float32)
    return a32 if dtype == F32 else f32_to_bf16_bits(a32)


def storage_to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    """Storage array -> the exact float64 values it denotes."""
    return (a if dtype == F32 else bf16_bits_to_f32(a)).astype(np.float64)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


def draw_x(n: int, dist: str, scale: float, dtype: int, seed: int) -> np.ndarray:
    """n activations in storage form.

    normal           N(0, scale^2)
    normal_outliers  N(0, scale^2) with 0.1 % of entries replaced by N(0, 8^2)
    student_t        scale * t(nu=4): Z / sqrt(V/4), V ~ chi^2_4 (heavy tails)
    """
    g = _rng(seed)
    if dist == "normal":
        a = g.standard_normal(n) * scale
    elif dist == "normal_outliers":
        a = g.standard_normal(n) * scale
        mask = g.random(n) < 1e-3
        a[mask] = g.standard_normal(int(mask.sum())) * 8.0
    elif dist == "student_t":
        z = g.standard_normal(n)
        v = g.chisquare(4.0, n)
        a = scale * z / np.sqrt(v / 4.0)
    else:
        raise ValueError(f"unknown distribution {dist!r}")
    return to_storage(a, dtype)


def draw_dy(n: int, scale: float, dtype: int, seed: int) -> np.ndarray:
    """n incoming gradients ~ N(0, scale^2) in storage form."""
    return to_storage(_rng(seed).standard_normal(n) * scale, dtype)


def layer_seed(w: Workload, layer: int, stage: int = 0, which: str = "x") -> int:
    """Seed of one tensor: distinct per workload, layer, stage and role."""
    return _SEED_BASE + 10_000 * w.index + 100 * layer + 10 * stage + (0 if which == "x" else 5)


def layer_inputs(w: Workload, layer: int = 0, stage: int = 0, n: int | None = None):
    """(x, dy) storage arrays for one launch of workload `w`; `n` truncates the draw."""
    size = w.sizes()[stage] if n is None else int(n)
    x = draw_x(size, w.dist, w.scale, w.dtype, layer_seed(w, layer, stage, "x"))
    dy = draw_dy(size, w.dy_scale, w.dtype, layer_seed(w, layer, stage, "dy"))
    return x, dy
