"""Seeded synthetic workloads: layer shapes, per-layer keep ratios and gradients.

This module holds NONE of the compressor's arithmetic: it only produces the
inputs (matrix shapes, keep ratios, float32 gradient matrices) that both the
GPU library and the CPU checker are fed with.  It depends on numpy and scipy
only.

The gradients stand in for the training gradients of the paper's networks
(Section IV: VGG and ResNet backbones on 21- and 45-class remote-sensing
scene datasets); the shapes are the standard VGG-19 / ResNet-18 / ResNet-50
weight layers with a 45-class head, each convolution weight viewed as an
out_ch x (in_ch*kh*kw) matrix (Section III-C: a layer's gradient is laid out
on a two-dimensional plane).

Recipe, per layer l and iteration t of a workload with seed s:
    rng    = default_rng(SeedSequence([s, t, l]))
    noise  = scale_l * Z            Z  i.i.d. N(0,1)  (or Student-t, nu = 3)
    smooth = scale_l * B / std(B)   B  = gaussian_filter(Z', sigma = 4 px,
                                        reflect boundary, truncated at 4 sigma)
    g      = float32(noise + smooth)
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np
from scipy import ndimage

Shape = Tuple[int, int]


# ------------------------------------------------------------------ shapes
def vgg19_shapes(num_classes: int = 45) -> List[Shape]:
    """16 conv layers (3x3) as out x (in*9), then fc6/fc7/fc8."""
    cfg = [64, 64, 128, 128, 256, 256, 256, 256, 512, 512, 512, 512, 512, 512, 512, 512]
    shapes, cin = [], 3
    for cout in cfg:
        shapes.append((cout, cin * 9))
        cin = cout
    shapes += [(25088, 4096), (4096, 4096), (4096, num_classes)]
    return shapes


def resnet18_shapes(num_classes: int = 45) -> List[Shape]:
    """conv1, four stages of two basic blocks (with 1x1 downsample convs), fc."""
    shapes = [(64, 3 * 49)]
    cin = 64
    for stage, planes in enumerate([64, 128, 256, 512]):
        for block in range(2):
            shapes.append((planes, cin * 9))
            shapes.append((planes, planes * 9))
            if block == 0 and stage > 0:
                shapes.append((planes, cin))
            cin = planes
    shapes.append((num_classes, 512))
    return shapes


def resnet50_shapes(num_classes: int = 45) -> List[Shape]:
    """conv1, bottleneck stages [3, 4, 6, 3] (with 1x1 downsample convs), fc."""
    shapes = [(64, 3 * 49)]
    cin = 64
    for planes, blocks in zip([64, 128, 256, 512], [3, 4, 6, 3]):
        for block in range(blocks):
            shapes.append((planes, cin))
            shapes.append((planes, planes * 9))
            shapes.append((planes * 4, planes))
            if block == 0:
                shapes.append((planes * 4, cin))
            cin = planes * 4
    shapes.append((num_classes, 2048))
    return shapes


# --------------------------------------------------------------- workloads
@dataclass
class Workload:
    name: str
    shapes: List[Shape]
    p: int
    alpha: float
    ratios: List[float]
    scales: List[float]
    seed: int
    iterations: int
    noise: str = "normal"          # "normal" or "student_t3"
    sigma_px: float = 4.0
    extra: dict = field(default_factory=dict)

    @property
    def n_layers(self) -> int:
        return len(self.shapes)

    @property
    def total_elems(self) -> int:
        return int(sum(r * c for r, c in self.shapes))


def layer_scales(n_layers: int, seed: int) -> List[float]:
    """s_l = 10**U(-5, -2), from a stream separate from the per-layer ones."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 10 ** 6]))
    return [float(x) for x in 10.0 ** rng.uniform(-5.0, -2.0, size=n_layers)]


def dynamic_ratios(shapes: Sequence[Shape], mean_ratio: float, seed: int) -> List[float]:
    """Per-layer keep ratios scattered log-normally around mean_ratio, clipped to
    [mean/8, 8*mean], then rescaled so that sum(rho_l * G_l) = mean_ratio * G."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 10 ** 6 + 1]))
    sizes = np.array([r * c for r, c in shapes], dtype=np.float64)
    rho = mean_ratio * np.exp(0.5 * rng.standard_normal(len(shapes)))
    rho = np.clip(rho, mean_ratio / 8.0, mean_ratio * 8.0)
    rho *= mean_ratio * sizes.sum() / float((rho * sizes).sum())
    return [float(min(1.0, x)) for x in rho]


def config(index: int) -> Workload:
    """The five benchmark configurations (0-based index)."""
    if index == 0:
        return Workload("single_512x512", [(512, 512)], 3, 0.5, [0.02], [1e-3], 0, 1)
    if index == 1:
        sh = resnet18_shapes()
        return Workload("resnet18_45c", sh, 3, 0.5, [0.01] * len(sh), layer_scales(len(sh), 2), 2, 2)
    if index == 2:
        sh = resnet50_shapes()
        return Workload("resnet50_45c", sh, 3, 0.5, dynamic_ratios(sh, 0.02, 3),
                        layer_scales(len(sh), 3), 3, 1)
    if index == 3:
        sh = vgg19_shapes()
        return Workload("vgg19_45c", sh, 3, 0.5, dynamic_ratios(sh, 0.02, 4),
                        layer_scales(len(sh), 4), 4, 10)
    if index == 4:
        return Workload("fc6_25088x4096_t3", [(25088, 4096)], 5, 0.5, [0.001], [1e-3], 5, 5,
                        noise="student_t3")
    raise ValueError("config index must be 0..4")


def scaled_down(w: Workload, max_rows: int, max_cols: int) -> Workload:
    """Same recipe on matrices clipped to max_rows x max_cols (for quick checks)."""
    sh = [(min(r, max_rows), min(c, max_cols)) for r, c in w.shapes]
    return Workload(w.name + f"_clip{max_rows}x{max_cols}", sh, w.p, w.alpha, list(w.ratios),
                    list(w.scales), w.seed, w.iterations, w.noise, w.sigma_px, dict(w.extra))


# --------------------------------------------------------------- gradients
def layer_gradient(shape: Shape, scale: float, seed: int, t: int, l: int,
                   noise: str = "normal", sigma_px: float = 4.0) -> np.ndarray:
    """One layer's float32 gradient matrix for iteration t."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, t, l]))
    if noise == "normal":
        z = rng.standard_normal(shape, dtype=np.float32)
    elif noise == "student_t3":
        z = rng.standard_t(3.0, size=shape).astype(np.float32)
    else:
        raise ValueError(noise)
    z2 = rng.standard_normal(shape, dtype=np.float32)
    b = ndimage.gaussian_filter(z2, sigma=sigma_px, mode="reflect", truncate=4.0)
    sd = float(b.std(dtype=np.float64))
    if sd > 0.0:
        b *= np.float32(1.0 / sd)
    g = (z + b) * np.float32(scale)
    return np.ascontiguousarray(g, dtype=np.float32)


def gradients(w: Workload, t: int) -> List[np.ndarray]:
    """All layers' gradients for iteration t."""
    return [layer_gradient(sh, s, w.seed, t, l, w.noise, w.sigma_px)
            for l, (sh, s) in enumerate(zip(w.shapes, w.scales))]
