"""Seeded synthetic conv-layer workloads (shapes and value distributions only).

This module holds no arithmetic of the method: it names layer shapes and draws
the three input tensors of a layer from a counter-based generator so that the
GPU path and the CPU oracle are handed bit-identical fp32 arrays.

The paper times layers described only by (k, n, f, f') at minibatch 128
(Sec. 3, per-layer timing table); no dataset contents enter any of its
numbers, so dense random tensors of the same shape stand in for them:
x ~ U[-1, 1], w ~ N(0, sigma_w^2), dL/dy ~ N(0, 1).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 0x13125851


@dataclass(frozen=True)
class Layer:
    """One convolutional layer in the paper's notation (Sec. 2.1)."""
    name: str
    S: int       # minibatch size
    f: int       # input feature maps
    fo: int      # output feature maps (f' in the paper)
    n: int       # input width (square maps)
    k: int       # kernel width (square kernels)
    sigma_w: float = 0.02
    seed: int = BASE_SEED

    @property
    def no(self) -> int:
        """Output width n' = n - k + 1 (stride 1, no spatial padding)."""
        return self.n - self.k + 1

    @property
    def direct_flops(self) -> int:
        """Direct-method multiply-adds of one pass, times two (Sec. 2.2 op-count table)."""
        return 2 * self.S * self.f * self.fo * self.no * self.no * self.k * self.k

    def shapes(self):
        return ((self.S, self.f, self.n, self.n),
                (self.fo, self.f, self.k, self.k),
                (self.S, self.fo, self.no, self.no))


TINY = Layer("tiny", 4, 8, 8, 16, 5, 0.05, BASE_SEED + 0)
MID = Layer("mid", 128, 96, 256, 32, 5, 0.02, BASE_SEED + 1)
FIRST = Layer("first", 128, 3, 96, 64, 11, 0.05, BASE_SEED + 2)
DEEP = Layer("deep", 128, 256, 384, 16, 3, 0.02, BASE_SEED + 3)

CONFIGS = {c.name: c for c in (TINY, MID, FIRST, DEEP)}


def sweep_layers():
    """Kernel-size x image-size sweep at S=128, f=f'=256 (stands in for the paper's Fig. 3 axes)."""
    out = []
    for n in (16, 32, 64):
        for k in (3, 5, 7, 9, 11, 13):
            if k < n:
                out.append(Layer(f"sweep_n{n}_k{k}", 128, 256, 256, n, k, 0.02,
                                 BASE_SEED + 100 + n * 16 + k))
    return out


def paper_table_layers():
    """The five (k, n, f, f') columns of the paper's per-layer timing table, S=128."""
    cols = ((11, 32, 3, 96), (7, 32, 96, 256), (5, 16, 256, 384), (5, 16, 384, 384), (3, 16, 384, 384))
    return [Layer(f"paper_k{k}_n{n}_f{f}_fo{fo}", 128, f, fo, n, k, 0.02, BASE_SEED + 200 + i)
            for i, (k, n, f, fo) in enumerate(cols)]


def fig3_layers():
    """The three axes of the paper's speed figure (Sec. 3): image size, kernel size and
    minibatch size, each varied alone around f=96, f'=256.  The figure's tick values are
    not given in the text; the points here bracket the table's layers and include image
    sizes that are not a power of two (Sec. 4 pads those up; n = 34 is its example)."""
    out = []
    for i, n in enumerate((8, 12, 14, 16, 20, 24, 28, 32, 34, 40, 48, 56, 64)):
        out.append(Layer(f"fig3_n{n}", 128, 96, 256, n, 5, 0.02, BASE_SEED + 300 + i))
    for i, k in enumerate((3, 7, 9, 11, 13)):          # k = 5 is the n = 32 point above
        out.append(Layer(f"fig3_k{k}", 128, 96, 256, 32, k, 0.02, BASE_SEED + 320 + i))
    for i, S in enumerate((16, 32, 64, 256)):          # S = 128 is the n = 32 point above
        out.append(Layer(f"fig3_S{S}", S, 96, 256, 32, 5, 0.02, BASE_SEED + 340 + i))
    return out


def large_layers():
    """Layers with maps larger than the largest transform (n > 64), which are computed in tiles:
    the far end of the figure's image-size axis and two image-sized first layers."""
    return [
        Layer("large_n96", 128, 96, 256, 96, 5, 0.02, BASE_SEED + 400),
        Layer("large_n128", 128, 96, 256, 128, 5, 0.02, BASE_SEED + 401),
        Layer("large_n224_k11_f3", 128, 3, 96, 224, 11, 0.05, BASE_SEED + 402),
        Layer("large_n112_k3_f64", 32, 64, 64, 112, 3, 0.05, BASE_SEED + 403),
    ]


def by_name(name: str) -> Layer:
    if name in CONFIGS:
        return CONFIGS[name]
    for lay in sweep_layers() + paper_table_layers() + fig3_layers() + large_layers():
        if lay.name == name:
            return lay
    raise KeyError(name)


def make_inputs(layer: Layer):
    """Return (x, w, g) as contiguous fp32 numpy arrays drawn from the layer's seed.

    Philox is counter-based: the stream depends only on the seed, not on the
    machine or on how many threads draw from it.
    """
    rng = np.random.Generator(np.random.Philox(key=layer.seed))
    xs, ws, gs = layer.shapes()
    x = rng.uniform(-1.0, 1.0, size=xs).astype(np.float32)
    w = (rng.standard_normal(size=ws) * layer.sigma_w).astype(np.float32)
    g = rng.standard_normal(size=gs).astype(np.float32)
    return x, w, g


def sample_units(total: int, count: int, seed: int):
    """A seeded sorted sample (without replacement) of ``count`` unit indices below ``total``."""
    rng = np.random.Generator(np.random.Philox(key=seed ^ 0x5EED))
    count = min(count, total)
    return np.sort(rng.choice(total, size=count, replace=False)).astype(np.int64)
