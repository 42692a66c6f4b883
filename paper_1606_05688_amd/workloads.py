"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the convolution method: it only names the layer shapes and draws the
random tensors both the GPU library and the CPU oracle are fed with.

Shapes follow the layer definition of Section IV: a batch of S inputs, each a tuple of f cubic images of
edge n, convolved with an f' x f bank of cubic kernels of edge k into S tuples of f' images of edge n-k+1.
Values: images U(-1, 1); kernels N(0, variance 1/(f k^3)) (fan-in scaling); biases N(0, variance 0.1);
all drawn in this order from numpy's default_rng(seed) in fp64 and rounded once to fp32.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    S: int
    f: int
    fo: int
    n: int
    k: int
    bias: bool = True
    relu: bool = True

    @property
    def n_out(self) -> int:
        return self.n - self.k + 1

    @property
    def out_voxels(self) -> int:
        return self.S * self.fo * self.n_out ** 3


# The five benchmark layers, smallest first.
CONFIGS = (
    Layer("cfg1_16c_f2x3_k3", S=1, f=2, fo=3, n=16, k=3, bias=False, relu=False),
    Layer("cfg2_64c_f8x8_k5", S=1, f=8, fo=8, n=64, k=5),
    Layer("cfg3_128c_f40x40_k3", S=1, f=40, fo=40, n=128, k=3),
    Layer("cfg4_S8_64c_f32x32_k7", S=8, f=32, fo=32, n=64, k=7),
    Layer("cfg5_320c_f48x48_k5", S=1, f=48, fo=48, n=320, k=5),
)


def make_inputs(layer: Layer, seed: int = 0):
    """Return (inp [S,f,n,n,n], w [fo,f,k,k,k], bias [fo] or None) as fp32 numpy arrays."""
    rng = np.random.default_rng(seed)
    n, k = layer.n, layer.k
    # Drawn channel by channel so the largest layer never holds an fp64 copy of the whole input.
    inp = np.empty((layer.S, layer.f, n, n, n), dtype=np.float32)
    for s in range(layer.S):
        for i in range(layer.f):
            inp[s, i] = rng.uniform(-1.0, 1.0, size=(n, n, n)).astype(np.float32)
    std_w = (layer.f * k ** 3) ** -0.5
    w = (rng.standard_normal((layer.fo, layer.f, k, k, k)) * std_w).astype(np.float32)
    bias = None
    if layer.bias:
        bias = (rng.standard_normal(layer.fo) * np.sqrt(0.1)).astype(np.float32)
    return inp, w, bias


def sample_points(layer: Layer, n_random: int = 1 << 20, seed: int = 1, block: int = 8, midplanes: bool = True):
    """Output positions (s, j, x, y, z) for checks of layers too large for a full CPU evaluation.

    Every output image contributes its 8 corner blocks (block^3 voxels each) and, at the centre of each of its
    6 faces, a patch of block x block voxels, two voxels deep.  One complete output image (the middle one of the
    last input of the batch) contributes its three mid-planes x = m/2, y = m/2, z = m/2.  n_random further
    positions are drawn uniformly over the whole output tensor.  Duplicates are removed; rows come back sorted.
    """
    m = layer.n_out
    b = min(block, m)
    dp = min(2, m)
    rng = np.random.default_rng(seed)
    c = m // 2
    lo, hi = np.arange(b), np.arange(m - b, m)
    mid = np.arange(max(c - b // 2, 0), max(c - b // 2, 0) + b)
    near, far = np.arange(dp), np.arange(m - dp, m)

    def grid(xs, ys, zs):
        return np.stack(np.meshgrid(xs, ys, zs, indexing="ij"), -1).reshape(-1, 3)

    per_image = [grid(xs, ys, zs) for xs in (lo, hi) for ys in (lo, hi) for zs in (lo, hi)]
    per_image += [grid(near, mid, mid), grid(far, mid, mid), grid(mid, near, mid), grid(mid, far, mid),
                  grid(mid, mid, near), grid(mid, mid, far)]
    per_image = np.unique(np.concatenate(per_image, 0), axis=0)
    pts = []
    for s in range(layer.S):
        for j in range(layer.fo):
            pts.append(np.concatenate([np.full((len(per_image), 1), s), np.full((len(per_image), 1), j),
                                       per_image], 1))
    if midplanes:
        s, j = layer.S - 1, layer.fo // 2
        full = np.arange(m)
        for g in (grid([c], full, full), grid(full, [c], full), grid(full, full, [c])):
            pts.append(np.concatenate([np.full((len(g), 1), s), np.full((len(g), 1), j), g], 1))
    if n_random > 0:
        r = np.stack([rng.integers(0, layer.S, n_random), rng.integers(0, layer.fo, n_random),
                      rng.integers(0, m, n_random), rng.integers(0, m, n_random),
                      rng.integers(0, m, n_random)], 1)
        pts.append(r)
    return np.unique(np.concatenate(pts, 0).astype(np.int32), axis=0)
