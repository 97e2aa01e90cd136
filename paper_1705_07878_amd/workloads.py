"""Seeded synthetic gradient workloads.

Input generators only: layer shapes of the networks the paper trains
(LeNet, AlexNet, GoogLeNet-like, VGG-A; Sections 4.1, 4.2, 5) and
Gaussian-like gradient values with a few heavy-tailed outliers (Figure 2 shows
near-Gaussian histograms).  Nothing of the method's arithmetic lives here and
this module imports neither the HIP binding nor the CPU oracle; both consume
the tensors it returns.

Every tensor of a network is one "layer" of the offset table: weights and
biases are ternarized separately (Section 3.3).
"""
from __future__ import annotations

import json
import math
import os
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_C3_MANIFEST = os.path.join(_HERE, "workload_googlenet_like.json")


@dataclass
class Workload:
    name: str
    layer_names: List[str]
    layer_sizes: List[int]
    n_workers: int
    clip_c: float = 2.5
    seed: int = 0
    step: int = 0
    outlier_frac: float = 1e-3
    outlier_scale: float = 10.0
    sigma_fixed: float | None = None     # None: sigma_l log-uniform in [1e-4, 1e-2]
    offsets: np.ndarray = field(init=False)

    def __post_init__(self):
        self.offsets = np.concatenate([[0], np.cumsum(np.asarray(self.layer_sizes, dtype=np.int64))]).astype(np.int64)

    @property
    def n(self) -> int:
        return int(self.offsets[-1])

    @property
    def n_layers(self) -> int:
        return len(self.layer_sizes)

    def layer_sigmas(self) -> np.ndarray:
        """sigma_l, drawn once per layer and shared by the workers (same model)."""
        if self.sigma_fixed is not None:
            return np.full(self.n_layers, self.sigma_fixed, dtype=np.float64)
        rng = np.random.default_rng([self.seed, 0x51674A])
        return 10.0 ** rng.uniform(-4.0, -2.0, size=self.n_layers)


def _with_biases(weights: Sequence[Tuple[str, Tuple[int, ...]]]):
    names, sizes = [], []
    for name, shape in weights:
        names.append(name + ".weight")
        sizes.append(int(np.prod(shape)))
        names.append(name + ".bias")
        sizes.append(int(shape[0]))
    return names, sizes


def lenet(n_workers: int = 2) -> Workload:
    w = [("conv1", (20, 1, 5, 5)), ("conv2", (50, 20, 5, 5)), ("fc1", (500, 800)), ("fc2", (10, 500))]
    names, sizes = _with_biases(w)
    return Workload("C1 LeNet-shaped", names, sizes, n_workers)


def alexnet(n_workers: int = 4) -> Workload:
    w = [("conv1", (96, 3, 11, 11)), ("conv2", (256, 48, 5, 5)), ("conv3", (384, 256, 3, 3)),
         ("conv4", (384, 192, 3, 3)), ("conv5", (256, 192, 3, 3)), ("fc6", (4096, 9216)),
         ("fc7", (4096, 4096)), ("fc8", (1000, 4096))]
    names, sizes = _with_biases(w)
    return Workload("C2 AlexNet-shaped", names, sizes, n_workers)


def googlenet_like_shapes(seed: int = 0, cap: int = 7_000_000):
    """58 conv shapes drawn from the seed; while the total exceeds the cap the
    currently largest layer is redrawn."""
    ch = [16, 32, 48, 64, 96, 128, 192, 256, 384]
    ks = [1, 3, 5]
    rng = np.random.default_rng([seed, 0x600613])

    def draw():
        return (int(rng.choice(ch)), int(rng.choice(ch)), int(rng.choice(ks)))

    shapes = [draw() for _ in range(58)]

    def total(sh):
        return sum(o * i * k * k + o for o, i, k in sh)

    while total(shapes) > cap:
        big = max(range(58), key=lambda j: shapes[j][0] * shapes[j][1] * shapes[j][2] ** 2)
        shapes[big] = draw()
    return shapes


def googlenet_like(n_workers: int = 4) -> Workload:
    """116 tensors; the shape manifest is a committed file so the workload does
    not depend on the numpy version that drew it."""
    with open(_C3_MANIFEST) as f:
        shapes = json.load(f)["conv_shapes_out_in_k"]
    w = [("conv%02d" % j, (o, i, k, k)) for j, (o, i, k) in enumerate(shapes)]
    names, sizes = _with_biases(w)
    return Workload("C3 GoogLeNet-like", names, sizes, n_workers)


def vgg_a(n_workers: int = 8) -> Workload:
    chans = [64, 128, 256, 256, 512, 512, 512, 512]
    w, cin = [], 3
    for j, c in enumerate(chans):
        w.append(("conv%d" % (j + 1), (c, cin, 3, 3)))
        cin = c
    w += [("fc6", (4096, 25088)), ("fc7", (4096, 4096)), ("fc8", (1000, 4096))]
    names, sizes = _with_biases(w)
    return Workload("C4 VGG-A-shaped", names, sizes, n_workers)


def flat(n: int = 1_000_000_000, n_workers: int = 8) -> Workload:
    return Workload("C5 flat %d" % n, ["flat"], [int(n)], n_workers,
                    outlier_frac=1e-4, outlier_scale=100.0, sigma_fixed=1e-3)


def custom(layer_sizes: Sequence[int], n_workers: int, name: str = "custom", **kw) -> Workload:
    return Workload(name, ["t%d" % j for j in range(len(layer_sizes))], [int(s) for s in layer_sizes],
                    n_workers, **kw)


BY_NAME = {"lenet": lenet, "alexnet": alexnet, "googlenet_like": googlenet_like, "vgg_a": vgg_a, "flat": flat}


def make_gradient(wl: Workload, worker: int, device="cpu", chunk: int = 1 << 26) -> torch.Tensor:
    """Worker `worker`'s flat fp32 gradient [n]: per layer N(0, sigma_l^2), a
    fraction `outlier_frac` of positions replaced by Student-t(3) * outlier_scale * sigma_l.
    Seeded by (wl.seed, worker); generated in chunks on `device`."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed((int(wl.seed) * 1_000_003 + int(worker) * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    n = wl.n
    g = torch.empty(n, dtype=torch.float32, device=dev)
    sig = wl.layer_sigmas()
    off = wl.offsets
    for l in range(wl.n_layers):
        lo, hi = int(off[l]), int(off[l + 1])
        s_l = float(sig[l])
        for a in range(lo, hi, chunk):
            b = min(hi, a + chunk)
            m = b - a
            z = torch.randn(m, generator=gen, device=dev, dtype=torch.float32)
            pick = torch.rand(m, generator=gen, device=dev, dtype=torch.float32) < wl.outlier_frac
            # Student-t(3) = Z / sqrt(chi2_3 / 3)
            num = torch.randn(m, generator=gen, device=dev, dtype=torch.float32)
            chi = torch.randn(3, m, generator=gen, device=dev, dtype=torch.float32).square_().sum(0)
            t3 = num / torch.sqrt(chi / 3.0)
            z = torch.where(pick, t3 * wl.outlier_scale, z)
            g[a:b] = z * s_l
            del z, pick, num, chi, t3
    return g


def make_gradients(wl: Workload, device="cpu") -> List[torch.Tensor]:
    return [make_gradient(wl, w, device) for w in range(wl.n_workers)]


def expected_zero_fraction(c_eff: float) -> float:
    """1 - E[min(|Z|, c)] / c for Z ~ N(0,1): share of codes that are 0 when the
    scaler equals c standard deviations (sanity figure, not a parity pin)."""
    phi = math.exp(-0.5 * c_eff * c_eff) / math.sqrt(2 * math.pi)
    q = 0.5 * math.erfc(c_eff / math.sqrt(2))
    e_min = 2 * (1 / math.sqrt(2 * math.pi) - phi) + 2 * c_eff * q
    return 1.0 - e_min / c_eff
