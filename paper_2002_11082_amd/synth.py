"""Seeded synthetic gradients with the sizes and value distributions of the benchmark workloads.

Input generation only: nothing of the quantization method lives here, so both the GPU path and the
CPU checker can be fed the same arrays.  Real gradients are sharply peaked at zero and far from
Gaussian (Section 5.1.2 of the paper), hence the heavy-tailed and mixture recipes.  Sizes follow
Table 1 of the paper (AlexNet 61.1 M, VGG-19 143.7 M, ResNet-50 25.6 M parameters).
All generators use numpy.random.default_rng(seed) and return contiguous float32 arrays.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BINGRAD_B = 0
ORQ = 1
BINGRAD_PB = 2
ORQ_PAPER = 3
SCALED_SIGN = 4
EVEN = 5
LINEAR = 6


def gaussian(n: int, sigma: float, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(n, dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def laplace_heavy_tail(n: int, scale: float, seed: int, frac: float = 0.01, factor: float = 20.0) -> np.ndarray:
    """Laplace(0, scale) with a uniformly random `frac` of the entries multiplied by `factor`."""
    rng = np.random.default_rng(seed)
    g = rng.laplace(0.0, scale, n).astype(np.float32)
    mask = rng.random(n, dtype=np.float32) < np.float32(frac)
    g[mask] *= np.float32(factor)
    return g


def gaussian_mixture(n: int, seed: int, sigma_a: float = 1e-4, sigma_b: float = 1e-2, p_a: float = 0.9) -> np.ndarray:
    rng = np.random.default_rng(seed)
    g = rng.standard_normal(n, dtype=np.float32)
    wide = rng.random(n, dtype=np.float32) >= np.float32(p_a)
    g *= np.where(wide, np.float32(sigma_b), np.float32(sigma_a))
    return g.astype(np.float32)


# VGG-19: sixteen 3x3 convolutions (in -> out channels) and three fully connected layers.
VGG19_CONV = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256), (256, 256),
              (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
VGG19_FC = [(25088, 4096), (4096, 4096), (4096, 1000)]


def vgg19_layer_sizes():
    """(number of weights, fan_in) per layer, in order."""
    layers = [(9 * cin * cout, 9 * cin) for cin, cout in VGG19_CONV]
    layers += [(fin * fout, fin) for fin, fout in VGG19_FC]
    return layers


def vgg19_shaped(n: int, seed: int, scale_elements: float = 1.0) -> np.ndarray:
    """Concatenation of per-layer tensors, each Student-t(nu=3) / sqrt(fan_in); elements beyond the
    layer weights (biases, rounding of the published parameter count) use the last layer's scale.
    `scale_elements` < 1 shrinks every layer proportionally (for small test cases)."""
    rng = np.random.default_rng(seed)
    out = np.empty(n, dtype=np.float32)
    pos = 0
    fan_in = 1
    for size, fan_in in vgg19_layer_sizes():
        size = int(size * scale_elements)
        take = min(size, n - pos)
        if take <= 0:
            break
        out[pos:pos + take] = (rng.standard_t(3, take) / np.sqrt(fan_in)).astype(np.float32)
        pos += take
    if pos < n:
        out[pos:] = (rng.standard_t(3, n - pos) / np.sqrt(fan_in)).astype(np.float32)
    return out


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    bucket_size: int
    bits: int
    scheme: int
    level_iters: int
    workers: int
    seed: int            # Philox seed of worker 0 (worker w uses seed + w)
    description: str
    clip_factor: float = 0.0
    data: str = ""       # name of the workload whose gradient recipe is reused ("" = own)

    def gradient(self, worker: int = 0, n: int | None = None) -> np.ndarray:
        n = self.n if n is None else n
        if self.data:
            return WORKLOADS[self.data].gradient(worker, n)
        if self.name == "cfg1":
            return gaussian(n, 1e-3, 0)
        if self.name == "cfg2":
            return laplace_heavy_tail(n, 5e-4, 1)
        if self.name == "cfg3":
            return gaussian_mixture(n, 2)
        if self.name == "cfg4":
            return vgg19_shaped(n, 3, scale_elements=n / self.n)
        if self.name == "cfg5":
            return gaussian(n, 1e-3, 100 + worker)
        raise KeyError(self.name)

    def philox_seed(self, worker: int = 0) -> int:
        return self.seed + worker


WORKLOADS = {
    "cfg1": Workload("cfg1", 1_048_576, 512, 1, BINGRAD_B, 0, 1, 0,
                     "BinGrad-b 1-bit, 1,048,576 x N(0,1e-3^2), bucket 512"),
    "cfg2": Workload("cfg2", 25_600_000, 2048, 1, BINGRAD_B, 0, 1, 0,
                     "BinGrad-b 1-bit, ResNet-50-sized 25.6M x Laplace(0,5e-4) with 1% x20, bucket 2048"),
    "cfg3": Workload("cfg3", 25_600_000, 2048, 2, ORQ, 2, 1, 2,
                     "ORQ 2-bit (s=4), 25.6M x 0.9 N(0,1e-4^2) + 0.1 N(0,1e-2^2), bucket 2048, 2 sweeps"),
    "cfg4": Workload("cfg4", 143_700_000, 4096, 3, ORQ, 2, 1, 3,
                     "ORQ 3-bit (s=8), VGG-19-shaped 143.7M x Student-t(3)/sqrt(fan_in), bucket 4096, 2 sweeps"),
    "cfg5": Workload("cfg5", 61_100_000, 2048, 2, ORQ, 2, 8, 200,
                     "8 workers x AlexNet-sized 61.1M x N(0,1e-3^2), ORQ 2-bit, bucket 2048, decode-average"),
    # the rows added after the five configurations (same inputs, other quantizers)
    "pb2": Workload("pb2", 25_600_000, 2048, 1, BINGRAD_PB, 0, 1, 4,
                    "BinGrad-pb 1-bit on the cfg2 gradient, bucket 2048", data="cfg2"),
    "orq5": Workload("orq5", 25_600_000, 2048, 3, ORQ_PAPER, 0, 1, 5,
                     "ORQ-5 (Algorithm 1 as printed, 5 levels in 3 bits) on the cfg3 gradient, bucket 2048", data="cfg3"),
    "orq3clip": Workload("orq3clip", 25_600_000, 512, 2, ORQ_PAPER, 0, 1, 6,
                         "ORQ-3 with clipping c=2.5, bucket 512 (the paper's ImageNet setting) on the cfg3 gradient",
                         clip_factor=2.5, data="cfg3"),
    "cfg2clip": Workload("cfg2clip", 25_600_000, 2048, 1, BINGRAD_B, 0, 1, 0,
                         "BinGrad-b 1-bit with clipping c=2.5 on the cfg2 gradient, bucket 2048",
                         clip_factor=2.5, data="cfg2"),
    "bin512": Workload("bin512", 25_600_000, 512, 1, BINGRAD_B, 0, 1, 0,
                       "BinGrad-b 1-bit on the cfg2 gradient, bucket 512 (the paper's ImageNet bucket size)", data="cfg2"),
    "orq3d32k": Workload("orq3d32k", 25_600_000, 32768, 2, ORQ_PAPER, 0, 1, 9,
                         "ORQ-3 on the cfg3 gradient, bucket 32768 (the largest of the paper's bucket-size sweep)", data="cfg3"),
    "orq3d128": Workload("orq3d128", 25_600_000, 128, 2, ORQ_PAPER, 0, 1, 10,
                         "ORQ-3 on the cfg3 gradient, bucket 128 (the smallest of the paper's bucket-size sweep)", data="cfg3"),
    # the level rules the paper compares against, on the same kernels and inputs
    "sign2": Workload("sign2", 25_600_000, 2048, 1, SCALED_SIGN, 0, 1, 0,
                      "Scaled SignSGD per bucket on the cfg2 gradient, bucket 2048", data="cfg2"),
    "tern3": Workload("tern3", 25_600_000, 2048, 2, EVEN, 0, 1, 7,
                      "TernGrad / QSGD-3 (3 evenly spaced levels) on the cfg3 gradient, bucket 2048", data="cfg3"),
    "linear5": Workload("linear5", 25_600_000, 2048, 3, LINEAR, 0, 1, 8,
                        "Linear-5 (5 equal-mass levels) on the cfg3 gradient, bucket 2048", data="cfg3"),
}
