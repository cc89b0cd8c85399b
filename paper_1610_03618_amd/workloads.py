"""Seeded synthetic inputs and the five benchmark configurations.

This module only makes inputs (random tensors with the shapes and value
distributions of the CNN layers in Table 1 and of AlexNet / VGG-16) and lists
which operation runs on which tensor.  It holds none of the arithmetic of the
transform, pooling or softmax themselves, so the CPU oracle's tests and the GPU
path's tests can both draw identical bits from it.

The activations of the paper's networks come from MNIST / CIFAR10 / ImageNet
images (Section III.A); here synthetic tensors of the same shapes stand in for
them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

NCHW, CHWN = 0, 1
POOL_MAX, POOL_AVG = 0, 1

SEED_BASE = 161003618 * 10


def rng_for(config: int, stream: int = 0) -> np.random.Generator:
    """Generator for benchmark configuration ``config`` (1..5)."""
    return np.random.default_rng([SEED_BASE + config, stream])


def uniform_pm1(rng: np.random.Generator, shape) -> np.ndarray:
    """float32 values uniform in [-1, 1)."""
    x = rng.random(shape, dtype=np.float32)
    x *= 2.0
    x -= 1.0
    return x


def relu_normal(rng: np.random.Generator, shape) -> np.ndarray:
    """Standard normal draws clamped at zero: the value mix behind a ReLU layer."""
    x = rng.standard_normal(shape, dtype=np.float32)
    np.maximum(x, 0.0, out=x)
    return x


def normal_logits(rng: np.random.Generator, n: int, classes: int, sigma: float) -> np.ndarray:
    z = rng.standard_normal((n, classes), dtype=np.float32)
    z *= np.float32(sigma)
    return z


def plant_outliers(z: np.ndarray, rng: np.random.Generator) -> np.ndarray:
    """Rows r with r % 8 == 0 get 1 + (r/8) % 5 outliers at distinct columns.

    Even groups add 50 to the drawn logit; odd groups overwrite it with exactly
    50.0 so that the row maximum is tied between several columns.
    """
    n, classes = z.shape
    for r in range(0, n, 8):
        g = r // 8
        k = min(1 + g % 5, classes)
        cols = rng.choice(classes, size=k, replace=False)
        if g % 2 == 0:
            z[r, cols] += np.float32(50.0)
        else:
            z[r, cols] = np.float32(50.0)
    return z


@dataclass(frozen=True)
class TensorSpec:
    """One 4-D activation tensor: logical N x C x H x W plus a value recipe."""
    name: str
    N: int
    C: int
    H: int
    W: int
    values: str  # "uniform" or "relu_normal"

    @property
    def numel(self) -> int:
        return self.N * self.C * self.H * self.W


@dataclass(frozen=True)
class PoolSpec:
    tensor: TensorSpec
    mode: int
    k: int
    s: int
    p: int = 0


@dataclass(frozen=True)
class SoftmaxSpec:
    name: str
    N: int
    classes: int
    sigma: float
    outliers: bool = False


@dataclass
class Config:
    index: int
    description: str
    pools: List[PoolSpec] = field(default_factory=list)
    transforms: List[TensorSpec] = field(default_factory=list)
    softmaxes: List[SoftmaxSpec] = field(default_factory=list)


def _cfg1() -> Config:
    x = TensorSpec("x", 16, 64, 32, 32, "uniform")
    return Config(1, "max-pool 3x3/s2 on 16x64x32x32, both layouts",
                  pools=[PoolSpec(x, POOL_MAX, 3, 2)], transforms=[x])


def _cfg2() -> Config:
    x = TensorSpec("x", 128, 96, 55, 55, "uniform")
    return Config(2, "transform round trip on 128x96x55x55 + softmax 128x1000",
                  transforms=[x], softmaxes=[SoftmaxSpec("z", 128, 1000, 2.0)])


def _cfg3() -> Config:
    ts = [TensorSpec("x1", 128, 96, 55, 55, "relu_normal"),
          TensorSpec("x2", 128, 256, 27, 27, "relu_normal"),
          TensorSpec("x3", 128, 256, 13, 13, "relu_normal")]
    return Config(3, "AlexNet pooling stack, max 3x3/s2, N=128, both layouts + transforms",
                  pools=[PoolSpec(t, POOL_MAX, 3, 2) for t in ts], transforms=ts)


def _cfg4() -> Config:
    shapes = [(64, 224), (128, 112), (256, 56), (512, 28), (512, 14)]
    ts = [TensorSpec(f"x{i + 1}", 64, c, hw, hw, "relu_normal") for i, (c, hw) in enumerate(shapes)]
    pools = [PoolSpec(t, m, 2, 2) for t in ts for m in (POOL_MAX, POOL_AVG)]
    return Config(4, "VGG-16 pooling, max and avg 2x2/s2, N=64", pools=pools)


def _cfg5() -> Config:
    x = TensorSpec("x", 256, 512, 14, 14, "relu_normal")
    return Config(5, "softmax 4096x21841 with planted outliers + transform 256x512x14x14",
                  transforms=[x], softmaxes=[SoftmaxSpec("z", 4096, 21841, 3.0, outliers=True)])


def config(index: int) -> Config:
    return {1: _cfg1, 2: _cfg2, 3: _cfg3, 4: _cfg4, 5: _cfg5}[index]()


def make_tensor(spec: TensorSpec, rng: np.random.Generator) -> np.ndarray:
    """The tensor's values in NCHW order, shape (N, C, H, W), float32."""
    shape = (spec.N, spec.C, spec.H, spec.W)
    if spec.values == "uniform":
        return uniform_pm1(rng, shape)
    if spec.values == "relu_normal":
        return relu_normal(rng, shape)
    raise ValueError(spec.values)


def make_logits(spec: SoftmaxSpec, rng: np.random.Generator) -> np.ndarray:
    z = normal_logits(rng, spec.N, spec.classes, spec.sigma)
    if spec.outliers:
        plant_outliers(z, rng)
    return z


# Pooling and classifier shapes of Table 1: (N, H=W, window, C, stride).
TABLE1_POOLS: List[Tuple[str, int, int, int, int, int]] = [
    ("PL1", 128, 28, 2, 16, 2), ("PL2", 128, 14, 2, 16, 2), ("PL3", 128, 24, 3, 64, 2),
    ("PL4", 128, 12, 3, 64, 2), ("PL5", 128, 55, 3, 96, 2), ("PL6", 128, 27, 3, 192, 2),
    ("PL7", 128, 13, 3, 256, 2), ("PL8", 64, 110, 3, 96, 2), ("PL9", 64, 26, 3, 256, 2),
    ("PL10", 64, 13, 3, 256, 2),
]
TABLE1_CLASSIFIERS: List[Tuple[str, int, int]] = [
    ("CLASS1", 128, 10), ("CLASS2", 128, 10), ("CLASS3", 128, 1000),
    ("CLASS4", 64, 1000), ("CLASS5", 32, 1000),
]


# Softmax sweep in the spirit of Fig. 13: batch size x number of categories.  The figure's own list of
# configurations is not legible in the text, so this grid spans its stated range (up to 10000 categories).
SOFTMAX_SWEEP: List[Tuple[int, int]] = [(n, c) for n in (32, 64, 128, 256) for c in (10, 100, 1000, 10000)]
