"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measures on ResNet-50/ImageNet and BERT/GLUE activations; an element-wise
kernel only sees the shape and the value distribution of the pre-activation tensor, so
seeded Gaussians of those shapes stand in for them.  This module holds NO arithmetic of
the method: it only draws numbers and rounds them to the storage dtype.  The
storage-rounded array is the input of record for the GPU path and the oracle alike.

Generator: numpy.random.default_rng(seed).standard_normal(n, float32) * std, then
round-to-nearest-even to the storage dtype (torch CPU cast).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np
import torch

GELU_TANH, GELU_ERF, SWISH, MISH = 0, 1, 2, 3
TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@dataclass(frozen=True)
class TensorSpec:
    shape: Tuple[int, ...]
    seed_x: int
    seed_gy: int

    @property
    def n(self) -> int:
        return int(np.prod(self.shape))


@dataclass(frozen=True)
class Config:
    name: str
    kinds: Tuple[int, ...]
    dtypes: Tuple[str, ...]
    tensors: Tuple[TensorSpec, ...]
    std_x: float
    std_gy: float
    outliers: bool = False      # 1% of entries replaced by sign * U[20, 80]
    note: str = ""


# The five benchmark configurations (index = position in the list of configs).
CONFIGS: List[Config] = [
    Config("C1 gelu_tanh f32 1-D 1Mi", (GELU_TANH,), ("f32",),
           (TensorSpec((1_048_576,), 0, 1),), 1.0, 1.0),
    Config("C2 swish f32 [32,256,56,56] ResNet-50 stage-1", (SWISH,), ("f32",),
           (TensorSpec((32, 256, 56, 56), 100, 101),), 1.0, 0.1),
    Config("C3 mish bf16 ResNet-50 activations", (MISH,), ("bf16",),
           (TensorSpec((64, 64, 112, 112), 200, 201),
            TensorSpec((64, 512, 28, 28), 202, 203),
            TensorSpec((64, 2048, 7, 7), 204, 205)), 1.5, 0.1),
    Config("C4 gelu_erf bf16+f16 BERT-base FFN [16384,3072]", (GELU_ERF,), ("bf16", "f16"),
           (TensorSpec((16384, 3072), 300, 301),), 1.0, 0.05),
    Config("C5 all four bf16 BERT-large FFN [32768,4096] with outliers",
           (GELU_TANH, GELU_ERF, SWISH, MISH), ("bf16",),
           (TensorSpec((32768, 4096), 400, 401),), 3.0, 0.1, outliers=True),
]


def gaussian(n: int, std: float, seed: int) -> np.ndarray:
    """float32 N(0, std) of n elements."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(n, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def add_outliers(a: np.ndarray, seed_mask: int, seed_mag: int, seed_sign: int) -> np.ndarray:
    """Replace ~1% of the entries (Bernoulli(0.01)) by sign * U[20, 80]; in place."""
    n = a.size
    mask = np.random.default_rng(seed_mask).random(n, dtype=np.float32) < np.float32(0.01)
    k = int(mask.sum())
    mag = np.random.default_rng(seed_mag).uniform(20.0, 80.0, k).astype(np.float32)
    sign = np.where(np.random.default_rng(seed_sign).random(k) < 0.5, -1.0, 1.0).astype(np.float32)
    a[mask] = mag * sign
    return a


def to_storage(a32: np.ndarray, dtype: str) -> torch.Tensor:
    """Round a float32 numpy array to the storage dtype (nearest even); CPU torch tensor."""
    t = torch.from_numpy(np.ascontiguousarray(a32))
    return t.to(TORCH_DTYPE[dtype]).contiguous()


def storage_to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a storage tensor (any device) to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def make_x(cfg: Config, spec: TensorSpec, dtype: str, n: int | None = None) -> torch.Tensor:
    """Pre-activation tensor of the config, flat, on the CPU, in storage dtype.
    n < spec.n draws only the first n elements (same stream prefix)."""
    n = spec.n if n is None else n
    a = gaussian(n, cfg.std_x, spec.seed_x)
    if cfg.outliers:
        add_outliers(a, spec.seed_x + 2, spec.seed_x + 3, spec.seed_x + 4)
    return to_storage(a, dtype)


def make_gy(cfg: Config, spec: TensorSpec, dtype: str, n: int | None = None) -> torch.Tensor:
    n = spec.n if n is None else n
    return to_storage(gaussian(n, cfg.std_gy, spec.seed_gy), dtype)
