"""The seeded generators: deterministic, of the stated shape and distribution, storage-exact."""
import numpy as np
import torch

from paper_2209_10778_amd import inputs


def test_config_shapes():
    n = [[t.n for t in c.tensors] for c in inputs.CONFIGS]
    assert n == [[1_048_576], [25_690_112], [51_380_224, 25_690_112, 6_422_528], [50_331_648], [134_217_728]]
    assert inputs.CONFIGS[0].tensors[0].seed_x == 0 and inputs.CONFIGS[0].tensors[0].seed_gy == 1


def test_deterministic_and_prefix_stable():
    cfg = inputs.CONFIGS[1]
    a = inputs.make_x(cfg, cfg.tensors[0], "f32", n=10000)
    b = inputs.make_x(cfg, cfg.tensors[0], "f32", n=10000)
    assert torch.equal(a, b)
    assert abs(float(a.std()) - 1.0) < 0.05 and abs(float(a.mean())) < 0.05
    g = inputs.make_gy(cfg, cfg.tensors[0], "f32", n=10000)
    assert abs(float(g.std()) - 0.1) < 0.01


def test_outliers_and_storage_rounding():
    cfg = inputs.CONFIGS[4]
    x = inputs.make_x(cfg, cfg.tensors[0], "bf16", n=400_000)
    assert x.dtype == torch.bfloat16
    big = (x.float().abs() >= 19.9)
    frac = float(big.float().mean())
    assert 0.007 < frac < 0.013
    assert float(x.float().abs().max()) <= 80.5
    assert bool((x.float()[big] > 0).any()) and bool((x.float()[big] < 0).any())
    # widening is exact
    x64 = inputs.storage_to_f64(x)
    assert np.array_equal(x64.astype(np.float32), x.float().numpy())
