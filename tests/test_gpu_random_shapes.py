"""Seeded sweep over random small layer shapes (all storage types, both activations, with and without
routing biases, per-expert and group capacities from starving to generous): forward and backward pass
against the oracle.  Complements the hand-picked cases with shapes nobody thought of."""
import os
import sys

import numpy as np
import pytest

from paper_2212_05191_amd import binding as B
from paper_2212_05191_amd import workloads as wl

pytestmark = pytest.mark.gpu

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity  # noqa: E402
import test_gpu_backward as bwd  # noqa: E402


def _random_config(i):
    rng = np.random.default_rng(9000 + i)
    dtype = ["f32", "bf16", "f16"][i % 3]
    step = 8 if dtype == "f32" else 64
    d = int(step * rng.integers(1, 6 if dtype != "f32" else 30))
    F = int(step * rng.integers(1, 8 if dtype != "f32" else 40))
    n = int(rng.choice([1, 2, 3, 5, 8, 17, 33]))
    m = int(rng.choice([1, 2, 4, 7, 9, 40]))
    T = int(rng.integers(1, 3000))
    mean = max(1.0, T / (n * m))
    C = max(1, int(mean * rng.choice([0.3, 0.8, 1.0, 1.5, 4.0])))
    Cg = 0 if rng.random() < 0.6 else max(1, int(T / n * rng.choice([0.5, 1.0, 2.0])))
    return wl.small_config(f"rand{i}", T, d, F, n, m, C, dtype, ["relu", "gelu"][int(rng.integers(2))],
                           skew=bool(rng.integers(2)), seed=9000 + i, group_capacity=Cg)


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.load()
    return torch


@pytest.mark.parametrize("i", range(18))
def test_random_shape_forward_and_backward(torch_cuda, i):
    cfg = _random_config(i)
    layer = bwd._forward_backward(cfg, chained=bool(i % 2), dloss=0.7)
    try:
        info = parity.check_full(cfg, layer)
        fwd, out, steps = bwd._check_steps(cfg, layer, dloss=0.7)
        errs = bwd._check_end_to_end(cfg, fwd, out, dloss=0.7)
        print(f"   forward {info}\n   backward {({k: float(f'{v:.1e}') for k, v in errs.items()})}", flush=True)
    finally:
        layer.close()
