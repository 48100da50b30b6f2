"""Seeded synthetic inputs for the SMILE bi-level MoE layer.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/bench.  It draws random tensors and converts number formats; it
contains none of the layer's arithmetic (no gate, softmax, routing, capacity
rule, FFN or loss), so a mistake in either implementation cannot hide here.

Shapes follow the paper's Switch-style BERT workloads (Section 4.1 "Model
Architecture", Table 2: hidden/intermediate 768/3072 and 1024/4096, 128
experts, sequence length 128): tokens are a flat [T, d_model] batch of hidden
vectors, x ~ N(0,1), every gate and expert weight ~ N(0, 0.02^2) (the BERT
initialiser's standard deviation).  The public C4 corpus the paper trains on
is not used: iid Gaussian activations of the same shape stand in for it.

Random numbers come from numpy's counter-based Philox generator keyed by
(seed, tensor id, sub-index), so any tensor (or any single expert's weights)
can be regenerated independently and identically on any machine.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

# tensor ids used as the second half of the Philox key
_TID_X, _TID_W_INTER, _TID_W_INTRA, _TID_W1, _TID_W2, _TID_B_INTER, _TID_B_INTRA, _TID_PERM, _TID_DY = range(9)


@dataclass(frozen=True)
class LayerConfig:
    """One benchmark / parity configuration of the layer.

    capacity is stored as the literal integer (rows per expert buffer) so that
    no implementation of the capacity rule lives in this module.
    """
    name: str
    T: int            # tokens in the batch
    d_model: int
    d_ff: int
    n_groups: int     # n: first-level (inter) routing fan-out
    m_local: int      # m: second-level (intra) routing fan-out
    capacity_factor: float
    capacity: int     # rows per expert buffer
    dtype: str        # "f32", "bf16" or "f16": storage type of x, weights, buffers, y
    act: str          # "relu" or "gelu"
    skew: bool = False  # add routing biases (Zipf inter-group, Gaussian per-expert)
    seed: int = 0
    group_capacity: int = 0   # rows of each group's first-hop buffer; 0 = no limit

    @property
    def N(self) -> int:
        return self.n_groups * self.m_local


CONFIGS = {
    "cfg1": LayerConfig("cfg1", 512, 64, 128, 2, 2, 1.25, 160, "f32", "relu", seed=1),
    "cfg2": LayerConfig("cfg2", 8192, 768, 3072, 2, 8, 1.0, 512, "bf16", "gelu", seed=2),
    "cfg3": LayerConfig("cfg3", 16384, 1024, 4096, 8, 8, 1.25, 320, "bf16", "gelu", seed=3),
    "cfg4": LayerConfig("cfg4", 32768, 768, 3072, 16, 8, 1.0, 256, "bf16", "gelu", seed=4),
    "cfg5": LayerConfig("cfg5", 65536, 1024, 4096, 32, 8, 1.0, 256, "bf16", "gelu", skew=True, seed=5),
}


# Further paper-shaped workloads (not part of the five benchmark configurations): the largest model of
# Table 2 (hidden 1600, intermediate 6400, micro-batch 64 x sequence 128 = 8192 tokens per GPU) with the
# capacity factor 2.0 of Section 4.2; 16 resident experts as in cfg2.
EXTRA_CONFIGS = {
    "t2_48b": LayerConfig("t2_48b", 8192, 1600, 6400, 2, 8, 2.0, 1024, "bf16", "gelu", seed=6),
    # cfg4 with the flat one-level router the paper compares against (Switch Transformer: Section 2,
    # Eq. 1-2 with k = 1): same tokens, experts and capacity, one 128-way gate instead of 16 x 8
    "cfg4_flat": LayerConfig("cfg4_flat", 32768, 768, 3072, 1, 128, 1.0, 256, "bf16", "gelu", seed=4),
    # cfg2 stored in IEEE half precision, the precision the paper trains in (Section 4.1)
    "cfg2_f16": LayerConfig("cfg2_f16", 8192, 768, 3072, 2, 8, 1.0, 512, "f16", "gelu", seed=2),
}


def get_config(name: str) -> LayerConfig:
    return CONFIGS[name] if name in CONFIGS else EXTRA_CONFIGS[name]


def _rng(seed: int, tid: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 8) | int(tid), int(sub)]))


# ---------------------------------------------------------------- number formats

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit pattern (uint16), round-to-nearest-even.  Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit pattern (uint16) -> the float32 with the same value."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32 array once to the storage dtype and return it as float32 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


# ---------------------------------------------------------------- tensors
# Every function returns float32 arrays whose values are exactly representable
# in cfg.dtype, so the oracle (which takes float32) and the HIP path (which
# takes the packed storage type) see identical numbers.

def gen_tokens(cfg: LayerConfig) -> np.ndarray:
    """x[T, d_model] ~ N(0, 1)."""
    x = _rng(cfg.seed, _TID_X).standard_normal((cfg.T, cfg.d_model), dtype=np.float32)
    return quantize(x, cfg.dtype)


def gen_output_grad(cfg: LayerConfig) -> np.ndarray:
    """dy[T, d_model] ~ N(0, 1): the upstream gradient of the layer output for the backward pass."""
    dy = _rng(cfg.seed, _TID_DY).standard_normal((cfg.T, cfg.d_model), dtype=np.float32)
    return quantize(dy, cfg.dtype)


def gen_router_weights(cfg: LayerConfig) -> tuple[np.ndarray, np.ndarray]:
    """(w_inter[n, d_model], w_intra[m, d_model]) ~ N(0, 0.02^2)."""
    wi = 0.02 * _rng(cfg.seed, _TID_W_INTER).standard_normal((cfg.n_groups, cfg.d_model), dtype=np.float32)
    wl = 0.02 * _rng(cfg.seed, _TID_W_INTRA).standard_normal((cfg.m_local, cfg.d_model), dtype=np.float32)
    return quantize(wi, cfg.dtype), quantize(wl, cfg.dtype)


def gen_expert_weights(cfg: LayerConfig, e: int) -> tuple[np.ndarray, np.ndarray]:
    """Expert e's (w1[d_ff, d_model], w2[d_model, d_ff]) ~ N(0, 0.02^2); out-features x in-features."""
    w1 = 0.02 * _rng(cfg.seed, _TID_W1, e).standard_normal((cfg.d_ff, cfg.d_model), dtype=np.float32)
    w2 = 0.02 * _rng(cfg.seed, _TID_W2, e).standard_normal((cfg.d_model, cfg.d_ff), dtype=np.float32)
    return quantize(w1, cfg.dtype), quantize(w2, cfg.dtype)


def gen_routing_biases(cfg: LayerConfig) -> tuple[np.ndarray | None, np.ndarray | None]:
    """(bias_inter[n], bias_intra[n, m]) float32, or (None, None) for unskewed configs.

    Skewed stress config: the inter-group bias is 2.0 * rank^-1.2 with the
    ranks 1..n assigned to groups by a seeded permutation (Zipf s=1.2, largest
    bias 2.0); every expert gets an independent N(0, 0.5^2) intra bias.
    """
    if not cfg.skew:
        return None, None
    ranks = _rng(cfg.seed, _TID_PERM).permutation(cfg.n_groups).astype(np.float64) + 1.0
    b_inter = (2.0 * ranks ** -1.2).astype(np.float32)
    b_intra = (0.5 * _rng(cfg.seed, _TID_B_INTRA).standard_normal((cfg.n_groups, cfg.m_local))).astype(np.float32)
    return b_inter, b_intra


def small_config(name: str, T: int, d_model: int, d_ff: int, n: int, m: int, capacity: int,
                 dtype: str = "f32", act: str = "relu", skew: bool = False, seed: int = 100,
                 group_capacity: int = 0) -> LayerConfig:
    """An ad-hoc configuration for tests (capacities given as integers)."""
    return LayerConfig(name, T, d_model, d_ff, n, m, float("nan"), capacity, dtype, act, skew, seed, group_capacity)
