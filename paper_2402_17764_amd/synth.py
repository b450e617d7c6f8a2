"""Seeded synthetic inputs with the shapes and value distributions of the BitLinear workloads.

This module serves both the GPU parity tests / benchmark and the CPU oracle's tests.  It holds
none of the method's arithmetic: it only draws random matrices and casts them.

Recipe (stands in for the trained 700M-70B checkpoints and real activations, which a kernel
benchmark neither has nor needs):
  * weights      fp32, i.i.d. N(0, 0.02^2), shape [N, K];
  * activations  i.i.d. N(0, 1), shape [M, K]; a fixed seeded set of ceil(0.01 K) channels (the
                 same for every token) is multiplied by 20 to mimic outlier channels; optionally
                 rounded to bf16 (round-to-nearest-even), returned as fp32 values that are exactly
                 representable in bf16 plus the raw bf16 bit patterns;
  * seeds        numpy.random.default_rng([2402, 17764, config, layer, tensor]).
"""
import math
import numpy as np

SIGMA_W = 0.02
OUTLIER_FRACTION = 0.01
OUTLIER_SCALE = 20.0

# (K, N) pairs per configuration, LLaMA-family projection shapes.  Names are for reports only.
CONFIGS = {
    0: dict(name="700M-class FFN up-projection", act_dtype="f32", Ms=(1, 16), layers=1,
            shapes=[("ffn_up", 1536, 4096)]),
    1: dict(name="3B-class decoder block, decode", act_dtype="bf16", Ms=(1,), layers=26,
            shapes=[("qkv", 3200, 9600), ("o", 3200, 3200), ("gate_up", 3200, 17280),
                    ("down", 8640, 3200)]),
    2: dict(name="7B-class layer set, batched decode", act_dtype="bf16", Ms=(1, 8, 32, 64), layers=32,
            shapes=[("qkv", 4096, 12288), ("o", 4096, 4096), ("gate_up", 4096, 22016),
                    ("down", 11008, 4096)]),
    3: dict(name="13B-class layer set, prefill", act_dtype="bf16", Ms=(512, 2048), layers=1,
            shapes=[("qkv", 5120, 15360), ("o", 5120, 5120), ("gate_up", 5120, 27648),
                    ("down", 13824, 5120)]),
    4: dict(name="70B-class FFN", act_dtype="bf16", Ms=(1, 4096), layers=80,
            shapes=[("gate_up", 8192, 57344), ("down", 28672, 8192)]),
}


def _rng(config, layer, tensor):
    return np.random.default_rng([2402, 17764, int(config), int(layer), int(tensor)])


def weights(N, K, config=0, layer=0, tensor=0, sigma=SIGMA_W):
    """fp32 [N, K] ~ N(0, sigma^2)."""
    w = _rng(config, layer, tensor).standard_normal((N, K), dtype=np.float32)
    w *= np.float32(sigma)
    return w


def to_bf16(x):
    """Round fp32 to bf16 (nearest, ties to even).  Returns (fp32 values, uint16 bit patterns)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32), (rounded >> np.uint32(16)).astype(np.uint16)


def outlier_channels(K, config=0, layer=0, tensor=1):
    n = int(math.ceil(OUTLIER_FRACTION * K))
    return np.sort(_rng(config, layer, 1000 + tensor).choice(K, size=n, replace=False))


def activations(M, K, config=0, layer=0, tensor=1, bf16=False):
    """[M, K] activations with outlier channels.

    Returns fp32 values; with bf16=True returns (fp32 values exactly representable in bf16,
    uint16 bf16 bits)."""
    x = _rng(config, layer, tensor).standard_normal((M, K), dtype=np.float32)
    x[:, outlier_channels(K, config, layer, tensor)] *= np.float32(OUTLIER_SCALE)
    if bf16:
        return to_bf16(x)
    return x
