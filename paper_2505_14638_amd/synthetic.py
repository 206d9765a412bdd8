"""Seeded synthetic inputs with the shapes and value distributions of Llama-style linear layers.

This module only draws random tensors and names shapes; it holds none of the method's
arithmetic (no quantizer, no FP8 rounding, no packing).  Both the CPU oracle's tests and the
HIP path's tests and benchmark start from these host arrays.

Recipe (stands in for real layer weights and activations, which need model checkpoints):
  weights      W[N, K] float32 ~ N(0, 0.02^2)
  activations  X[M, K] float32 ~ N(0, 1) with a fraction of the K channels (whole columns, the
               same for every token) multiplied by a constant -- the outlier channels that
               force a large static FP8 scale (Sec. 2.3 of the paper names them as the main
               difficulty of activation quantization)
  s_x          the static per-tensor activation scale handed to the layer as an *input*:
               max|X| / 448 over the same tensor, as one float32 division (the calibration
               rule of Eq. 13 applied to the synthetic tensor itself)
Random streams: numpy PCG64, seed = 20250514 * 10 + config id, one spawned child per tensor.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20250514

# (K, N) of the four linear layers of one decoder block
LLAMA3_8B = {"qkv": (4096, 6144), "o": (4096, 4096), "gate_up": (4096, 28672), "down": (14336, 4096)}
LLAMA3_70B = {"qkv": (8192, 10240), "o": (8192, 8192), "gate_up": (8192, 57344), "down": (28672, 8192)}

CONFIGS = {
    1: dict(name="single", shapes=[(8, 1024, 1024)], group="channel", out="f32", frac=0.01, mult=20.0),
    2: dict(name="decode-8b", shapes=[(m, k, n) for (k, n) in LLAMA3_8B.values() for m in (1, 4, 16)],
            group=128, out="bf16", frac=0.01, mult=20.0),
    3: dict(name="prefill-8b", shapes=[(m, k, n) for (k, n) in LLAMA3_8B.values() for m in (512, 2048, 8192)],
            group=128, out="bf16", frac=0.01, mult=20.0),
    4: dict(name="llama-70b", shapes=[(m, k, n) for (k, n) in LLAMA3_70B.values() for m in (1, 16, 4096)],
            group=128, out="bf16", frac=0.005, mult=50.0),
    5: dict(name="block-8b", batches=(1, 8, 32, 128, 1024), hidden=4096, ffn=14336, heads=32,
            group=128, out="bf16", frac=0.01, mult=20.0),
}


def rng_for(config_id: int, *extra: int) -> np.random.Generator:
    """Root generator of a config; `extra` integers derive independent streams (shape index ...)."""
    return np.random.default_rng([BASE_SEED * 10 + config_id, *extra])


def make_weights(rng: np.random.Generator, n: int, k: int, std: float = 0.02) -> np.ndarray:
    return (rng.standard_normal((n, k), dtype=np.float32) * np.float32(std)).astype(np.float32)


def make_activations(rng: np.random.Generator, m: int, k: int, frac: float, mult: float) -> np.ndarray:
    x = rng.standard_normal((m, k), dtype=np.float32)
    n_out = max(1, int(round(frac * k)))
    cols = rng.choice(k, size=n_out, replace=False)
    x[:, cols] *= np.float32(mult)
    return x


def static_act_scale(x: np.ndarray) -> np.float32:
    """The static scale input of the workload recipe: float32(max|X|) / float32(448)."""
    return np.float32(np.float32(np.max(np.abs(x))) / np.float32(448.0))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16); input plumbing for the
    bf16-activation cases, not part of the method."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def make_layer(config_id: int, shape_index: int, m: int, k: int, n: int):
    """(W, X, s_x) for one linear layer of a config."""
    cfg = CONFIGS[config_id]
    rw, rx = rng_for(config_id, shape_index).spawn(2)
    w = make_weights(rw, n, k)
    x = make_activations(rx, m, k, cfg["frac"], cfg["mult"])
    return w, x, static_act_scale(x)
