"""Seeded synthetic inputs with the shapes and outlier structure of the paper's workloads.

This module holds NO arithmetic of the method (no smoothing, no quantization): it only draws the
random tensors that both the GPU library and the CPU oracle are fed with.  NumPy only.

The paper observes (Sec. 3, Fig. 4) that LLM activations carry a few persistent outlier channels
roughly 100x larger than the rest while weights are flat; the tensors here reproduce that: N(0,1)
activations with a seed-chosen set of channels multiplied by a factor, N(0, 0.02^2) weights.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20221118


@dataclass(frozen=True)
class LinearShape:
    name: str
    c_i: int
    c_o: int


# OPT-175B-shaped linears at hidden 12288 (the shapes the headline metric is quoted on).
OPT175B_LINEARS = (
    LinearShape("qkv", 12288, 36864),
    LinearShape("out_proj", 12288, 12288),
    LinearShape("fc1", 12288, 49152),
    LinearShape("fc2", 49152, 12288),
)
OPT175B_TOKENS = (1, 16, 128, 2048)

# OPT-13B-shaped FFN pair.
OPT13B_FFN = (LinearShape("fc1", 5120, 20480), LinearShape("fc2", 20480, 5120))

# OPT-125m-shaped single linear.
OPT125M_LINEAR = LinearShape("fc1", 768, 3072)

# OPT-66B-shaped decoder layer.
OPT66B_LAYER = dict(hidden=9216, ffn=36864, heads=72, head_dim=128, batch=4, seq=1024)


def n_outlier_channels(c_i: int, fraction: float) -> int:
    return int(round(fraction * c_i))


def outlier_channels(c_i: int, n_out: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(c_i, size=n_out, replace=False))


def activations(t: int, c_i: int, channels: np.ndarray, factor: float, seed: int) -> np.ndarray:
    """fp16 [t, c_i]: N(0,1) with the given channels multiplied by ``factor``."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((t, c_i), dtype=np.float32)
    if len(channels):
        x[:, channels] *= np.float32(factor)
    return x.astype(np.float16)


def weights(c_i: int, c_o: int, seed: int, std: float = 0.02) -> np.ndarray:
    """fp16 [c_i, c_o] (the paper's W orientation): N(0, std^2)."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((c_i, c_o), dtype=np.float32)
    w *= np.float32(std)
    return w.astype(np.float16)


def normal_fp16(shape, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.standard_normal(shape, dtype=np.float32).astype(np.float16)


def int8_codes(shape, seed: int, lo: int = -127, hi: int = 127) -> np.ndarray:
    """Uniform int8 codes in [lo, hi] (for contraction-only tests)."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int8)


def bias(c_o: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(c_o, dtype=np.float32) * np.float32(0.1)).astype(np.float32)


def linear_case(t: int, c_i: int, c_o: int, outlier_fraction: float, factor: float, seed: int,
                n_out: int | None = None, calib_tokens: int = 512):
    """One linear-layer workload: activation X, a calibration batch with the SAME outlier channels
    (standing in for the paper's 512 calibration sentences), and weight W."""
    n_out = n_outlier_channels(c_i, outlier_fraction) if n_out is None else n_out
    ch = outlier_channels(c_i, n_out, seed)
    x = activations(t, c_i, ch, factor, seed + 1)
    x_calib = activations(calib_tokens, c_i, ch, factor, seed + 2)
    w = weights(c_i, c_o, seed + 3)
    return dict(x=x, x_calib=x_calib, w=w, channels=ch)
