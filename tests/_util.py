"""Helpers shared by the GPU parity tests: host<->device plumbing and ULP comparison."""
import numpy as np
import torch

import oracle

F16, BF16 = oracle.F16, oracle.BF16


def to_dev_16(bits_or_f16: np.ndarray, dtype: int) -> torch.Tensor:
    """fp16 ndarray or uint16 bit patterns -> GPU tensor of torch.float16 / torch.bfloat16."""
    u = oracle.bits16(np.ascontiguousarray(bits_or_f16))
    t = torch.from_numpy(u.view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == F16 else torch.bfloat16)


def bits_from_dev(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in units in the last place between two arrays of 16-bit float patterns
    (works for fp16 and bf16: both are sign-magnitude with monotone magnitude bits)."""
    def ordered(u):
        u = u.astype(np.int32)
        mag = u & 0x7FFF
        return np.where(u & 0x8000, -mag, mag)
    return np.abs(ordered(a_bits) - ordered(b_bits))


def random_bf16_bits(shape, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    f = (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale))
    u = f.view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)  # plain input generation, not the method


def torch_dtype(dt: int):
    return torch.float16 if dt == F16 else torch.bfloat16
