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


def assert_identical_16(d: np.ndarray, what: str = ""):
    """Gate for the dequantizing epilogues (Eq. 2 outer scaling): a fixed sequence of IEEE fp32 operations without
    contraction on both sides, so the 16-bit outputs must be identical; 1 ulp is the hard limit of the contract
    and is reported separately so that a failure says which of the two was broken."""
    assert d.max() <= 1, f"{what} max ulp distance {d.max()} (contract: <= 1)"
    assert d.max() == 0, f"{what} {int((d != 0).sum())} of {d.size} outputs differ by 1 ulp (expected identical)"


def random_bf16_bits(shape, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    f = (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale))
    u = f.view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)  # plain input generation, not the method


def torch_dtype(dt: int):
    return torch.float16 if dt == F16 else torch.bfloat16


def tiled_index(rows: int, k: int) -> np.ndarray:
    """Byte offset of element (r, c) of an int8 [rows, k] operand in the library's TILED layout,
    written from the formula in include/sqmi.h (index plumbing for the tests, no method arithmetic)."""
    r = np.arange(rows, dtype=np.int64)[:, None]
    c = np.arange(k, dtype=np.int64)[None, :]
    rr = r % 16
    sw = ((rr >> 1) & 3) ^ ((rr >> 3) & 1)
    return ((r // 16) * (k // 64) + c // 64) * 1024 + rr * 64 + ((((c % 64) // 16) ^ sw) * 16) + c % 16


def tiled_to_rows(t: torch.Tensor) -> np.ndarray:
    """Logical [rows, k] codes of a tensor returned by the binding in TILED layout.  Block-wise inverse of
    rows_to_tiled_dev (reshapes instead of a gather through tiled_index, which would need an int64 index per
    byte: too much for a 600 MB weight)."""
    rows, k = t.shape
    base = t._base if t._base is not None else t
    raw = base.cpu().numpy().reshape(-1)
    pad = (rows + 15) // 16 * 16
    blk = raw[:pad * k].reshape(pad // 16, k // 64, 16, 4, 16)  # [R/16, K/64, row, stored position, byte]
    rr = np.arange(16)
    sw = ((rr >> 1) & 3) ^ ((rr >> 3) & 1)
    pos_of_chunk = np.arange(4)[None, :] ^ sw[:, None]  # chunk c of row r is stored at position c ^ sw(r)
    out = blk[:, :, rr[:, None], pos_of_chunk, :]  # [R/16, K/64, row, chunk, byte]
    return np.ascontiguousarray(out.transpose(0, 2, 1, 3, 4)).reshape(pad, k)[:rows]


def rows_to_tiled_dev(codes: np.ndarray) -> torch.Tensor:
    """Upload row-major codes in TILED layout; returns the [rows, k] view the binding expects.
    Block-wise (16 rows x 64 columns -> 1 KB, the four 16-byte chunks of row r stored at chunk ^ sw(r)):
    the same layout as tiled_index, built with reshapes so that large operands stay cheap."""
    rows, k = codes.shape
    pad = (rows + 15) // 16 * 16
    full = np.zeros((pad, k), np.int8)
    full[:rows] = codes
    blk = full.reshape(pad // 16, 16, k // 64, 4, 16).transpose(0, 2, 1, 3, 4)  # [R/16, K/64, row, chunk, byte]
    rr = np.arange(16)
    sw = ((rr >> 1) & 3) ^ ((rr >> 3) & 1)
    src_chunk = np.arange(4)[None, :] ^ sw[:, None]  # stored position p of row r holds chunk p ^ sw(r)
    out = blk[:, :, rr[:, None], src_chunk, :]
    return torch.from_numpy(np.ascontiguousarray(out).reshape(pad, k)).cuda()[:rows]
