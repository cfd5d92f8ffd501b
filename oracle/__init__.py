"""CPU oracle for the SmoothQuant W8A8 hot path (TEST INFRASTRUCTURE ONLY).

Thin ctypes wrapper over ``sq_oracle.c`` (plain C, fp32 without contraction, exact int32 loops).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package; the product package never does, and this package never imports the product.

All arrays are NumPy; 16-bit floating tensors travel as ``uint16`` bit patterns plus a dtype code
(0 = fp16, 1 = bf16) so that bf16 needs no NumPy support.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sq_oracle.c")
_LIB = os.path.join(_HERE, "libsq_oracle.so")

F16, BF16 = 0, 1
PER_TOKEN_DYNAMIC, PER_TENSOR_DYNAMIC, PER_TENSOR_STATIC = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every fp32 product and sum separately
    rounded; x86-64-v3 (AVX2) keeps the binary portable between the build host and the GPU machine."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-std=c11", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_h2f.restype = ctypes.c_float
        L.orc_h2f.argtypes = [ctypes.c_uint16]
        L.orc_bf2f.restype = ctypes.c_float
        L.orc_bf2f.argtypes = [ctypes.c_uint16]
        L.orc_f2h.restype = ctypes.c_uint16
        L.orc_f2h.argtypes = [ctypes.c_float]
        L.orc_f2bf.restype = ctypes.c_uint16
        L.orc_f2bf.argtypes = [ctypes.c_float]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid arguments (code {rc})")


def _c(a, dtype):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def bits16(x: np.ndarray) -> np.ndarray:
    """fp16 ndarray -> raw uint16 bits (bf16 data is already carried as uint16)."""
    if x.dtype == np.float16:
        return x.view(np.uint16)
    if x.dtype == np.uint16:
        return x
    raise TypeError(f"16-bit tensor expected, got {x.dtype}")


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest-even) with the oracle's own converter."""
    L = lib()
    flat = np.ascontiguousarray(x, dtype=np.float32).ravel()
    out = np.fromiter((L.orc_f2bf(float(v)) for v in flat), dtype=np.uint16, count=flat.size)
    return out.reshape(x.shape)


def f32_from_bits16(u: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of fp16 / bf16 bit patterns to fp32."""
    u = np.ascontiguousarray(u, dtype=np.uint16)
    if dtype == F16:
        return u.view(np.float16).astype(np.float32)
    return (u.astype(np.uint32) << 16).view(np.float32)


def smooth_scales(x_absmax, w_absmax, alpha: float):
    ax = _c(x_absmax, np.float32)
    aw = _c(w_absmax, np.float32)
    s = np.empty_like(ax)
    inv_s = np.empty_like(ax)
    _chk(lib().orc_smooth_scales(_p(ax), _p(aw), ctypes.c_float(alpha), ctypes.c_int64(ax.size), _p(s), _p(inv_s)),
         "smooth_scales")
    return s, inv_s


def act_absmax_per_channel(x_bits, dtype: int):
    x = _c(bits16(x_bits), np.uint16)
    t, c_i = x.shape
    out = np.empty(c_i, np.float32)
    _chk(lib().orc_act_absmax_per_channel(_p(x), dtype, ctypes.c_int64(t), ctypes.c_int64(c_i), _p(out)), "act_absmax")
    return out


def weight_absmax_per_in_channel(w_bits, dtype: int):
    w = _c(bits16(w_bits), np.uint16)
    c_i, c_o = w.shape
    out = np.empty(c_i, np.float32)
    _chk(lib().orc_weight_absmax_per_in_channel(_p(w), dtype, ctypes.c_int64(c_i), ctypes.c_int64(c_o), _p(out)),
         "weight_absmax")
    return out


def prepare_weight(w_bits, dtype: int, s=None, per_channel: bool = False):
    """W [c_i, c_o] -> (wq int8 [c_o, c_i], Delta_W fp32 [1], or [c_o] with per_channel)."""
    w = _c(bits16(w_bits), np.uint16)
    c_i, c_o = w.shape
    s = _c(s, np.float32)
    wq = np.empty((c_o, c_i), np.int8)
    ws = np.empty(c_o if per_channel else 1, np.float32)
    fn = lib().orc_prepare_weight_per_channel if per_channel else lib().orc_prepare_weight
    _chk(fn(_p(w), dtype, _p(s), ctypes.c_int64(c_i), ctypes.c_int64(c_o), _p(wq), _p(ws)), "prepare_weight")
    return wq, ws


def quantize_act(x_bits, dtype: int, mode: int, inv_s=None, static_scale=None, ldx=None, c_i=None):
    """x [t, ldx] (first c_i columns used) -> (codes int8 [t, c_i], scale fp32 [t] or [1])."""
    x = _c(bits16(x_bits), np.uint16)
    t, ld = x.shape
    ldx = ld if ldx is None else ldx
    c_i = ld if c_i is None else c_i
    inv_s = _c(inv_s, np.float32)
    scale = np.empty(t if mode == PER_TOKEN_DYNAMIC else 1, np.float32)
    if mode == PER_TENSOR_STATIC:
        scale[0] = np.float32(static_scale)
    xq = np.empty((t, c_i), np.int8)
    _chk(lib().orc_quantize_act(_p(x), dtype, ctypes.c_int64(t), ctypes.c_int64(c_i), ctypes.c_int64(ldx),
                                _p(inv_s), mode, _p(scale), _p(xq)), "quantize_act")
    return xq, scale


def i8_gemm_i32(xq, wq):
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    t, c_i = xq.shape
    c_o, c_i2 = wq.shape
    assert c_i == c_i2
    acc = np.empty((t, c_o), np.int32)
    _chk(lib().orc_i8_gemm_i32(_p(xq), _p(wq), _p(acc), ctypes.c_int64(t), ctypes.c_int64(c_i), ctypes.c_int64(c_o)),
         "i8_gemm_i32")
    return acc


def w8a8_linear(xq, x_scale, wq, w_scale, out_dtype: int, bias=None, residual_bits=None, relu=False,
                rows=None, w_per_channel=False):
    """Returns y as uint16 bits [t, c_o]; with ``rows`` only those rows are computed (others zero)."""
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    x_scale = _c(np.atleast_1d(x_scale), np.float32)
    w_scale = _c(np.atleast_1d(w_scale), np.float32)
    t, c_i = xq.shape
    c_o = wq.shape[0]
    if x_scale.size not in (1, t):
        raise ValueError("x_scale must have 1 or t entries")
    per_token = int(x_scale.size == t)
    bias = _c(bias, np.float32)
    res = None if residual_bits is None else _c(bits16(residual_bits), np.uint16)
    y = np.zeros((t, c_o), np.uint16)
    rows_a = None if rows is None else _c(np.asarray(rows, dtype=np.int64), np.int64)
    _chk(lib().orc_w8a8_linear_rows(_p(xq), _p(x_scale), per_token, _p(wq), _p(w_scale), int(w_per_channel),
                                    _p(bias), _p(res), int(relu), _p(y), out_dtype, ctypes.c_int64(t),
                                    ctypes.c_int64(c_i), ctypes.c_int64(c_o), _p(rows_a),
                                    ctypes.c_int64(0 if rows_a is None else rows_a.size)), "w8a8_linear")
    return y


def w8a8_bmm(a, bm, trans_b: bool, alpha: float, out_dtype: int, batches=None):
    """a [b, m, k]; bm [b, n, k] if trans_b else [b, k, n]; returns uint16 bits [b, m, n]."""
    a = _c(a, np.int8)
    bm = _c(bm, np.int8)
    b, m, k = a.shape
    n = bm.shape[1] if trans_b else bm.shape[2]
    c = np.zeros((b, m, n), np.uint16)
    bl = None if batches is None else _c(np.asarray(batches, dtype=np.int64), np.int64)
    _chk(lib().orc_w8a8_bmm(_p(a), _p(bm), int(trans_b), ctypes.c_float(alpha), _p(c), out_dtype,
                            ctypes.c_int64(b), ctypes.c_int64(m), ctypes.c_int64(n), ctypes.c_int64(k),
                            ctypes.c_int64(m * k), ctypes.c_int64(n * k), ctypes.c_int64(m * n), _p(bl),
                            ctypes.c_int64(0 if bl is None else bl.size)), "w8a8_bmm")
    return c


def softmax_quant_p(s_bits, dtype: int):
    s = _c(bits16(s_bits), np.uint16)
    rows = int(np.prod(s.shape[:-1]))
    cols = s.shape[-1]
    pq = np.empty(s.shape, np.int8)
    _chk(lib().orc_softmax_quant_p(_p(s), dtype, ctypes.c_int64(rows), ctypes.c_int64(cols), _p(pq)), "softmax_quant_p")
    return pq


def softmax_quant_p_causal(s_bits, dtype: int):
    """s [b, s_q, s_k] 16-bit scores; query i sees the keys j <= i + (s_k - s_q); returns the codes [b, s_q, s_k]."""
    s = _c(bits16(s_bits), np.uint16)
    b, s_q, s_k = s.shape
    pq = np.empty(s.shape, np.int8)
    _chk(lib().orc_softmax_quant_p_causal(_p(s), dtype, ctypes.c_int64(b), ctypes.c_int64(s_q), ctypes.c_int64(s_k), _p(pq)),
         "softmax_quant_p_causal")
    return pq


def ln_quantize(x_bits, dtype: int, gamma_f, beta_f, eps: float = 1e-5):
    x = _c(bits16(x_bits), np.uint16)
    t, c_i = x.shape
    g = _c(gamma_f, np.float32)
    b = _c(beta_f, np.float32)
    scale = np.empty(t, np.float32)
    xq = np.empty((t, c_i), np.int8)
    _chk(lib().orc_ln_quantize(_p(x), dtype, ctypes.c_int64(t), ctypes.c_int64(c_i), _p(g), _p(b),
                               ctypes.c_float(eps), _p(scale), _p(xq)), "ln_quantize")
    return xq, scale


def num_threads() -> int:
    return int(lib().orc_num_threads())
