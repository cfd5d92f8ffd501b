"""Thin Python binding of the sqmi C ABI (``include/sqmi.h``): argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used for device memory and
streams, nothing else), passes their pointers and the current HIP stream to ``libsqmi.so`` and
returns the output tensors.  There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsqmi.so")

F16, BF16 = 0, 1
PER_TOKEN_DYNAMIC, PER_TENSOR_DYNAMIC, PER_TENSOR_STATIC = 0, 1, 2
OP_QUANTIZE_ACT, OP_PREPARE_WEIGHT, OP_W8A8_LINEAR, OP_I8_GEMM_I32, OP_W8A8_BMM = range(5)
ROW_MAJOR, TILED = 0, 1

EXPORTS = (
    "sq_status_string", "sq_smooth_scales", "sq_act_absmax_per_channel", "sq_weight_absmax_per_in_channel",
    "sq_prepare_weight", "sq_quantize_act", "sq_w8a8_linear", "sq_w8a8_linear_q8", "sq_i8_gemm_i32", "sq_w8a8_bmm",
    "sq_softmax_quant_p", "sq_ln_quantize", "sq_workspace_bytes", "sq_tiled_bytes", "sq_probe_mfma_i8",
    "sq_w8a8_linear_noalloc", "sq_static_scratch_bytes", "sq_w8a8_attention", "sq_w8a8_attention_causal",
)


class SqmiError(RuntimeError):
    pass


_lib = None


def lib() -> ctypes.CDLL:
    """Load libsqmi.so (built by ``paper_2211_10438_amd.build``); fail loudly if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SqmiError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                            "(hipcc, gfx950) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
        L.sq_status_string.restype = ctypes.c_char_p
        L.sq_status_string.argtypes = [i32]
        L.sq_smooth_scales.argtypes = [vp, vp, f32, i64, vp, vp]
        L.sq_act_absmax_per_channel.argtypes = [vp, i32, i64, i64, vp, vp]
        L.sq_weight_absmax_per_in_channel.argtypes = [vp, i32, i64, i64, vp, vp]
        L.sq_prepare_weight.argtypes = [vp, i32, vp, i64, i64, vp, i32, vp, i32, vp, ctypes.c_size_t, vp]
        L.sq_quantize_act.argtypes = [vp, i32, i64, i64, i64, vp, i32, vp, vp, i32, vp, ctypes.c_size_t, vp]
        L.sq_w8a8_linear.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, i32, vp, i32, i64, i64, i64, i32, vp, ctypes.c_size_t, vp]
        L.sq_w8a8_linear_noalloc.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, i32, vp, i32, i64, i64, i64, i32, vp]
        L.sq_static_scratch_bytes.restype = ctypes.c_size_t
        L.sq_static_scratch_bytes.argtypes = []
        L.sq_w8a8_linear_q8.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, i32, i32, vp, vp, i32, i64, i64, i64, i32, vp,
                                        ctypes.c_size_t, vp]
        L.sq_i8_gemm_i32.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, ctypes.c_size_t, vp]
        L.sq_w8a8_bmm.argtypes = [vp, vp, i32, f32, vp, i32, i64, i64, i64, i64, i64, i64, i64, vp]
        L.sq_w8a8_attention.argtypes = [vp, vp, vp, f32, f32, vp, i32, i64, i64, i64, i64, i64, i64, i64, i64, vp, vp]
        L.sq_w8a8_attention_causal.argtypes = L.sq_w8a8_attention.argtypes
        L.sq_probe_mfma_i8.argtypes = [vp, ctypes.c_size_t, i32, i32, vp, vp]
        L.sq_softmax_quant_p.argtypes = [vp, i32, i64, i64, vp, vp]
        L.sq_ln_quantize.argtypes = [vp, i32, i64, i64, vp, vp, f32, vp, vp, i32, vp]
        L.sq_workspace_bytes.restype = ctypes.c_size_t
        L.sq_workspace_bytes.argtypes = [i32, i64, i64, i64]
        L.sq_tiled_bytes.restype = ctypes.c_size_t
        L.sq_tiled_bytes.argtypes = [i64, i64]
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


def _check(st: int, what: str):
    if st != 0:
        raise SqmiError(f"{what}: {lib().sq_status_string(st).decode()} (status {st})")


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"16-bit floating tensor expected, got {t.dtype}")


def _dev(t: torch.Tensor, dtype=None, name="tensor"):
    if not t.is_cuda:
        raise SqmiError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise SqmiError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _opt(t, dtype, name):
    return None if t is None else _dev(t, dtype, name)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def workspace_bytes(op: int, t: int, c_i: int, c_o: int) -> int:
    return int(lib().sq_workspace_bytes(op, t, c_i, c_o))


def _workspace(nbytes: int, device, workspace):
    if nbytes == 0 and workspace is None:
        return None, 0, None
    if workspace is None:
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    elif workspace.numel() * workspace.element_size() < nbytes:
        raise SqmiError("workspace too small")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size(), workspace


def empty_codes(rows: int, k: int, layout: int = ROW_MAJOR, device="cuda") -> torch.Tensor:
    """int8 [rows, k] operand buffer.  In the TILED layout the storage is padded to a multiple of 16 rows
    and the returned tensor is the [rows, k] view of it (its bytes are in tiled order, not row order)."""
    if layout == TILED:
        nbytes = int(lib().sq_tiled_bytes(rows, k))
        if nbytes == 0:
            raise SqmiError("tiled layout needs k % 64 == 0")
        return torch.empty((nbytes // k, k), dtype=torch.int8, device=device)[:rows]
    return torch.empty((rows, k), dtype=torch.int8, device=device)


def smooth_scales(x_absmax: torch.Tensor, w_absmax: torch.Tensor, alpha: float):
    """Eq. 4 on HOST fp32 tensors -> (s, inv_s) host fp32 tensors."""
    xa = x_absmax.detach().to("cpu", torch.float32).contiguous()
    wa = w_absmax.detach().to("cpu", torch.float32).contiguous()
    s = torch.empty_like(xa)
    inv_s = torch.empty_like(xa)
    _check(lib().sq_smooth_scales(xa.data_ptr(), wa.data_ptr(), alpha, xa.numel(), s.data_ptr(), inv_s.data_ptr()),
           "sq_smooth_scales")
    return s, inv_s


def act_absmax_per_channel(x: torch.Tensor) -> torch.Tensor:
    t, c_i = x.shape
    out = torch.empty(c_i, dtype=torch.float32, device=x.device)
    _check(lib().sq_act_absmax_per_channel(_dev(x, None, "x"), _dt(x), t, c_i, out.data_ptr(), _stream()),
           "sq_act_absmax_per_channel")
    return out


def weight_absmax_per_in_channel(w: torch.Tensor) -> torch.Tensor:
    c_i, c_o = w.shape
    out = torch.empty(c_i, dtype=torch.float32, device=w.device)
    _check(lib().sq_weight_absmax_per_in_channel(_dev(w, None, "w"), _dt(w), c_i, c_o, out.data_ptr(), _stream()),
           "sq_weight_absmax_per_in_channel")
    return out


def prepare_weight(w: torch.Tensor, s: torch.Tensor | None = None, workspace=None, layout: int = ROW_MAJOR,
                   per_channel: bool = False):
    """W [c_i, c_o] (+ optional device fp32 s [c_i]) -> (wq int8 [c_o, c_i] in `layout`, w_scale fp32 [1], or
    [c_o] with per_channel: one step per output channel)."""
    c_i, c_o = w.shape
    wq = empty_codes(c_o, c_i, layout, w.device)
    w_scale = torch.empty(c_o if per_channel else 1, dtype=torch.float32, device=w.device)
    wp, wb, keep = _workspace(workspace_bytes(OP_PREPARE_WEIGHT, 0, c_i, c_o), w.device, workspace)
    _check(lib().sq_prepare_weight(_dev(w, None, "w"), _dt(w), _opt(s, torch.float32, "s"), c_i, c_o, wq.data_ptr(),
                                   layout, w_scale.data_ptr(), int(per_channel), wp, wb, _stream()), "sq_prepare_weight")
    return wq, w_scale


def quantize_act(x: torch.Tensor, mode: int, inv_s: torch.Tensor | None = None, static_scale: torch.Tensor | None = None,
                 c_i: int | None = None, out=None, workspace=None, layout: int = ROW_MAJOR):
    """x [t, ldx] -> (xq int8 [t, c_i], scale fp32 [t] or [1]).  ``c_i`` < ldx quantizes a column prefix; a
    column slice of a wider matrix (unit column stride, row stride >= its width) is taken in place: its row
    stride becomes ldx."""
    if x.dim() != 2 or not x.is_cuda:
        raise SqmiError("x must be a 2-D GPU tensor")
    if x.is_contiguous():
        t, ldx = x.shape
        c_i = ldx if c_i is None else c_i
        x_ptr = x.data_ptr()
    else:
        if x.stride(1) != 1 or x.stride(0) < x.shape[1]:
            raise SqmiError("x must be contiguous or a column slice of a contiguous matrix")
        t, ldx = x.shape[0], x.stride(0)
        c_i = x.shape[1] if c_i is None else c_i
        x_ptr = x.data_ptr()
    if out is None:
        xq = empty_codes(t, c_i, layout, x.device)
        if mode == PER_TENSOR_STATIC:
            if static_scale is None:
                raise SqmiError("static mode needs static_scale")
            scale = static_scale
        else:
            scale = torch.empty(t if mode == PER_TOKEN_DYNAMIC else 1, dtype=torch.float32, device=x.device)
    else:
        xq, scale = out
    if workspace is not None:  # passed through as it is: a small one selects the library's three-launch O2 path
        wp, wb, keep = workspace.data_ptr(), workspace.numel() * workspace.element_size(), workspace
    else:
        wp, wb, keep = _workspace(workspace_bytes(OP_QUANTIZE_ACT, t, c_i, 0) if mode == PER_TENSOR_DYNAMIC else 0,
                                  x.device, None)
    _check(lib().sq_quantize_act(x_ptr, _dt(x), t, c_i, ldx, _opt(inv_s, torch.float32, "inv_s"), mode,
                                 _dev(scale, torch.float32, "scale"), _dev(xq, torch.int8, "xq"), layout, wp, wb,
                                 _stream()), "sq_quantize_act")
    return xq, scale


def w8a8_linear(xq: torch.Tensor, x_scale: torch.Tensor, wq: torch.Tensor, w_scale: torch.Tensor, out_dtype,
                bias=None, residual=None, relu: bool = False, out=None, workspace=None,
                layout: int = ROW_MAJOR, w_per_channel: bool | None = None) -> torch.Tensor:
    """w_scale: fp32 [1] (per tensor) or [c_o] (per output channel; inferred from its length unless
    ``w_per_channel`` says otherwise)."""
    t, c_i = xq.shape
    c_o = wq.shape[0]
    if w_per_channel is None:
        w_per_channel = w_scale.numel() == c_o and c_o > 1
    if w_scale.numel() != (c_o if w_per_channel else 1):
        raise SqmiError("w_scale must have 1 entry, or c_o entries with w_per_channel")
    if wq.shape[1] != c_i:
        raise SqmiError("wq must be [c_o, c_i]")
    if x_scale.numel() not in (1, t):
        raise SqmiError("x_scale must have 1 or t entries")
    y = torch.empty((t, c_o), dtype=out_dtype, device=xq.device) if out is None else out
    wp, wb, keep = _workspace(workspace_bytes(OP_W8A8_LINEAR, t, c_i, c_o), xq.device, workspace)
    per_token = int(x_scale.numel() == t)
    _check(lib().sq_w8a8_linear(_dev(xq, torch.int8, "xq"), _dev(x_scale, torch.float32, "x_scale"), per_token,
                                _dev(wq, torch.int8, "wq"), _dev(w_scale, torch.float32, "w_scale"), int(w_per_channel),
                                _opt(bias, torch.float32, "bias"), _opt(residual, out_dtype, "residual"), int(relu),
                                _dev(y, out_dtype, "y"), _dt(y), t, c_i, c_o, layout, wp, wb, _stream()),
           "sq_w8a8_linear")
    return y


def w8a8_linear_noalloc(xq: torch.Tensor, x_scale: torch.Tensor, wq: torch.Tensor, w_scale: torch.Tensor, out: torch.Tensor,
                        bias=None, residual=None, relu: bool = False, layout: int = ROW_MAJOR,
                        w_per_channel: bool | None = None) -> torch.Tensor:
    """sq_w8a8_linear_noalloc: the caller passes inputs and the output tensor; nothing is allocated here or in
    the library (K-split scratch is the library's built-in device array)."""
    t, c_i = xq.shape
    c_o = wq.shape[0]
    if w_per_channel is None:
        w_per_channel = w_scale.numel() == c_o and c_o > 1
    if tuple(out.shape) != (t, c_o):
        raise SqmiError("out must be [t, c_o]")
    _check(lib().sq_w8a8_linear_noalloc(_dev(xq, torch.int8, "xq"), _dev(x_scale, torch.float32, "x_scale"),
                                        int(x_scale.numel() == t), _dev(wq, torch.int8, "wq"),
                                        _dev(w_scale, torch.float32, "w_scale"), int(w_per_channel),
                                        _opt(bias, torch.float32, "bias"), _opt(residual, out.dtype, "residual"),
                                        int(relu), _dev(out, None, "out"), _dt(out), t, c_i, c_o, layout, _stream()),
           "sq_w8a8_linear_noalloc")
    return out


def w8a8_linear_q8(xq: torch.Tensor, x_scale: torch.Tensor, wq: torch.Tensor, w_scale: torch.Tensor, y_step: torch.Tensor,
                   mid_dtype, bias=None, residual=None, relu: bool = False, out=None, workspace=None,
                   layout: int = ROW_MAJOR, out_layout: int = ROW_MAJOR, w_per_channel: bool | None = None) -> torch.Tensor:
    """W8A8 linear whose epilogue also applies the static quantizer of the next int8 kernel: returns int8 codes
    [t, c_o] (in ``out_layout``) of the value rounded to ``mid_dtype``, with the calibrated step ``y_step`` [1]."""
    t, c_i = xq.shape
    c_o = wq.shape[0]
    if w_per_channel is None:
        w_per_channel = w_scale.numel() == c_o and c_o > 1
    yq = empty_codes(t, c_o, out_layout, xq.device) if out is None else out
    wp, wb, keep = _workspace(workspace_bytes(OP_W8A8_LINEAR, t, c_i, c_o), xq.device, workspace)
    mid = F16 if mid_dtype == torch.float16 else BF16
    _check(lib().sq_w8a8_linear_q8(_dev(xq, torch.int8, "xq"), _dev(x_scale, torch.float32, "x_scale"),
                                   int(x_scale.numel() == t), _dev(wq, torch.int8, "wq"),
                                   _dev(w_scale, torch.float32, "w_scale"), int(w_per_channel),
                                   _opt(bias, torch.float32, "bias"), _opt(residual, mid_dtype, "residual"), int(relu), mid,
                                   _dev(y_step, torch.float32, "y_step"), yq.data_ptr(), out_layout, t, c_i, c_o, layout,
                                   wp, wb, _stream()), "sq_w8a8_linear_q8")
    return yq


def i8_gemm_i32(xq: torch.Tensor, wq: torch.Tensor, workspace=None, layout: int = ROW_MAJOR) -> torch.Tensor:
    t, c_i = xq.shape
    c_o = wq.shape[0]
    acc = torch.empty((t, c_o), dtype=torch.int32, device=xq.device)
    wp, wb, keep = _workspace(workspace_bytes(OP_I8_GEMM_I32, t, c_i, c_o), xq.device, workspace)
    _check(lib().sq_i8_gemm_i32(_dev(xq, torch.int8, "xq"), _dev(wq, torch.int8, "wq"), acc.data_ptr(), t, c_i, c_o,
                                layout, wp, wb, _stream()), "sq_i8_gemm_i32")
    return acc


def w8a8_bmm(a: torch.Tensor, bm: torch.Tensor, trans_b: bool, alpha: float, out_dtype, out=None) -> torch.Tensor:
    """a [b, m, k]; bm [b, n, k] if trans_b else [b, k, n] -> c [b, m, n]."""
    b, m, k = a.shape
    n = bm.shape[1] if trans_b else bm.shape[2]
    c = torch.empty((b, m, n), dtype=out_dtype, device=a.device) if out is None else out
    _check(lib().sq_w8a8_bmm(_dev(a, torch.int8, "a"), _dev(bm, torch.int8, "bm"), int(trans_b), alpha,
                             _dev(c, out_dtype, "c"), _dt(c), b, m, n, k, m * k, n * k, m * n, _stream()), "sq_w8a8_bmm")
    return c


def w8a8_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, alpha1: float, alpha2: float, out_dtype, out=None,
                   p_codes: torch.Tensor | None = None, causal: bool = False) -> torch.Tensor:
    """Fused INT8 attention: q [b, s_q, d], k and v [b, s_k, d] int8 -> o [b, s_q, d].  ``p_codes`` (int8
    [b, s_q, s_k]) optionally receives the probability codes the kernel formed.  ``causal`` selects
    sq_w8a8_attention_causal (query i sees the keys j <= i + (s_k - s_q))."""
    b, s_q, d = q.shape
    s_k = k.shape[1]
    if tuple(k.shape) != (b, s_k, d) or tuple(v.shape) != (b, s_k, d):
        raise SqmiError("k and v must be [b, s_k, d]")
    o = torch.empty((b, s_q, d), dtype=out_dtype, device=q.device) if out is None else out
    if p_codes is not None and tuple(p_codes.shape) != (b, s_q, s_k):
        raise SqmiError("p_codes must be [b, s_q, s_k]")
    fn = lib().sq_w8a8_attention_causal if causal else lib().sq_w8a8_attention
    _check(fn(_dev(q, torch.int8, "q"), _dev(k, torch.int8, "k"), _dev(v, torch.int8, "v"), alpha1, alpha2,
              _dev(o, out_dtype, "o"), _dt(o), b, s_q, s_k, d, s_q * d, s_k * d, s_k * d, s_q * d,
              _opt(p_codes, torch.int8, "p_codes"), _stream()), "sq_w8a8_attention_causal" if causal else "sq_w8a8_attention")
    return o


def softmax_quant_p(s: torch.Tensor, out=None) -> torch.Tensor:
    cols = s.shape[-1]
    rows = s.numel() // cols
    pq = torch.empty(s.shape, dtype=torch.int8, device=s.device) if out is None else out
    _check(lib().sq_softmax_quant_p(_dev(s, None, "s"), _dt(s), rows, cols, _dev(pq, torch.int8, "pq"), _stream()),
           "sq_softmax_quant_p")
    return pq


def probe_mfma_i8(data: torch.Tensor, workgroups: int, iters: int) -> float:
    """Measurement aid: enqueue the MFMA-only loop; returns the number of integer operations it performs."""
    sink = torch.empty(workgroups * 512, dtype=torch.int32, device=data.device)
    _check(lib().sq_probe_mfma_i8(_dev(data, torch.int8, "data"), data.numel(), workgroups, iters, sink.data_ptr(), _stream()),
           "sq_probe_mfma_i8")
    return float(workgroups) * 8 * iters * 8 * 65536


def ln_quantize(x: torch.Tensor, gamma_f: torch.Tensor, beta_f: torch.Tensor, eps: float = 1e-5, out=None,
                layout: int = ROW_MAJOR):
    t, c_i = x.shape
    if out is None:
        xq = empty_codes(t, c_i, layout, x.device)
        scale = torch.empty(t, dtype=torch.float32, device=x.device)
    else:
        xq, scale = out
    _check(lib().sq_ln_quantize(_dev(x, None, "x"), _dt(x), t, c_i, _dev(gamma_f, torch.float32, "gamma_f"),
                                _dev(beta_f, torch.float32, "beta_f"), eps, _dev(scale, torch.float32, "scale"),
                                _dev(xq, torch.int8, "xq"), layout, _stream()), "sq_ln_quantize")
    return xq, scale
