"""GPU parity of the linear layer whose epilogue applies the next kernel's static activation quantizer
(sq_w8a8_linear_q8).  The expected codes are the oracle's own chain: w8a8_linear (16-bit output) followed by
quantize_act in static mode -- the fused kernel must produce exactly those codes, on every GEMM path."""
import numpy as np
import pytest

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import (BF16, F16, dev, random_bf16_bits, rows_to_tiled_dev, tiled_to_rows, to_dev_16, torch_dtype)

pytestmark = pytest.mark.gpu


def _progress(msg):
    print(f"[case] {msg}", flush=True)


CASES = [
    # t, c_i, c_o, mid dtype, bias, relu, residual, in layout, out layout, per-channel W
    (300, 1024, 1000, BF16, True, True, False, sq.ROW_MAJOR, sq.ROW_MAJOR, False),   # prefill tiles, ragged
    (2048, 256, 1536, F16, False, True, False, sq.TILED, sq.TILED, False),           # FC1 + ReLU -> codes for FC2
    (513, 320, 2048, F16, True, False, True, sq.ROW_MAJOR, sq.TILED, True),          # K tail, residual, per-channel W
    (16, 4096, 1024, BF16, True, False, False, sq.TILED, sq.ROW_MAJOR, False),       # split-K + reduction kernel
    (5, 1024, 4096, F16, True, True, True, sq.ROW_MAJOR, sq.TILED, False),           # weight streaming
    (128, 4096, 4096, BF16, True, False, False, sq.TILED, sq.TILED, True),           # streaming with a K split
    (70, 1088, 8192, F16, False, False, False, sq.TILED, sq.ROW_MAJOR, False),       # streaming, 8-wave shape
]


@pytest.mark.parametrize("t,c_i,c_o,mid,use_bias,relu,use_res,lay_in,lay_out,w_pc", CASES)
def test_linear_q8_matches_linear_then_static_quantize(t, c_i, c_o, mid, use_bias, relu, use_res, lay_in, lay_out, w_pc):
    _progress(f"linear_q8 t={t} c_i={c_i} c_o={c_o} mid={mid} in={lay_in} out={lay_out} w_pc={w_pc}")
    seed = 11000 + t + c_i + c_o
    case = synth.linear_case(t, c_i, c_o, 0.01, 40.0, seed, calib_tokens=64)
    ax = oracle.act_absmax_per_channel(case["x_calib"], F16)
    aw = oracle.weight_absmax_per_in_channel(case["w"], F16)
    s, inv_s = oracle.smooth_scales(ax, aw, 0.5)
    wq, ws = oracle.prepare_weight(case["w"], F16, s, per_channel=w_pc)
    xq, xs = oracle.quantize_act(case["x"], F16, oracle.PER_TOKEN_DYNAMIC, inv_s=inv_s)
    bias = synth.bias(c_o, seed + 9) if use_bias else None
    res = None
    if use_res:
        res = synth.normal_fp16((t, c_o), seed + 10) if mid == F16 else random_bf16_bits((t, c_o), seed + 10)
    y16 = oracle.w8a8_linear(xq, xs, wq, ws, mid, bias=bias, residual_bits=res, relu=relu, w_per_channel=w_pc)
    # calibrated output step: a little below absmax / 127 so that the saturation to +-127 is exercised as well
    amax = np.abs(oracle.f32_from_bits16(y16, mid)).max()
    step = np.float32(0.9) * np.float32(amax) / np.float32(127.0)
    ref, _ = oracle.quantize_act(y16, mid, oracle.PER_TENSOR_STATIC, static_scale=step)
    assert np.abs(ref).max() == 127
    xq_d, wq_d = (rows_to_tiled_dev(xq), rows_to_tiled_dev(wq)) if lay_in == sq.TILED else (dev(xq), dev(wq))
    yq = sq.w8a8_linear_q8(xq_d, dev(xs), wq_d, dev(ws), dev(np.array([step], np.float32)), torch_dtype(mid),
                           bias=None if bias is None else dev(bias), residual=None if res is None else to_dev_16(res, mid),
                           relu=relu, layout=lay_in, out_layout=lay_out)
    got = tiled_to_rows(yq) if lay_out == sq.TILED else yq.cpu().numpy()
    bad = np.argwhere(got != ref)
    assert bad.size == 0, f"{len(bad)} codes differ, first at {bad[:5].tolist()}"


def test_linear_q8_zero_step_gives_zero_codes():
    _progress("linear_q8 zero step")
    xq, wq = synth.int8_codes((40, 256), 1), synth.int8_codes((512, 256), 2)
    yq = sq.w8a8_linear_q8(dev(xq), dev(np.full(40, 1e-4, np.float32)), dev(wq), dev(np.ones(1, np.float32)),  # finite values
                           dev(np.zeros(1, np.float32)), torch_dtype(F16))
    assert not yq.cpu().numpy().any()
