"""GPU parity of per-output-channel weight steps (the weight granularity of Table 7; Eq. 2's diag(Delta_W) as a
vector): weight preparation (codes and steps bit-exact) and the linear layer on every GEMM path (prefill tiles,
few-token tiles with split-K, weight streaming with and without a K split), both operand layouts."""
import numpy as np
import pytest

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import (assert_identical_16, BF16, F16, bits_from_dev, dev, random_bf16_bits, rows_to_tiled_dev, tiled_to_rows, to_dev_16,
                         torch_dtype, ulp_distance)

pytestmark = pytest.mark.gpu


def _progress(msg):
    print(f"[case] {msg}", flush=True)


@pytest.mark.parametrize("c_i,c_o,with_s,layout", [(16, 8, True, sq.ROW_MAJOR), (768, 3072, True, sq.TILED),
                                                   (1040, 520, False, sq.ROW_MAJOR), (2048, 264, True, sq.TILED),
                                                   (4096, 12288, True, sq.ROW_MAJOR)])
def test_prepare_weight_per_channel(c_i, c_o, with_s, layout):
    _progress(f"prepare_weight per-channel c_i={c_i} c_o={c_o} s={with_s} layout={layout}")
    w = synth.weights(c_i, c_o, 900 + c_o)
    w[:, 3] = 0  # a dead output channel: step 0, codes 0
    s = None
    if with_s:
        s = (np.random.default_rng(901 + c_i).random(c_i, dtype=np.float32) * 4 + np.float32(0.25)).astype(np.float32)
    wq_ref, ws_ref = oracle.prepare_weight(w, F16, s, per_channel=True)
    wq, ws = sq.prepare_weight(to_dev_16(w, F16), None if s is None else dev(s), layout=layout, per_channel=True)
    assert np.array_equal(ws.cpu().numpy(), ws_ref)
    got = tiled_to_rows(wq) if layout == sq.TILED else wq.cpu().numpy()
    assert np.array_equal(got, wq_ref)


PC_LINEAR = [
    # t, c_i, c_o, out dtype, per_token, bias, relu, residual, layout
    (300, 1024, 1000, BF16, True, True, True, True, sq.ROW_MAJOR),    # prefill tiles, ragged
    (2048, 256, 1536, F16, True, False, False, False, sq.TILED),      # prefill tiles
    (513, 320, 2056, F16, False, True, False, True, sq.ROW_MAJOR),    # K tail, per-tensor activation step
    (16, 4096, 1024, BF16, True, True, False, False, sq.TILED),       # few tokens, narrow C_o: split-K + reduction
    (5, 1024, 4096, F16, True, True, True, True, sq.ROW_MAJOR),       # weight streaming
    (128, 4096, 4096, BF16, True, False, False, True, sq.TILED),      # weight streaming with a K split
    (70, 1088, 8192, F16, True, True, False, False, sq.TILED),        # weight streaming, 8-wave shape
]


@pytest.mark.parametrize("t,c_i,c_o,odt,per_token,use_bias,relu,use_res,layout", PC_LINEAR)
def test_linear_per_channel_weight_scale(t, c_i, c_o, odt, per_token, use_bias, relu, use_res, layout):
    _progress(f"per-channel w8a8_linear t={t} c_i={c_i} c_o={c_o} out={odt} layout={layout}")
    seed = 9000 + t + c_i + c_o
    case = synth.linear_case(t, c_i, c_o, 0.01, 40.0, seed, calib_tokens=64)
    # spread the column magnitudes so that per-channel steps differ by orders of magnitude
    col_gain = (2.0 ** np.random.default_rng(seed + 3).integers(-3, 4, c_o)).astype(np.float32)
    w = (case["w"].astype(np.float32) * col_gain[None, :]).astype(np.float16)
    ax = oracle.act_absmax_per_channel(case["x_calib"], F16)
    aw = oracle.weight_absmax_per_in_channel(w, F16)
    s, inv_s = oracle.smooth_scales(ax, aw, 0.5)
    wq, ws = oracle.prepare_weight(w, F16, s, per_channel=True)
    mode = oracle.PER_TOKEN_DYNAMIC if per_token else oracle.PER_TENSOR_DYNAMIC
    xq, xs = oracle.quantize_act(case["x"], F16, mode, inv_s=inv_s)
    bias = synth.bias(c_o, seed + 9) if use_bias else None
    res = None
    if use_res:
        res = synth.normal_fp16((t, c_o), seed + 10) if odt == F16 else random_bf16_bits((t, c_o), seed + 10)
    ref = oracle.w8a8_linear(xq, xs, wq, ws, odt, bias=bias, residual_bits=res, relu=relu, w_per_channel=True)
    if layout == sq.TILED:
        xq_d, wq_d = rows_to_tiled_dev(xq), rows_to_tiled_dev(wq)
    else:
        xq_d, wq_d = dev(xq), dev(wq)
    y = sq.w8a8_linear(xq_d, dev(xs), wq_d, dev(ws), torch_dtype(odt), bias=None if bias is None else dev(bias),
                       residual=None if res is None else to_dev_16(res, odt), relu=relu, layout=layout)
    d = ulp_distance(bits_from_dev(y), ref)
    assert_identical_16(d)
