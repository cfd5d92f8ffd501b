"""GPU parity of the few-token (decode) GEMM path: at most 128 tokens against a wide C_o, where the library
streams W once through one workgroup per compute unit.  Shapes are chosen to cover every activation-block
count (1, 2, 4, 8 blocks of 16 tokens), slabs of 1 to 16 column units, uneven slabs, a ragged last unit,
1 / 2 / 4 K steps per pipeline stage, K ranges shorter than the pipeline, more workgroups than one round, and
the plans that split K (64..128 tokens against a C_o that gives narrow slabs)."""
import numpy as np
import pytest

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import (assert_identical_16, BF16, F16, bits_from_dev, dev, random_bf16_bits, rows_to_tiled_dev, to_dev_16, torch_dtype,
                         ulp_distance)

pytestmark = pytest.mark.gpu


def _progress(msg):
    print(f"[case] {msg}", flush=True)


STREAM_GEMM = [
    (1, 64, 4096), (7, 192, 4096), (16, 640, 7688), (17, 1024, 8192), (33, 2048, 12288), (64, 1088, 36864),
    (100, 4096, 4096), (128, 1024, 65536), (128, 12288, 12288), (1, 49152, 12288), (128, 512, 50272),
    (16, 256, 70000), (2, 12288, 36864), (65, 3072, 49152), (64, 12288, 12288), (128, 9216, 4096),
]


@pytest.mark.parametrize("layout", [sq.ROW_MAJOR, sq.TILED])
@pytest.mark.parametrize("t,c_i,c_o", STREAM_GEMM)
def test_stream_gemm_i32_exact(t, c_i, c_o, layout):
    _progress(f"stream i8_gemm_i32 t={t} c_i={c_i} c_o={c_o} layout={layout}")
    if t <= 32:
        assert sq.workspace_bytes(sq.OP_I8_GEMM_I32, t, c_i, c_o) == 0  # up to 32 tokens: never a K split
    xq = synth.int8_codes((t, c_i), 51 + t)
    wq = synth.int8_codes((c_o, c_i), 52 + c_o % 1000)
    ref = oracle.i8_gemm_i32(xq, wq)
    if layout == sq.TILED:
        acc = sq.i8_gemm_i32(rows_to_tiled_dev(xq), rows_to_tiled_dev(wq), layout=sq.TILED).cpu().numpy()
    else:
        acc = sq.i8_gemm_i32(dev(xq), dev(wq)).cpu().numpy()
    bad = np.argwhere(acc != ref)
    assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[:5].tolist()}"


def test_stream_gemm_extreme_values_do_not_wrap():
    _progress("stream i8_gemm_i32 extremes")
    t, c_i, c_o = 20, 49152, 4096
    xq = np.full((t, c_i), 127, np.int8)
    wq = np.full((c_o, c_i), -127, np.int8)
    wq[::2] = 127
    acc = sq.i8_gemm_i32(dev(xq), dev(wq)).cpu().numpy()
    want = np.where(np.arange(c_o) % 2 == 0, c_i * 127 * 127, -c_i * 127 * 127).astype(np.int32)
    assert np.array_equal(acc, np.broadcast_to(want, (t, c_o)))


STREAM_LINEAR = [
    # t, c_i, c_o, out dtype, per_token, bias, relu, residual, layout
    (1, 2048, 4096, BF16, True, False, False, False, sq.TILED),
    (5, 1024, 4096, F16, True, True, True, True, sq.ROW_MAJOR),
    (16, 768, 8192, BF16, False, True, False, True, sq.TILED),
    (40, 768, 8192, F16, True, False, True, False, sq.ROW_MAJOR),
    (128, 2048, 7688, F16, True, True, True, True, sq.TILED),
    (100, 1024, 12288, BF16, True, True, False, False, sq.ROW_MAJOR),
    (128, 1024, 36864, BF16, True, False, False, True, sq.TILED),
    (128, 4096, 4096, BF16, True, True, True, True, sq.TILED),      # wide slabs over a quarter of K each
    (64, 12288, 12288, F16, True, True, False, True, sq.ROW_MAJOR),  # two K splits
]


@pytest.mark.parametrize("t,c_i,c_o,odt,per_token,use_bias,relu,use_res,layout", STREAM_LINEAR)
def test_stream_linear_parity(t, c_i, c_o, odt, per_token, use_bias, relu, use_res, layout):
    _progress(f"stream w8a8_linear t={t} c_i={c_i} c_o={c_o} out={odt} per_token={per_token} bias={use_bias} "
              f"relu={relu} res={use_res} layout={layout}")
    seed = 7000 + t + c_i + c_o
    case = synth.linear_case(t, c_i, c_o, 0.01, 40.0, seed, calib_tokens=64)
    ax = oracle.act_absmax_per_channel(case["x_calib"], F16)
    aw = oracle.weight_absmax_per_in_channel(case["w"], F16)
    s, inv_s = oracle.smooth_scales(ax, aw, 0.5)
    wq, ws = oracle.prepare_weight(case["w"], F16, s)
    mode = oracle.PER_TOKEN_DYNAMIC if per_token else oracle.PER_TENSOR_DYNAMIC
    xq, xs = oracle.quantize_act(case["x"], F16, mode, inv_s=inv_s)
    bias = synth.bias(c_o, seed + 9) if use_bias else None
    res = None
    if use_res:
        res = synth.normal_fp16((t, c_o), seed + 10) if odt == F16 else random_bf16_bits((t, c_o), seed + 10)
    ref = oracle.w8a8_linear(xq, xs, wq, ws, odt, bias=bias, residual_bits=res, relu=relu)
    if layout == sq.TILED:
        xq_d, wq_d = rows_to_tiled_dev(xq), rows_to_tiled_dev(wq)
    else:
        xq_d, wq_d = dev(xq), dev(wq)
    y = sq.w8a8_linear(xq_d, dev(xs), wq_d, dev(ws), torch_dtype(odt), bias=None if bias is None else dev(bias),
                       residual=None if res is None else to_dev_16(res, odt), relu=relu, layout=layout)
    d = ulp_distance(bits_from_dev(y), ref)
    assert_identical_16(d)
