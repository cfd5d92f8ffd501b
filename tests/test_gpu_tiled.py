"""GPU parity of the TILED operand layout (the layout the GEMM streams fastest): the same codes, the
same accumulators and the same outputs as the row-major path and the oracle, only stored differently."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import (assert_identical_16, BF16, F16, bits_from_dev, dev, random_bf16_bits, rows_to_tiled_dev, tiled_to_rows, to_dev_16,
                         torch_dtype, ulp_distance)

pytestmark = pytest.mark.gpu


def _progress(msg):
    print(f"[case] {msg}", flush=True)


@pytest.mark.parametrize("t,c_i", [(1, 64), (5, 128), (33, 1024), (16, 12288), (3, 49152), (260, 192), (2, 65600)])
@pytest.mark.parametrize("mode", [sq.PER_TOKEN_DYNAMIC, sq.PER_TENSOR_DYNAMIC, sq.PER_TENSOR_STATIC])
def test_quantize_tiled(t, c_i, mode):
    _progress(f"quantize tiled t={t} c_i={c_i} mode={mode}")
    x = synth.activations(t, c_i, synth.outlier_channels(c_i, max(1, c_i // 200), 7), 50.0, 8 + t)
    inv_s = (np.random.default_rng(9).random(c_i, dtype=np.float32) + np.float32(0.5))
    static = np.float32(0.21)
    q_ref, s_ref = oracle.quantize_act(x, F16, mode, inv_s=inv_s, static_scale=static)
    q, s = sq.quantize_act(to_dev_16(x, F16), mode, inv_s=dev(inv_s), static_scale=dev(np.array([static], np.float32)),
                           layout=sq.TILED)
    assert np.array_equal(tiled_to_rows(q), q_ref)
    assert np.array_equal(s.cpu().numpy(), s_ref)


@pytest.mark.parametrize("c_i,c_o,with_s", [(64, 8, True), (768, 3072, True), (1088, 520, False), (2048, 264, True)])
def test_prepare_weight_tiled(c_i, c_o, with_s):
    _progress(f"prepare_weight tiled c_i={c_i} c_o={c_o}")
    w = synth.weights(c_i, c_o, 11 + c_i)
    s = (np.random.default_rng(12).random(c_i, dtype=np.float32) * 4 + np.float32(0.1)) if with_s else None
    wq_ref, ws_ref = oracle.prepare_weight(w, F16, s)
    wq, ws = sq.prepare_weight(to_dev_16(w, F16), None if s is None else dev(s), layout=sq.TILED)
    assert ws.item() == ws_ref[0]
    assert np.array_equal(tiled_to_rows(wq), wq_ref)


TILED_GEMM = [(1, 64, 16), (16, 768, 3072), (31, 320, 100), (33, 1024, 260), (64, 2048, 256), (100, 1088, 777),
              (129, 320, 515), (256, 512, 256), (257, 1088, 258), (300, 1984, 1000), (512, 5120, 1280), (16, 12288, 1536),
              (1, 49152, 768), (520, 192, 2064),
              # weight streaming with more than 32 tokens (loader waves + weights through registers): the shortest K
              # range it takes and one below it, ragged tokens, slabs of unequal width, K steps that fill neither a
              # stage nor the unrolled body, a K split, the widest slabs
              (33, 1024, 4096), (40, 960, 4096), (100, 1088, 4112), (128, 4160, 8208), (65, 12288, 4096), (64, 2048, 36880),
              (128, 1024, 65536)]


@pytest.mark.parametrize("t,c_i,c_o", TILED_GEMM)
def test_i8_gemm_i32_tiled(t, c_i, c_o):
    _progress(f"i8_gemm_i32 tiled t={t} c_i={c_i} c_o={c_o}")
    xq = synth.int8_codes((t, c_i), 21 + t)
    wq = synth.int8_codes((c_o, c_i), 22 + c_o)
    ref = oracle.i8_gemm_i32(xq, wq)
    acc = sq.i8_gemm_i32(rows_to_tiled_dev(xq), rows_to_tiled_dev(wq), layout=sq.TILED).cpu().numpy()
    bad = np.argwhere(acc != ref)
    assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[:5].tolist()}"


@pytest.mark.parametrize("t,c_i,c_o,odt,use_bias,relu,use_res", [
    (16, 768, 3072, F16, False, False, False), (70, 1088, 520, BF16, True, False, True),
    (300, 1024, 1000, BF16, False, True, False), (513, 320, 2056, F16, True, True, True),
    (128, 4096, 768, BF16, True, False, False), (2048, 256, 1536, BF16, False, False, False),
    (100, 1088, 4104, BF16, True, True, True), (128, 2048, 8192, F16, True, False, True), (48, 12288, 4096, BF16, False, False, False)])
def test_linear_tiled_end_to_end(t, c_i, c_o, odt, use_bias, relu, use_res):
    """quantize_act (tiled out) -> w8a8_linear (tiled in) with weights prepared tiled, all on the GPU."""
    _progress(f"linear tiled t={t} c_i={c_i} c_o={c_o} out={odt}")
    seed = 300 + t + c_i
    case = synth.linear_case(t, c_i, c_o, 0.01, 40.0, seed, calib_tokens=64)
    s, inv_s = oracle.smooth_scales(oracle.act_absmax_per_channel(case["x_calib"], F16),
                                    oracle.weight_absmax_per_in_channel(case["w"], F16), 0.5)
    wq_ref, ws_ref = oracle.prepare_weight(case["w"], F16, s)
    xq_ref, xs_ref = oracle.quantize_act(case["x"], F16, oracle.PER_TOKEN_DYNAMIC, inv_s=inv_s)
    bias = synth.bias(c_o, seed + 1) if use_bias else None
    res = None
    if use_res:
        res = synth.normal_fp16((t, c_o), seed + 2) if odt == F16 else random_bf16_bits((t, c_o), seed + 2)
    ref = oracle.w8a8_linear(xq_ref, xs_ref, wq_ref, ws_ref, odt, bias=bias, residual_bits=res, relu=relu)
    wq, ws = sq.prepare_weight(to_dev_16(case["w"], F16), dev(s), layout=sq.TILED)
    xq, xs = sq.quantize_act(to_dev_16(case["x"], F16), sq.PER_TOKEN_DYNAMIC, inv_s=dev(inv_s), layout=sq.TILED)
    y = sq.w8a8_linear(xq, xs, wq, ws, torch_dtype(odt), bias=None if bias is None else dev(bias),
                       residual=None if res is None else to_dev_16(res, odt), relu=relu, layout=sq.TILED)
    d = ulp_distance(bits_from_dev(y), ref)
    assert_identical_16(d)


def test_ln_quantize_tiled_matches_row_major():
    _progress("ln_quantize tiled")
    t, c_i = 19, 9216
    x = synth.normal_fp16((t, c_i), 41)
    rng = np.random.default_rng(42)
    g = rng.standard_normal(c_i, dtype=np.float32)
    b = rng.standard_normal(c_i, dtype=np.float32) * np.float32(0.1)
    q0, s0 = sq.ln_quantize(to_dev_16(x, F16), dev(g), dev(b))
    q1, s1 = sq.ln_quantize(to_dev_16(x, F16), dev(g), dev(b), layout=sq.TILED)
    assert np.array_equal(tiled_to_rows(q1), q0.cpu().numpy()) and torch.equal(s0, s1)
