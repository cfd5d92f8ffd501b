"""The 256x384 output tile of the prefill GEMM (taken where it saves a round of tiles: many tokens, wide C_o, long
C_i) with everything its two-half epilogue has to handle: ragged last row block and last column tile, bias, ReLU,
residual, per-channel weight steps, both operand layouts, fp16 / bf16, and the int8 (fused static quantizer) output.
Sampled rows (tile and half-tile borders included) against the oracle, int32 accumulators of those rows exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import assert_identical_16, BF16, F16, bits_from_dev, dev, random_bf16_bits, rows_to_tiled_dev, to_dev_16, torch_dtype, ulp_distance

pytestmark = pytest.mark.gpu

T, C_I = 2040, 12288  # 8 row blocks (the last one ragged), 192 K steps: the planner picks the 384-wide tile (one round of 256 tiles)


def _rows(t):
    rng = np.random.default_rng(11)
    rows = set(rng.choice(t, size=24, replace=False).tolist())
    rows.update({0, 127, 128, 255, 256, 383, t - 129, t - 128, t - 1})  # tile, half-tile and wave borders
    return np.array(sorted(rows), dtype=np.int64)


@pytest.mark.parametrize("c_o,tiled,odt,per_channel", [(12280, False, F16, False), (12288, True, BF16, True)])
def test_wide_tile_epilogue_variants(c_o, tiled, odt, per_channel):
    print(f"[case] wide tile t={T} c_i={C_I} c_o={c_o} tiled={tiled} out={odt} per_channel={per_channel}", flush=True)
    rng = np.random.default_rng(c_o)
    xq = synth.int8_codes((T, C_I), 301)
    wq = synth.int8_codes((c_o, C_I), 302)
    xs = (rng.random(T, dtype=np.float32) + np.float32(0.5)) * np.float32(2e-3)
    ws = ((rng.random(c_o, dtype=np.float32) + np.float32(0.5)) * np.float32(3e-3)) if per_channel else np.array([3e-3], np.float32)
    bias = synth.bias(c_o, 303)
    res = random_bf16_bits((T, c_o), 304) if odt == BF16 else synth.normal_fp16((T, c_o), 304)
    rows = _rows(T)
    lay = sq.TILED if tiled else sq.ROW_MAJOR
    xq_d, wq_d = (rows_to_tiled_dev(xq), rows_to_tiled_dev(wq)) if tiled else (dev(xq), dev(wq))
    rows_d = torch.from_numpy(rows).cuda()

    acc = sq.i8_gemm_i32(xq_d, wq_d, layout=lay)
    want = oracle.i8_gemm_i32(np.ascontiguousarray(xq[rows]), wq)
    assert np.array_equal(acc[rows_d].cpu().numpy(), want)
    del acc

    for kw in (dict(), dict(bias=True, relu=True, residual=True)):
        ref = oracle.w8a8_linear(xq, xs, wq, ws, odt, bias=bias if kw else None, residual_bits=res if kw else None,
                                 relu=bool(kw), rows=rows, w_per_channel=per_channel)
        y = sq.w8a8_linear(xq_d, dev(xs), wq_d, dev(ws), torch_dtype(odt), bias=dev(bias) if kw else None,
                           residual=to_dev_16(res, odt) if kw else None, relu=bool(kw), layout=lay, w_per_channel=per_channel)
        d = ulp_distance(bits_from_dev(y[rows_d]), ref[rows])
        assert_identical_16(d)
        del y

    # int8 output with the next layer's static step
    full = oracle.w8a8_linear(xq, xs, wq, ws, odt, bias=bias, relu=True, rows=rows, w_per_channel=per_channel)
    step = np.float32(0.7) * np.float32(np.abs(oracle.f32_from_bits16(full[rows], odt)).max()) / np.float32(127.0)
    ref_q, _ = oracle.quantize_act(full[rows], odt, oracle.PER_TENSOR_STATIC, static_scale=step)
    out_tiled = tiled and c_o % 64 == 0
    yq = sq.w8a8_linear_q8(xq_d, dev(xs), wq_d, dev(ws), dev(np.array([step], np.float32)), torch_dtype(odt), bias=dev(bias),
                           relu=True, layout=lay, out_layout=sq.TILED if out_tiled else sq.ROW_MAJOR, w_per_channel=per_channel)
    if out_tiled:
        from tests._util import tiled_to_rows
        got = tiled_to_rows(yq)[rows]
    else:
        got = yq[rows_d].cpu().numpy()
    assert np.array_equal(got, ref_q)
