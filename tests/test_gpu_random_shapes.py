"""Seeded sweep of random small shapes through every GEMM path and both operand layouts: int32 accumulators exact,
16-bit outputs within 1 ulp, int8 outputs (fused static quantizer) identical to the oracle's chain.  The shapes are
drawn so that all dispatch branches are hit many times: few tokens against narrow / wide C_o (split-K tiles, weight
streaming with and without a K split), many tokens with short and long K (one-shot tiles, 256x256 / 256x192 tiles),
ragged edges in every dimension."""
import numpy as np
import pytest

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import (assert_identical_16, BF16, F16, bits_from_dev, dev, random_bf16_bits, rows_to_tiled_dev, tiled_to_rows, to_dev_16,
                         torch_dtype, ulp_distance)

pytestmark = pytest.mark.gpu


def _shapes(seed, n):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        t = int(rng.choice([1, 2, 7, 16, 17, 31, 33, 64, 65, 100, 128, 129, 200, 257, 300, 520]))
        tiled = bool(rng.integers(0, 2))
        c_i = int(rng.integers(1, 40)) * (64 if tiled else 16)
        wide = bool(rng.integers(0, 2))
        c_o = int(rng.integers(512, 900)) * 8 if wide else int(rng.integers(1, 300)) * 8
        out.append((t, c_i, c_o, tiled))
    return out


@pytest.mark.parametrize("t,c_i,c_o,tiled", _shapes(20221118, 48))
def test_random_shape_gemm_and_linear(t, c_i, c_o, tiled):
    print(f"[case] random shape t={t} c_i={c_i} c_o={c_o} tiled={tiled}", flush=True)
    seed = t * 131 + c_i * 7 + c_o
    rng = np.random.default_rng(seed)
    lay = sq.TILED if tiled else sq.ROW_MAJOR
    xq = synth.int8_codes((t, c_i), seed + 1)
    wq = synth.int8_codes((c_o, c_i), seed + 2)
    xq_d, wq_d = (rows_to_tiled_dev(xq), rows_to_tiled_dev(wq)) if tiled else (dev(xq), dev(wq))
    acc = sq.i8_gemm_i32(xq_d, wq_d, layout=lay).cpu().numpy()
    assert np.array_equal(acc, oracle.i8_gemm_i32(xq, wq))
    odt = BF16 if rng.integers(0, 2) else F16
    per_token, use_bias, relu, use_res, w_pc = (bool(rng.integers(0, 2)) for _ in range(5))
    xs = (rng.random(t if per_token else 1, dtype=np.float32) * np.float32(0.01) + np.float32(1e-3)).astype(np.float32)
    ws = (rng.random(c_o if w_pc else 1, dtype=np.float32) * np.float32(0.01) + np.float32(1e-3)).astype(np.float32)
    bias = synth.bias(c_o, seed + 3) if use_bias else None
    res = None
    if use_res:
        res = synth.normal_fp16((t, c_o), seed + 4) if odt == F16 else random_bf16_bits((t, c_o), seed + 4)
    ref = oracle.w8a8_linear(xq, xs, wq, ws, odt, bias=bias, residual_bits=res, relu=relu, w_per_channel=w_pc)
    y = sq.w8a8_linear(xq_d, dev(xs), wq_d, dev(ws), torch_dtype(odt), bias=None if bias is None else dev(bias),
                       residual=None if res is None else to_dev_16(res, odt), relu=relu, layout=lay, w_per_channel=w_pc)
    d = ulp_distance(bits_from_dev(y), ref)
    assert_identical_16(d)
    # the same layer with the next kernel's static quantizer fused in
    out_tiled = tiled and c_o % 64 == 0
    step = np.float32(0.8) * np.float32(np.abs(oracle.f32_from_bits16(ref, odt)).max()) / np.float32(127.0)
    ref_q, _ = oracle.quantize_act(ref, odt, oracle.PER_TENSOR_STATIC, static_scale=step)
    yq = sq.w8a8_linear_q8(xq_d, dev(xs), wq_d, dev(ws), dev(np.array([step], np.float32)), torch_dtype(odt),
                           bias=None if bias is None else dev(bias), residual=None if res is None else to_dev_16(res, odt),
                           relu=relu, layout=lay, out_layout=sq.TILED if out_tiled else sq.ROW_MAJOR, w_per_channel=w_pc)
    got = tiled_to_rows(yq) if out_tiled else yq.cpu().numpy()
    assert np.array_equal(got, ref_q)


@pytest.mark.parametrize("seed", range(12))
def test_random_shape_bmm(seed):
    rng = np.random.default_rng(900 + seed)
    b = int(rng.integers(1, 6))
    m = int(rng.choice([1, 16, 33, 100, 128, 200, 300, 512]))
    k = int(rng.integers(1, 20)) * 16
    n = int(rng.integers(1, 24)) * 16
    odt = BF16 if seed % 2 else F16
    print(f"[case] random bmm b={b} m={m} n={n} k={k}", flush=True)
    a = synth.int8_codes((b, m, k), 910 + seed)
    kt = synth.int8_codes((b, n, k), 920 + seed)
    v = synth.int8_codes((b, k, n), 930 + seed)
    alpha = float(np.float32(3e-4))
    ref1 = oracle.w8a8_bmm(a, kt, True, alpha, odt)
    got1 = sq.w8a8_bmm(dev(a), dev(kt), True, alpha, torch_dtype(odt))
    assert ulp_distance(bits_from_dev(got1), ref1).max() <= 1
    ref2 = oracle.w8a8_bmm(a, v, False, alpha, odt)
    got2 = sq.w8a8_bmm(dev(a), dev(v), False, alpha, torch_dtype(odt))
    assert ulp_distance(bits_from_dev(got2), ref2).max() <= 1
