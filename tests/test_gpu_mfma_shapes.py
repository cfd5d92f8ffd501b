"""The compute-bound GEMM tiles exist in two MFMA shapes: 16x16x64 (taken when the K range is an even number of whole
64-byte steps and is not split) and 32x32x32 (everything else).  These shapes are chosen so that the planner's cost
model picks the 256x256, the 256x384 and the 256x192 tile in each of the two forms (300 tokens = one full and one ragged row block;
32760 / 49144 output channels = one round of 256 tiles with a ragged last column tile; 4096 resp. 4160 input
channels = 64 resp. 65 K steps), in both operand layouts.  Sampled rows against the oracle: int32 accumulators exact,
16-bit outputs with bias, ReLU and residual identical."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import assert_identical_16, BF16, F16, bits_from_dev, dev, random_bf16_bits, rows_to_tiled_dev, to_dev_16, torch_dtype, ulp_distance

pytestmark = pytest.mark.gpu

T = 300
ROWS = np.array([0, 15, 16, 63, 64, 127, 128, 255, 256, 271, 299], dtype=np.int64)  # wave, block and tile borders


@pytest.mark.parametrize("c_i,c_o,tiled,odt", [
    (4096, 32760, False, F16),   # 256x256, 16x16x64
    (4160, 32760, True, BF16),   # 256x256, 32x32x32 (65 K steps)
    (4096, 49144, True, BF16),   # 256x384, 16x16x64
    (4160, 49144, False, F16),   # 256x384, 32x32x32
    (4112, 32760, False, BF16),  # 256x256, 32x32x32 with a K tail (row-major only)
    (384, 49144, True, F16),     # 256x384, 16x16x64 on the shortest K range that form takes (6 steps: 3 in flight before the loop)
    (640, 49144, False, BF16),   # 256x384, 16x16x64, 10 steps
    (12288, 24568, True, BF16),  # 256x192, 16x16x64 (taken from 192 K steps on: an odd number of parts per step, 5-stage ring)
    (12352, 24568, False, F16),  # 256x192, 32x32x32 (193 K steps)
])
def test_tile_forms_vs_oracle(c_i, c_o, tiled, odt):
    print(f"[case] tile forms t={T} c_i={c_i} c_o={c_o} tiled={tiled} out={odt}", flush=True)
    rng = np.random.default_rng(c_i + c_o)
    xq = synth.int8_codes((T, c_i), 401)
    wq = synth.int8_codes((c_o, c_i), 402)
    xs = (rng.random(T, dtype=np.float32) + np.float32(0.5)) * np.float32(2e-3)
    ws = np.array([3e-3], np.float32)
    bias = synth.bias(c_o, 403)
    res = random_bf16_bits((T, c_o), 404) if odt == BF16 else synth.normal_fp16((T, c_o), 404)
    lay = sq.TILED if tiled else sq.ROW_MAJOR
    xq_d, wq_d = (rows_to_tiled_dev(xq), rows_to_tiled_dev(wq)) if tiled else (dev(xq), dev(wq))
    rows_d = torch.from_numpy(ROWS).cuda()

    acc = sq.i8_gemm_i32(xq_d, wq_d, layout=lay)
    assert np.array_equal(acc[rows_d].cpu().numpy(), oracle.i8_gemm_i32(np.ascontiguousarray(xq[ROWS]), wq))
    del acc
    for kw in (dict(), dict(bias=True, relu=True, residual=True)):
        ref = oracle.w8a8_linear(xq, xs, wq, ws, odt, bias=bias if kw else None, residual_bits=res if kw else None,
                                 relu=bool(kw), rows=ROWS)
        y = sq.w8a8_linear(xq_d, dev(xs), wq_d, dev(ws), torch_dtype(odt), bias=dev(bias) if kw else None,
                           residual=to_dev_16(res, odt) if kw else None, relu=bool(kw), layout=lay)
        assert_identical_16(ulp_distance(bits_from_dev(y[rows_d]), ref[ROWS]))
        del y


def test_batched_product_on_the_16x16x64_tile():
    """A batched Q K^T-shaped product with a long contraction (30 x [300, 2048] x [1024, 2048]^T): 240 tiles of 256x256
    in one round against two rounds of 256x192, so the batched launch takes the 16x16x64 form; three batch entries
    against the oracle, every element."""
    b, m, n, k = 30, 300, 1024, 2048
    print(f"[case] batched product b={b} m={m} n={n} k={k}", flush=True)
    a = synth.int8_codes((b, m, k), 411)
    kt = synth.int8_codes((b, n, k), 412)
    alpha = float(np.float32(2e-4))
    got = sq.w8a8_bmm(dev(a), dev(kt), True, alpha, torch.float16)
    for i in (0, 13, 29):
        ref = oracle.w8a8_bmm(a[i:i + 1], kt[i:i + 1], True, alpha, F16)
        assert_identical_16(ulp_distance(bits_from_dev(got[i:i + 1]), ref), f"batch entry {i}")


# Seeded shapes that the planner's cost model sends to the 256- and 384-wide tiles, about half of them in each MFMA form
# (the general random sweep of test_gpu_random_shapes.py stays below one round of tiles and so on the 256x192 tile):
# (t, c_i, c_o, tiled)
WIDE_TILE_SHAPES = [
    (768, 1904, 30064, False), (700, 2144, 24112, False), (255, 2416, 57112, False), (500, 1344, 41992, False),
    (384, 384, 25456, True), (700, 576, 53440, True), (130, 2080, 62664, False), (129, 1600, 53552, False),
    (513, 1408, 61968, True), (256, 2480, 53872, False), (512, 1664, 41280, True), (513, 1536, 60736, False),
    (512, 2048, 25120, False), (255, 1664, 64000, True),
]


@pytest.mark.parametrize("t,c_i,c_o,tiled", WIDE_TILE_SHAPES)
def test_random_shapes_on_the_wide_tiles(t, c_i, c_o, tiled):
    print(f"[case] wide-tile sweep t={t} c_i={c_i} c_o={c_o} tiled={tiled}", flush=True)
    seed = t * 131 + c_i * 7 + c_o
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([rng.choice(t, size=6, replace=False), [0, min(t - 1, 127), min(t - 1, 128), t - 1]])).astype(np.int64)
    odt = BF16 if rng.integers(0, 2) else F16
    per_token, use_bias, relu, use_res = (bool(rng.integers(0, 2)) for _ in range(4))
    xq = synth.int8_codes((t, c_i), seed + 1)
    wq = synth.int8_codes((c_o, c_i), seed + 2)
    xs = (rng.random(t if per_token else 1, dtype=np.float32) * np.float32(0.01) + np.float32(1e-3)).astype(np.float32)
    ws = np.array([2e-3], np.float32)
    bias = synth.bias(c_o, seed + 3) if use_bias else None
    res = None
    if use_res:
        res = synth.normal_fp16((t, c_o), seed + 4) if odt == F16 else random_bf16_bits((t, c_o), seed + 4)
    lay = sq.TILED if tiled else sq.ROW_MAJOR
    xq_d, wq_d = (rows_to_tiled_dev(xq), rows_to_tiled_dev(wq)) if tiled else (dev(xq), dev(wq))
    rows_d = torch.from_numpy(rows).cuda()
    acc = sq.i8_gemm_i32(xq_d, wq_d, layout=lay)
    assert np.array_equal(acc[rows_d].cpu().numpy(), oracle.i8_gemm_i32(np.ascontiguousarray(xq[rows]), wq))
    del acc
    ref = oracle.w8a8_linear(xq, xs, wq, ws, odt, bias=bias, residual_bits=res, relu=relu, rows=rows)
    y = sq.w8a8_linear(xq_d, dev(xs), wq_d, dev(ws), torch_dtype(odt), bias=None if bias is None else dev(bias),
                       residual=None if res is None else to_dev_16(res, odt), relu=relu, layout=lay)
    assert_identical_16(ulp_distance(bits_from_dev(y[rows_d]), ref[rows]))
