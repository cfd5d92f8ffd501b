"""Pins for the CPU oracle: closed forms, invariants, worked examples, library special cases and
brute force.  None of these re-types the oracle's own formula: each checks a property the paper or
the mathematics fixes, so that a dropped term, a wrong axis or a transposed operand fails here.
CPU only."""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2211_10438_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
F16, BF16 = oracle.F16, oracle.BF16


# ------------------------------------------------------------------ 16-bit conversions vs libraries

def test_fp16_widening_matches_numpy_for_all_bit_patterns():
    L = oracle.lib()
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([L.orc_h2f(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def _interesting_floats(seed):
    rng = np.random.default_rng(seed)
    vals = [rng.standard_normal(20000).astype(np.float32) * s for s in (1e-8, 1e-6, 1e-4, 1.0, 300.0, 7e4)]
    # exact ties and neighbours of every fp16 value: midpoints between consecutive fp16 numbers
    h = np.arange(0, 0x7c00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = ((h[:-1] + h[1:]) / 2).astype(np.float32)
    vals += [mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf)), -mid]
    vals.append(np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e9, -1e9, np.inf, -np.inf,
                          2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -26], dtype=np.float32))
    return np.concatenate(vals)


def test_fp16_narrowing_is_round_to_nearest_even_like_numpy():
    L = oracle.lib()
    v = _interesting_floats(1)
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16).view(np.uint16)
    got = np.array([L.orc_f2h(float(x)) for x in v], dtype=np.uint16)
    assert np.array_equal(got, ref)


def test_bf16_conversions_match_torch():
    L = oracle.lib()
    v = _interesting_floats(2)
    ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([L.orc_f2bf(float(x)) for x in v], dtype=np.uint16)
    assert np.array_equal(got, ref)
    back = np.array([L.orc_bf2f(int(b)) for b in got[:5000]], dtype=np.float32)
    ref_back = torch.from_numpy(ref[:5000].view(np.int16)).view(torch.bfloat16).float().numpy()
    ok = np.isnan(ref_back) | (back == ref_back)
    assert ok.all()


# ------------------------------------------------------------------ Eq. 4 / Eq. 3

def test_smooth_scales_closed_form_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "smooth_scales_closed_form.txt")) if l[0] not in "#\n"]
    for ax, aw, alpha, s_ref in rows:
        s, inv_s = oracle.smooth_scales(np.array([ax], np.float32), np.array([aw], np.float32), float(alpha))
        assert s[0] == pytest.approx(float(s_ref), rel=1e-6), (ax, aw, alpha)
        assert inv_s[0] == pytest.approx(1.0 / float(s_ref), rel=1e-6)


def _case(t=48, c_i=96, c_o=80, seed=5):
    c = synth.linear_case(t, c_i, c_o, 0.0, 50.0, seed, n_out=5, calib_tokens=64)
    ax = oracle.act_absmax_per_channel(c["x_calib"], F16)
    aw = oracle.weight_absmax_per_in_channel(c["w"], F16)
    return c, ax, aw


def test_absmax_axes():
    c, ax, aw = _case()
    assert ax.shape == (96,) and aw.shape == (96,)
    assert np.array_equal(ax, np.abs(c["x_calib"].astype(np.float32)).max(axis=0))
    # max|W_j| runs along the row of W [C_i, C_o] that belongs to input channel j
    assert np.array_equal(aw, np.abs(c["w"].astype(np.float32)).max(axis=1))
    # the outlier channels must dominate the activation maxima
    assert set(np.argsort(ax)[-5:]) == set(c["channels"])


@pytest.mark.parametrize("alpha", [0.0, 0.25, 0.5, 0.8, 1.0])
def test_smoothing_equivalence_invariant(alpha):
    """(X diag(s)^-1)(diag(s) W) = X W (Eq. 3), fp64, relative 1e-5."""
    c, ax, aw = _case()
    s, inv_s = oracle.smooth_scales(ax, aw, alpha)
    x = c["x"].astype(np.float64)
    w = c["w"].astype(np.float64)
    y = x @ w
    y_s = (x * inv_s.astype(np.float64)) @ (w * s.astype(np.float64)[:, None])
    assert np.abs(y_s - y).max() <= 1e-5 * np.abs(y).max()
    assert np.allclose(s.astype(np.float64) * inv_s.astype(np.float64), 1.0, rtol=2e-7)


def test_smoothing_extreme_and_balanced_choices():
    c, ax, aw = _case()
    xc = np.abs(c["x_calib"].astype(np.float64))
    w = np.abs(c["w"].astype(np.float64))
    s1, _ = oracle.smooth_scales(ax, aw, 1.0)  # s_j = max|X_j|: every smoothed channel peaks at 1
    assert np.allclose((xc / s1).max(axis=0), 1.0, rtol=1e-6)
    s0, _ = oracle.smooth_scales(ax, aw, 0.0)  # s_j = 1/max|W_j|: every smoothed weight row peaks at 1
    assert np.allclose((w * s0[:, None]).max(axis=1), 1.0, rtol=1e-6)
    sh, _ = oracle.smooth_scales(ax, aw, 0.5)  # both sides share sqrt(ax*aw)
    target = np.sqrt(ax.astype(np.float64) * aw.astype(np.float64))
    assert np.allclose((xc / sh).max(axis=0), target, rtol=1e-6)
    assert np.allclose((w * sh[:, None]).max(axis=1), target, rtol=1e-6)
    same, inv = oracle.smooth_scales(ax, ax, 0.5)
    assert np.allclose(same, 1.0, rtol=1e-7) and np.allclose(inv, 1.0, rtol=1e-7)


def test_smooth_scales_guards():
    s, inv_s = oracle.smooth_scales(np.zeros(4, np.float32), np.ones(4, np.float32), 0.5)
    assert np.all(np.isfinite(s)) and np.all(s > 0) and np.all(np.isfinite(inv_s))
    with pytest.raises(ValueError):
        oracle.smooth_scales(np.ones(4, np.float32), np.ones(4, np.float32), 1.5)


# ------------------------------------------------------------------ Eq. 1

def test_quantizer_worked_examples_fixture():
    for line in open(os.path.join(GOLDEN, "quantizer_worked_examples.txt")):
        if line[0] in "#\n":
            continue
        xs, delta, codes = [np.array(p.split(), dtype=np.float64) for p in line.split("|")]
        x = xs.astype(np.float16)[None, :]
        assert np.array_equal(x.astype(np.float64)[0], xs)  # fixture values are exact in fp16
        for mode in (oracle.PER_TOKEN_DYNAMIC, oracle.PER_TENSOR_DYNAMIC):
            q, sc = oracle.quantize_act(x, F16, mode)
            assert sc[0] == delta[0]
            assert np.array_equal(q[0], codes.astype(np.int8)), line
        q, _ = oracle.quantize_act(x, F16, oracle.PER_TENSOR_STATIC, static_scale=delta[0])
        assert np.array_equal(q[0], codes.astype(np.int8))


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN_DYNAMIC, oracle.PER_TENSOR_DYNAMIC])
@pytest.mark.parametrize("with_s", [False, True])
def test_quantizer_error_bound_and_range(mode, with_s):
    c, ax, aw = _case(t=64, c_i=200)
    inv_s = oracle.smooth_scales(ax, aw, 0.5)[1] if with_s else None
    q, sc = oracle.quantize_act(c["x"], F16, mode, inv_s=inv_s)
    xh = c["x"].astype(np.float32)
    if with_s:
        xh = xh * inv_s  # one fp32 multiply, exactly what smoothing an fp16 activation means
    xh = xh.astype(np.float64)
    delta = sc.astype(np.float64)[:, None] if mode == oracle.PER_TOKEN_DYNAMIC else sc.astype(np.float64)[0]
    assert q.min() >= -127 and q.max() <= 127
    err = np.abs(xh - q.astype(np.float64) * delta)
    assert np.all(err <= delta / 2 * (1 + 2.0 ** -12))
    amax = np.abs(xh).max(axis=1) if mode == oracle.PER_TOKEN_DYNAMIC else np.abs(xh).max()
    assert np.allclose(np.atleast_1d(delta).ravel() * 127.0, np.atleast_1d(amax).ravel(), rtol=1e-6)
    if mode == oracle.PER_TOKEN_DYNAMIC:
        assert np.all(np.abs(q).max(axis=1) == 127)  # the arg-max element of every token maps to +-127
        j = np.abs(xh).argmax(axis=1)
        assert np.array_equal(q[np.arange(q.shape[0]), j], 127 * np.sign(xh[np.arange(q.shape[0]), j]).astype(np.int8))
    else:
        assert np.abs(q).max() == 127


def test_quantizer_degenerate_and_static_cases():
    z = np.zeros((3, 16), np.float16)
    for mode in (oracle.PER_TOKEN_DYNAMIC, oracle.PER_TENSOR_DYNAMIC):
        q, sc = oracle.quantize_act(z, F16, mode)
        assert not q.any() and not sc.any()
    x = np.array([[1.0, -300.0, 0.5, 127.0, 128.0, -126.5]], np.float16)
    q, _ = oracle.quantize_act(x, F16, oracle.PER_TENSOR_STATIC, static_scale=1.0)
    assert q.tolist() == [[1, -127, 0, 127, 127, -126]]  # saturation + tie to even
    # per-token on one row equals per-tensor dynamic on that row; rows are independent
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 64)).astype(np.float16)
    qt, st = oracle.quantize_act(x, F16, oracle.PER_TOKEN_DYNAMIC)
    for i in range(5):
        q1, s1 = oracle.quantize_act(x[i:i + 1], F16, oracle.PER_TENSOR_DYNAMIC)
        assert np.array_equal(q1[0], qt[i]) and s1[0] == st[i]
    # row stride: a padded buffer gives the same codes as the packed one
    xp = np.zeros((5, 80), np.float16)
    xp[:, :64] = x
    xp[:, 64:] = 1000.0  # must be ignored
    qp, sp = oracle.quantize_act(xp, F16, oracle.PER_TOKEN_DYNAMIC, c_i=64)
    assert np.array_equal(qp, qt) and np.array_equal(sp, st)


def test_quantizer_bf16_input_grid_idempotence():
    k = np.arange(-127, 128, dtype=np.float32)
    xb = oracle.bf16_bits_from_f32(k * 0.5)[None, :]  # k/2 is exact in bf16 for |k| <= 127
    q, sc = oracle.quantize_act(xb, BF16, oracle.PER_TOKEN_DYNAMIC)
    assert sc[0] == 0.5 and np.array_equal(q[0], k.astype(np.int8))


def test_prepare_weight_matches_quantizer_on_transposed_smoothed_weight():
    c, ax, aw = _case()
    s, _ = oracle.smooth_scales(ax, aw, 0.5)
    wq, ws = oracle.prepare_weight(c["w"], F16, s)
    assert wq.shape == (80, 96)  # [C_o, C_i]: contraction index contiguous
    wh = (c["w"].astype(np.float32) * s[:, None]).astype(np.float64)
    assert np.isclose(ws[0] * 127.0, np.abs(wh).max(), rtol=1e-6)
    err = np.abs(wh.T - wq.astype(np.float64) * float(ws[0]))
    assert np.all(err <= float(ws[0]) / 2 * (1 + 2.0 ** -12))
    assert np.abs(wq).max() == 127
    wq1, ws1 = oracle.prepare_weight(c["w"], F16, None)  # s = 1
    assert np.isclose(ws1[0] * 127.0, np.abs(c["w"].astype(np.float64)).max(), rtol=1e-6)
    assert not np.array_equal(wq1, wq)


def test_prepare_weight_per_channel_pins():
    """Per-output-channel weight steps (the weight granularity of Table 7)."""
    c, ax, aw = _case()
    s, _ = oracle.smooth_scales(ax, aw, 0.5)
    wq, ws = oracle.prepare_weight(c["w"], F16, s, per_channel=True)
    assert wq.shape == (80, 96) and ws.shape == (80,)
    wh = (c["w"].astype(np.float32) * s[:, None]).astype(np.float64)  # W_hat [C_i, C_o]
    # every column: step = its own absmax / 127, every code within half a step, the extreme code is used
    assert np.allclose(ws.astype(np.float64) * 127.0, np.abs(wh).max(axis=0), rtol=1e-6)
    err = np.abs(wh.T - wq.astype(np.float64) * ws[:, None].astype(np.float64))
    assert np.all(err <= ws[:, None].astype(np.float64) / 2 * (1 + 2.0 ** -12))
    assert np.all(np.abs(wq).max(axis=1) == 127)
    # a column equals the per-tensor quantizer run on that column alone (brute force through another function)
    for n in (0, 17, 79):
        col = np.ascontiguousarray(c["w"][:, n:n + 1])
        wq1, ws1 = oracle.prepare_weight(col, F16, s)
        assert np.array_equal(wq1[0], wq[n]) and ws1[0] == ws[n]
    # when every column has the same absmax, per-channel and per-tensor agree
    w2 = c["w"].copy()
    w2[0, :] = np.float16(8.0)  # dominates every column (|w| ~ 0.02), s = 1
    a, sa = oracle.prepare_weight(w2, F16, None, per_channel=True)
    b, sb = oracle.prepare_weight(w2, F16, None)
    assert np.array_equal(a, b) and np.all(sa == sb[0])
    # an all-zero column: step 0, codes 0
    w3 = c["w"].copy()
    w3[:, 5] = 0
    z, sz = oracle.prepare_weight(w3, F16, None, per_channel=True)
    assert sz[5] == 0.0 and not z[5].any()


# ------------------------------------------------------------------ integer contraction

def test_int_gemm_brute_force_tiny():
    xq = synth.int8_codes((3, 5), 11)
    wq = synth.int8_codes((4, 5), 12)
    acc = oracle.i8_gemm_i32(xq, wq)
    for i, n in itertools.product(range(3), range(4)):
        assert acc[i, n] == sum(int(xq[i, j]) * int(wq[n, j]) for j in range(5))


def test_int_gemm_matches_numpy_int64_and_extremes():
    xq = synth.int8_codes((37, 200), 13)
    wq = synth.int8_codes((53, 200), 14)
    assert np.array_equal(oracle.i8_gemm_i32(xq, wq).astype(np.int64), xq.astype(np.int64) @ wq.astype(np.int64).T)
    # one-hot weight rows pick activation columns
    eye = np.zeros((200, 200), np.int8)
    eye[np.arange(200), np.arange(200)[::-1]] = 1
    assert np.array_equal(oracle.i8_gemm_i32(xq, eye), xq[:, ::-1].astype(np.int32))
    # the largest accumulator the configs can produce does not wrap: 49152 * 127^2
    full = np.full((1, 49152), 127, np.int8)
    assert oracle.i8_gemm_i32(full, -full)[0, 0] == -49152 * 127 * 127


# ------------------------------------------------------------------ Eq. 2 epilogue

def test_linear_factorisation_eq2():
    """Dequantized output equals the fp64 product of the dequantized operands to 16-bit rounding."""
    c, ax, aw = _case(t=40, c_i=128, c_o=72)
    s, inv_s = oracle.smooth_scales(ax, aw, 0.5)
    wq, ws = oracle.prepare_weight(c["w"], F16, s)
    xq, xs = oracle.quantize_act(c["x"], F16, oracle.PER_TOKEN_DYNAMIC, inv_s=inv_s)
    ref = (xq.astype(np.float64) * xs.astype(np.float64)[:, None]) @ (wq.astype(np.float64).T * float(ws[0]))
    for dt, rel in ((F16, 2.0 ** -10), (BF16, 2.0 ** -7)):
        y = oracle.f32_from_bits16(oracle.w8a8_linear(xq, xs, wq, ws, dt), dt).astype(np.float64)
        assert np.all(np.abs(y - ref) <= rel * np.abs(ref) + 6e-8)
    # and the whole pipeline approximates X W: smoothing must help on outlier activations (Sec. 3)
    exact = c["x"].astype(np.float64) @ c["w"].astype(np.float64)
    wq0, ws0 = oracle.prepare_weight(c["w"], F16, None)
    for mode in (oracle.PER_TOKEN_DYNAMIC, oracle.PER_TENSOR_DYNAMIC):
        xq0, xs0 = oracle.quantize_act(c["x"], F16, mode)
        xq1, xs1 = oracle.quantize_act(c["x"], F16, mode, inv_s=inv_s)
        y0 = oracle.f32_from_bits16(oracle.w8a8_linear(xq0, xs0, wq0, ws0, F16), F16).astype(np.float64)
        y1 = oracle.f32_from_bits16(oracle.w8a8_linear(xq1, xs1, wq, ws, F16), F16).astype(np.float64)
        e0 = np.linalg.norm(y0 - exact) / np.linalg.norm(exact)
        e1 = np.linalg.norm(y1 - exact) / np.linalg.norm(exact)
        assert e1 < 0.5 * e0, (mode, e0, e1)


def test_epilogue_exact_cases():
    xq = np.array([[1, -2, 3, 4], [0, 0, 0, 0], [127, 127, 127, 127]], np.int8)
    wq = np.array([[1, 1, 1, 1], [-1, 2, -3, 4], [127, 127, 127, 127]], np.int8)
    acc = xq.astype(np.int64) @ wq.astype(np.int64).T  # [[6,6,762],[0,0,0],[508,254,64516]]
    xs = np.array([0.5, 4.0, 0.25], np.float32)  # powers of two: every product is exact
    ws = np.array([0.125], np.float32)
    ref = acc * xs[:, None].astype(np.float64) * 0.125
    y = oracle.f32_from_bits16(oracle.w8a8_linear(xq, xs, wq, ws, F16), F16)
    assert np.array_equal(y.astype(np.float64), ref.astype(np.float16).astype(np.float64))
    bias = np.array([1.0, -1.0, 0.5], np.float32)
    res = np.full((3, 3), 2.0, np.float16)
    y = oracle.f32_from_bits16(oracle.w8a8_linear(xq, xs, wq, ws, F16, bias=bias, relu=True, residual_bits=res), F16)
    want = np.maximum(ref + bias, 0.0) + 2.0  # bias before ReLU, residual after
    assert np.array_equal(y.astype(np.float64), want.astype(np.float16).astype(np.float64))
    # per-tensor activation scale: one entry
    y = oracle.f32_from_bits16(oracle.w8a8_linear(xq, np.array([2.0], np.float32), wq, ws, BF16), BF16)
    want = torch.from_numpy(acc * 0.25).to(torch.bfloat16).double().numpy()
    assert np.array_equal(y.astype(np.float64), want)
    # row subset computes exactly those rows
    part = oracle.w8a8_linear(xq, xs, wq, ws, F16, rows=[2])
    full = oracle.w8a8_linear(xq, xs, wq, ws, F16)
    assert np.array_equal(part[2], full[2]) and not part[:2].any()


def test_linear_per_channel_weight_scale():
    xq = synth.int8_codes((4, 32), 21)
    wq = synth.int8_codes((6, 32), 22)
    xs = np.array([0.5, 1.0, 0.25, 0.125], np.float32)
    wsc = np.array([1.0, 0.5, 0.25, 2.0 ** -4, 2.0 ** -5, 0.125], np.float32)
    y = oracle.f32_from_bits16(oracle.w8a8_linear(xq, xs, wq, wsc, F16, w_per_channel=True), F16).astype(np.float64)
    ref = (xq.astype(np.int64) @ wq.astype(np.int64).T) * xs[:, None].astype(np.float64) * wsc[None, :]
    assert np.array_equal(y, ref.astype(np.float16).astype(np.float64))


# ------------------------------------------------------------------ attention BMMs

def test_bmm_layouts_against_numpy():
    a = synth.int8_codes((3, 7, 24), 31)
    bt = synth.int8_codes((3, 9, 24), 32)  # [b, n, k]
    alpha = 2.0 ** -6
    ref = np.einsum("bmk,bnk->bmn", a.astype(np.int64), bt.astype(np.int64)) * alpha
    c = oracle.f32_from_bits16(oracle.w8a8_bmm(a, bt, True, alpha, F16), F16)
    assert np.array_equal(c.astype(np.float64), ref.astype(np.float16).astype(np.float64))
    bn = np.ascontiguousarray(bt.transpose(0, 2, 1))  # [b, k, n]
    c2 = oracle.f32_from_bits16(oracle.w8a8_bmm(a, bn, False, alpha, F16), F16)
    assert np.array_equal(c2, c)
    # batch 1 is the linear-layer contraction with unit scales
    acc = oracle.i8_gemm_i32(a[1], bt[1])
    c1 = oracle.f32_from_bits16(oracle.w8a8_bmm(a[1:2], bt[1:2], True, 0.125, F16), F16)
    assert np.array_equal(c1[0].astype(np.float64), (acc * 0.125).astype(np.float16).astype(np.float64))
    # batch subset
    sub = oracle.w8a8_bmm(a, bt, True, alpha, F16, batches=[2])
    assert np.array_equal(oracle.f32_from_bits16(sub[2], F16), c[2]) and not sub[:2].any()


def test_softmax_quant_special_cases():
    from scipy.special import softmax
    s = np.zeros((1, 8), np.float16)  # uniform row: p = 1/8 exactly, code = round(15.875) = 16
    assert oracle.softmax_quant_p(s, F16).tolist() == [[16] * 8]
    s = np.full((1, 6), -20.0, np.float16)
    s[0, 2] = 20.0  # one dominant score
    assert oracle.softmax_quant_p(s, F16).tolist() == [[0, 0, 127, 0, 0, 0]]
    rng = np.random.default_rng(41)
    s = (rng.standard_normal((32, 300)) * 3).astype(np.float16)
    pq = oracle.softmax_quant_p(s, F16)
    p16 = softmax(s.astype(np.float64), axis=-1).astype(np.float16)
    want = np.rint(p16.astype(np.float32) * np.float32(127.0)).astype(np.int8)
    assert np.array_equal(pq, want)
    assert pq.min() >= 0 and np.all(np.abs(pq.astype(np.int64).sum(axis=1) - 127) <= 0.5 * 300)
    # shifting a row by a constant that is exact in fp16 leaves the probabilities unchanged
    si = np.rint(s.astype(np.float32)).astype(np.float16)
    assert np.array_equal(oracle.softmax_quant_p(si + np.float16(4.0), F16), oracle.softmax_quant_p(si, F16))


def _bf16_bits(f32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, nearest-even (input plumbing for the pins; values used here are exact in bf16
    or compared through torch's own conversion)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(f32, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_softmax_quant_special_cases_bf16():
    """The bf16 branch of the softmax + P quantization (Sec. 4: softmax stays in the 16-bit type, P gets the fixed
    step 1/127): probabilities are rounded to bf16 (8 significant bits) before the multiplication by 127."""
    import torch
    from scipy.special import softmax
    z = _bf16_bits(np.zeros((1, 8), np.float32))  # uniform row: p = 1/8 exactly (a power of two) -> round(15.875) = 16
    assert oracle.softmax_quant_p(z, BF16).tolist() == [[16] * 8]
    # uniform row of 3: p = 1/3 -> bf16(1/3) = 0.333984375 (0x3EAB) -> 42.416 -> 42; in fp16 1/3 -> 0.33325 -> 42.32 -> 42
    z = _bf16_bits(np.full((1, 3), 1.5, np.float32))
    assert oracle.softmax_quant_p(z, BF16).tolist() == [[42] * 3]
    # uniform row of 5: p = 0.2 -> bf16 0.2001953125 (0x3E4D) -> 25.4248 -> 25
    assert oracle.softmax_quant_p(_bf16_bits(np.zeros((1, 5), np.float32)), BF16).tolist() == [[25] * 5]
    # a case where bf16 rounding of p changes the code: two scores 0 and ln(3)-ish. Take scores (0, 1): p = (0.26894, 0.73106);
    # bf16: 0.26953125 (0x3E8A) -> 34.23 -> 34; 0.73046875 (0x3F3B) -> 92.77 -> 93; (fp16 gives 34.16 -> 34 and 92.84 -> 93)
    assert oracle.softmax_quant_p(_bf16_bits(np.array([[0.0, 1.0]], np.float32)), BF16).tolist() == [[34, 93]]
    d = np.full((1, 6), -20.0, np.float32)
    d[0, 2] = 20.0  # one dominant score
    assert oracle.softmax_quant_p(_bf16_bits(d), BF16).tolist() == [[0, 0, 127, 0, 0, 0]]
    # random rows against the textbook softmax (scipy, fp64) rounded to bf16 by torch, then round(127 p)
    rng = np.random.default_rng(43)
    sb = _bf16_bits((rng.standard_normal((32, 300)) * 3).astype(np.float32))
    s64 = oracle.f32_from_bits16(sb, BF16).astype(np.float64)
    p_bf = torch.from_numpy(softmax(s64, axis=-1)).to(torch.bfloat16).to(torch.float32).numpy()
    want = np.rint(p_bf * np.float32(127.0)).astype(np.int8)
    got = oracle.softmax_quant_p(sb, BF16)
    assert np.array_equal(got, want)
    # the two 16-bit types must really differ somewhere (a branch that ignored the dtype would pass the rows above
    # only by accident): same real scores, fp16 vs bf16 rounding of p
    s16 = s64.astype(np.float16)
    same_scores = np.array_equal(s16.astype(np.float64), s64)
    if same_scores:
        assert not np.array_equal(oracle.softmax_quant_p(s16, F16), got)
    # shift invariance with an exactly representable shift
    si = _bf16_bits(np.rint(s64).astype(np.float32))
    sj = _bf16_bits(np.rint(s64).astype(np.float32) + np.float32(4.0))
    assert np.array_equal(oracle.softmax_quant_p(si, BF16), oracle.softmax_quant_p(sj, BF16))


def test_softmax_quant_causal_pins():
    """Causal variant of the softmax + P quantization (Sec. 4 keeps the softmax in the 16-bit type; the mask itself is
    the usual rule of a decoder: query i sees the keys j <= i + (s_k - s_q)).  Pinned by closed forms, by the textbook
    softmax of the truncated rows, and by the unmasked function on scores that hold -inf where the mask hides a key."""
    from scipy.special import softmax
    # uniform scores, square: row i sees i + 1 keys with p = 1 / (i + 1) each
    pq = oracle.softmax_quant_p_causal(np.zeros((1, 6, 6), np.float16), F16)
    for i in range(6):
        p16 = np.float16(1.0 / (i + 1))
        code = int(np.rint(np.float32(p16) * np.float32(127.0)))
        assert pq[0, i].tolist() == [code] * (i + 1) + [0] * (5 - i)
    assert pq[0, 0, 0] == 127 and pq[0, 1, 0] == 64 and pq[0, 3, 0] == 32
    # four cached keys in front (s_k - s_q = 4): the first query sees five keys, the last one all of them
    pq = oracle.softmax_quant_p_causal(np.zeros((2, 3, 7), np.float16), F16)
    assert pq[1].tolist() == [[25] * 5 + [0] * 2, [21] * 6 + [0], [18] * 7]
    # a hidden key never matters, however large its score
    s = np.zeros((1, 4, 4), np.float16)
    s[0, 1, 3] = 30.0
    s[0, 2, 2] = 30.0  # visible to query 2: takes the whole row
    pq = oracle.softmax_quant_p_causal(s, F16)
    assert pq[0, 1].tolist() == [64, 64, 0, 0] and pq[0, 2].tolist() == [0, 0, 127, 0]
    # random scores, both 16-bit types: textbook softmax over the visible prefix of every row
    rng = np.random.default_rng(43)
    b, s_q, s_k = 3, 37, 53
    off = s_k - s_q
    s64 = np.rint(rng.standard_normal((b, s_q, s_k)) * 3 * 8) / 8  # exact in fp16 and in bf16
    for dtype in (F16, BF16):
        bits = s64.astype(np.float16) if dtype == F16 else _bf16_bits(s64.astype(np.float32)).reshape(s64.shape)
        got = oracle.softmax_quant_p_causal(bits, dtype)
        masked = s64.copy()
        for i in range(s_q):
            masked[:, i, i + off + 1:] = -np.inf
        p = softmax(masked, axis=-1)
        if dtype == F16:
            p16 = p.astype(np.float16).astype(np.float32)
        else:
            import torch
            p16 = torch.from_numpy(p).to(torch.bfloat16).to(torch.float32).numpy()
        want = np.rint(p16 * np.float32(127.0)).astype(np.int8)
        assert np.array_equal(got, want)
        for i in range(s_q):
            assert not got[:, i, i + off + 1:].any()
        # the unmasked function fed with -inf at the hidden positions agrees
        mb = masked.astype(np.float16) if dtype == F16 else _bf16_bits(masked.astype(np.float32)).reshape(masked.shape)
        assert np.array_equal(oracle.softmax_quant_p(mb, dtype), got)
    # the mask is bottom-right aligned: the last query's row equals the unmasked softmax of that row
    last = oracle.softmax_quant_p(s64[:, -1:, :].astype(np.float16), F16)
    assert np.array_equal(oracle.softmax_quant_p_causal(s64.astype(np.float16), F16)[:, -1:, :], last)


def test_ln_quantize_properties():
    rng = np.random.default_rng(51)
    t, c_i = 6, 512
    x = (rng.standard_normal((t, c_i)) * 3 + 1.5).astype(np.float16)
    ones, zeros = np.ones(c_i, np.float32), np.zeros(c_i, np.float32)
    q, sc = oracle.ln_quantize(x, F16, ones, zeros)
    deq = q.astype(np.float64) * sc.astype(np.float64)[:, None]
    assert np.all(np.abs(deq.mean(axis=1)) < 0.02)  # normalized rows: mean 0, variance 1 up to quant. noise
    assert np.all(np.abs(deq.var(axis=1) - 1.0) < 0.02)
    assert np.all(np.abs(q).max(axis=1) == 127)
    # alternating +-1 row: mean 0, variance 1 -> x_hat = +-gamma/sqrt(1 + eps) + beta, closed form
    alt = np.tile(np.array([1.0, -1.0], np.float16), c_i // 2)[None, :]
    g = np.full(c_i, 2.0, np.float32)
    b = np.full(c_i, 0.5, np.float32)
    q, sc = oracle.ln_quantize(alt, F16, g, b, eps=1e-5)
    hi = 2.0 / np.sqrt(1.0 + 1e-5) + 0.5
    lo = -2.0 / np.sqrt(1.0 + 1e-5) + 0.5
    assert np.isclose(sc[0] * 127.0, hi, rtol=1e-6)
    assert q[0, 0] == 127 and q[0, 1] == int(np.rint(lo / (hi / 127.0)))
    # folding 1/s into gamma and beta equals smoothing the LayerNorm output channel by channel
    inv_s = (rng.random(c_i) + 0.5).astype(np.float32)
    gamma = rng.standard_normal(c_i).astype(np.float32)
    beta = rng.standard_normal(c_i).astype(np.float32)
    q, sc = oracle.ln_quantize(x, F16, gamma * inv_s, beta * inv_s)
    x64 = x.astype(np.float64)
    ln = (x64 - x64.mean(1, keepdims=True)) / np.sqrt(x64.var(1, keepdims=True) + 1e-5) * gamma + beta
    xh = ln * inv_s
    err = np.abs(xh - q.astype(np.float64) * sc.astype(np.float64)[:, None])
    assert np.all(err <= sc.astype(np.float64)[:, None] * 0.5 * 1.01 + 1e-5)
