"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times.  Where the oracle cannot afford every output it computes a seeded sample of rows /
heads one by one, and integer checksums that cover every output (sum over tokens of the int32
accumulators equals (sum of activation codes) x weight codes, exactly)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import BF16, F16, bits_from_dev, dev, to_dev_16, ulp_distance

pytestmark = pytest.mark.gpu


def _progress(msg):
    print(f"[case] {msg}", flush=True)


def _smooth(case, alpha):
    ax = oracle.act_absmax_per_channel(case["x_calib"], F16)
    aw = oracle.weight_absmax_per_in_channel(case["w"], F16)
    return oracle.smooth_scales(ax, aw, alpha)


def _sample_rows(t, n, seed):
    rng = np.random.default_rng(seed)
    rows = set(rng.choice(t, size=min(n, t), replace=False).tolist())
    rows.update({0, t - 1, min(255, t - 1), min(256, t - 1)})  # tile borders
    return np.array(sorted(rows), dtype=np.int64)


def _column_checksum(xq, wq, chunk=4096):
    """sum_t acc[t, n] for every n, exactly (float64 holds these integers: < 2^53)."""
    xsum = xq.astype(np.float64).sum(axis=0)
    out = np.empty(wq.shape[0], np.float64)
    for n0 in range(0, wq.shape[0], chunk):
        out[n0:n0 + chunk] = wq[n0:n0 + chunk].astype(np.float64) @ xsum
    return out


def test_config1_opt125m_static_linear():
    _progress("config 1: 16x768x3072 static per-tensor, fp16")
    c = synth.linear_case(16, 768, 3072, 0.0, 60.0, synth.BASE_SEED + 1, n_out=6)
    s, inv_s = _smooth(c, 0.5)
    wq_ref, ws_ref = oracle.prepare_weight(c["w"], F16, s)
    _, calib = oracle.quantize_act(c["x_calib"], F16, oracle.PER_TENSOR_DYNAMIC, inv_s=inv_s)
    xq_ref, xs_ref = oracle.quantize_act(c["x"], F16, oracle.PER_TENSOR_STATIC, inv_s=inv_s, static_scale=calib[0])
    y_ref = oracle.w8a8_linear(xq_ref, xs_ref, wq_ref, ws_ref, F16)
    wq, ws = sq.prepare_weight(to_dev_16(c["w"], F16), dev(s))
    _, calib_g = sq.quantize_act(to_dev_16(c["x_calib"], F16), sq.PER_TENSOR_DYNAMIC, inv_s=dev(inv_s))
    xq, xs = sq.quantize_act(to_dev_16(c["x"], F16), sq.PER_TENSOR_STATIC, inv_s=dev(inv_s), static_scale=calib_g)
    y = sq.w8a8_linear(xq, xs, wq, ws, torch.float16)
    assert calib_g.item() == calib[0]
    assert np.array_equal(wq.cpu().numpy(), wq_ref) and np.array_equal(xq.cpu().numpy(), xq_ref)
    assert ulp_distance(bits_from_dev(y), y_ref).max() <= 1


def test_config2_opt13b_ffn_pair():
    _progress("config 2: FFN pair 512 x 5120 -> 20480 (ReLU) -> 5120, per-token dynamic, fp16")
    t, h, f = 512, 5120, 20480
    c = synth.linear_case(t, h, f, 0.01, 40.0, synth.BASE_SEED + 2)
    s, inv_s = _smooth(c, 0.5)
    w2 = synth.weights(f, h, synth.BASE_SEED + 22)
    # FC1 (smoothed input), ReLU fused
    wq1_ref, ws1_ref = oracle.prepare_weight(c["w"], F16, s)
    wq1, ws1 = sq.prepare_weight(to_dev_16(c["w"], F16), dev(s))
    assert np.array_equal(wq1.cpu().numpy(), wq1_ref) and ws1.item() == ws1_ref[0]
    xq_ref, xs_ref = oracle.quantize_act(c["x"], F16, oracle.PER_TOKEN_DYNAMIC, inv_s=inv_s)
    xq, xs = sq.quantize_act(to_dev_16(c["x"], F16), sq.PER_TOKEN_DYNAMIC, inv_s=dev(inv_s))
    assert np.array_equal(xq.cpu().numpy(), xq_ref) and np.array_equal(xs.cpu().numpy(), xs_ref)
    y1 = sq.w8a8_linear(xq, xs, wq1, ws1, torch.float16, relu=True)
    y1_ref = oracle.w8a8_linear(xq_ref, xs_ref, wq1_ref, ws1_ref, F16, relu=True)
    d = ulp_distance(bits_from_dev(y1), y1_ref)
    assert d.max() <= 1 and (d == 0).mean() > 0.999
    acc = sq.i8_gemm_i32(xq, wq1).cpu().numpy()
    assert np.array_equal(acc, oracle.i8_gemm_i32(xq_ref, wq1_ref))
    # FC2 on the real ReLU output (s = 1)
    wq2_ref, ws2_ref = oracle.prepare_weight(w2, F16, None)
    wq2, ws2 = sq.prepare_weight(to_dev_16(w2, F16), None)
    assert np.array_equal(wq2.cpu().numpy(), wq2_ref)
    y1_bits = bits_from_dev(y1)
    xq2_ref, xs2_ref = oracle.quantize_act(y1_bits, F16, oracle.PER_TOKEN_DYNAMIC)
    xq2, xs2 = sq.quantize_act(y1, sq.PER_TOKEN_DYNAMIC)
    assert np.array_equal(xq2.cpu().numpy(), xq2_ref) and np.array_equal(xs2.cpu().numpy(), xs2_ref)
    assert xq2_ref.min() >= 0  # ReLU output: the codes use only the non-negative half
    y2 = sq.w8a8_linear(xq2, xs2, wq2, ws2, torch.float16)
    y2_ref = oracle.w8a8_linear(xq2_ref, xs2_ref, wq2_ref, ws2_ref, F16)
    d = ulp_distance(bits_from_dev(y2), y2_ref)
    assert d.max() <= 1 and (d == 0).mean() > 0.999


OPT175B = [(l.name, l.c_i, l.c_o) for l in synth.OPT175B_LINEARS]


@pytest.mark.parametrize("name,c_i,c_o", OPT175B)
def test_config3_opt175b_linears(name, c_i, c_o):
    """All token counts of the configuration for one layer shape; bf16 out, per-token dynamic."""
    _progress(f"config 3: {name} {c_i} -> {c_o}: generating inputs")
    idx = [n for n, _, _ in OPT175B].index(name)
    smoothed = name in ("qkv", "fc1")
    n_out = synth.n_outlier_channels(c_i, 0.005)
    ch = synth.outlier_channels(c_i, n_out, synth.BASE_SEED + 30 + idx)
    w = synth.weights(c_i, c_o, synth.BASE_SEED + 40 + idx)
    s = inv_s = None
    if smoothed:
        xc = synth.activations(512, c_i, ch, 80.0, synth.BASE_SEED + 50 + idx)
        s, inv_s = oracle.smooth_scales(oracle.act_absmax_per_channel(xc, F16), oracle.weight_absmax_per_in_channel(w, F16), 0.5)
    _progress(f"config 3: {name}: weight preparation (oracle + GPU)")
    wq_ref, ws_ref = oracle.prepare_weight(w, F16, s)
    wd = to_dev_16(w, F16)
    if smoothed:
        assert np.array_equal(sq.weight_absmax_per_in_channel(wd).cpu().numpy(), oracle.weight_absmax_per_in_channel(w, F16))
    wq, ws = sq.prepare_weight(wd, None if s is None else dev(s))
    del wd, w
    assert ws.item() == ws_ref[0]
    assert torch.equal(wq.cpu(), torch.from_numpy(wq_ref)), "weight codes differ"
    inv_s_d = None if inv_s is None else dev(inv_s)
    for m in synth.OPT175B_TOKENS:
        _progress(f"config 3: {name} M={m}")
        x = synth.activations(m, c_i, ch, 80.0, synth.BASE_SEED + 60 + idx + m)
        xq_ref, xs_ref = oracle.quantize_act(x, F16, oracle.PER_TOKEN_DYNAMIC, inv_s=inv_s)
        xq, xs = sq.quantize_act(to_dev_16(x, F16), sq.PER_TOKEN_DYNAMIC, inv_s=inv_s_d)
        assert np.array_equal(xq.cpu().numpy(), xq_ref) and np.array_equal(xs.cpu().numpy(), xs_ref)
        y = sq.w8a8_linear(xq, xs, wq, ws, torch.bfloat16)
        rows = _sample_rows(m, 40 if m > 128 else m, 70 + idx + m)
        y_ref = oracle.w8a8_linear(xq_ref, xs_ref, wq_ref, ws_ref, BF16, rows=rows)
        d = ulp_distance(bits_from_dev(y[torch.from_numpy(rows).cuda()]), y_ref[rows])
        assert d.max() <= 1 and (d == 0).mean() > 0.999, f"M={m}: max ulp {d.max()}"
        # every accumulator is covered by the exact column checksum
        acc = sq.i8_gemm_i32(xq, wq)
        got = acc.sum(dim=0, dtype=torch.int64).cpu().numpy().astype(np.float64)
        assert np.array_equal(got, _column_checksum(xq_ref, wq_ref)), f"M={m}: column checksum differs"
        del acc, y


def test_config4_int8_attention_bmms():
    """batch 8 x 96 heads, seq 2048, head_dim 128 at full size on the GPU; the oracle checks sampled heads."""
    bh, s_len, d = 8 * 96, 2048, 128
    _progress("config 4: generating Q, K, V")
    qkv = [synth.normal_fp16((bh * s_len, d), synth.BASE_SEED + 80 + i) for i in range(3)]
    heads = [0, 377, bh - 1]
    codes, steps = [], []
    for i, x in enumerate(qkv):
        delta = np.float32(np.abs(x).max().astype(np.float32) / np.float32(127.0))  # calibrated per-tensor step
        xq, _ = sq.quantize_act(to_dev_16(x, F16), sq.PER_TENSOR_STATIC, static_scale=dev(np.array([delta], np.float32)))
        xq = xq.view(bh, s_len, d)
        for h in heads:
            ref, _ = oracle.quantize_act(x[h * s_len:(h + 1) * s_len], F16, oracle.PER_TENSOR_STATIC, static_scale=delta)
            assert np.array_equal(xq[h].cpu().numpy(), ref)
        codes.append(xq)
        steps.append(delta)
    del qkv
    _progress("config 4: BMM1 Q K^T")
    alpha1 = float(np.float32(steps[0] * steps[1]) / np.float32(np.sqrt(np.float32(d))))
    sc = sq.w8a8_bmm(codes[0], codes[1], True, alpha1, torch.float16)
    for h in heads:
        ref = oracle.w8a8_bmm(codes[0][h:h + 1].cpu().numpy(), codes[1][h:h + 1].cpu().numpy(), True, alpha1, F16)
        assert ulp_distance(bits_from_dev(sc[h]), ref[0]).max() <= 1, f"head {h}"
    _progress("config 4: softmax + P quantization")
    pq = sq.softmax_quant_p(sc)
    for h in heads:
        ref = oracle.softmax_quant_p(bits_from_dev(sc[h]), F16).astype(np.int32)
        diff = np.abs(pq[h].cpu().numpy().astype(np.int32) - ref)
        assert diff.max() <= 1 and (diff != 0).mean() <= 1e-3, f"head {h}"
    del sc
    _progress("config 4: BMM2 P V")
    alpha2 = float(np.float32(steps[2]) / np.float32(127.0))
    o = sq.w8a8_bmm(pq, codes[2], False, alpha2, torch.float16)
    for h in heads:
        ref = oracle.w8a8_bmm(pq[h:h + 1].cpu().numpy(), codes[2][h:h + 1].cpu().numpy(), False, alpha2, F16)
        assert ulp_distance(bits_from_dev(o[h]), ref[0]).max() <= 1, f"head {h}"
    assert bool(torch.isfinite(o.float()).all())
