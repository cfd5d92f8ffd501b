"""GPU parity at the full sizes of the benchmark configurations.  The OPT-175B linears (configuration 3, the
workload bench.py times) run in both operand layouts: TILED is the launch configuration bench.py times (weights
prepared TILED on the GPU, activations quantized TILED, the TILED instantiations of the GEMM kernels), ROW_MAJOR
the default of the C ABI.  Where the oracle cannot afford every output it computes a seeded sample of rows /
heads one by one, and integer checksums that cover every output (sum over tokens of the int32
accumulators equals (sum of activation codes) x weight codes, exactly)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import BF16, F16, assert_identical_16, bits_from_dev, dev, tiled_to_rows, to_dev_16, ulp_distance

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
    assert_identical_16(d)
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
    assert_identical_16(d)


OPT175B = [(l.name, l.c_i, l.c_o) for l in synth.OPT175B_LINEARS]


@pytest.mark.parametrize("layout", [sq.TILED, sq.ROW_MAJOR], ids=["tiled", "rows"])
@pytest.mark.parametrize("name,c_i,c_o", OPT175B)
def test_config3_opt175b_linears(name, c_i, c_o, layout):
    """All token counts of the configuration for one layer shape; bf16 out, per-token dynamic.  In the TILED layout the
    GPU's code tensors are brought back to row order (index plumbing only) before they are compared with the oracle's."""
    _progress(f"config 3: {name} {c_i} -> {c_o} layout={layout}: generating inputs")
    codes_of = tiled_to_rows if layout == sq.TILED else (lambda tns: tns.cpu().numpy())
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
    wq, ws = sq.prepare_weight(wd, None if s is None else dev(s), layout=layout)
    del wd, w
    assert ws.item() == ws_ref[0]
    assert np.array_equal(codes_of(wq), wq_ref), "weight codes differ"
    inv_s_d = None if inv_s is None else dev(inv_s)
    for m in synth.OPT175B_TOKENS:
        _progress(f"config 3: {name} M={m}")
        x = synth.activations(m, c_i, ch, 80.0, synth.BASE_SEED + 60 + idx + m)
        xq_ref, xs_ref = oracle.quantize_act(x, F16, oracle.PER_TOKEN_DYNAMIC, inv_s=inv_s)
        xq, xs = sq.quantize_act(to_dev_16(x, F16), sq.PER_TOKEN_DYNAMIC, inv_s=inv_s_d, layout=layout)
        assert np.array_equal(codes_of(xq), xq_ref) and np.array_equal(xs.cpu().numpy(), xs_ref)
        y = sq.w8a8_linear(xq, xs, wq, ws, torch.bfloat16, layout=layout)
        rows = _sample_rows(m, 40 if m > 128 else m, 70 + idx + m)
        y_ref = oracle.w8a8_linear(xq_ref, xs_ref, wq_ref, ws_ref, BF16, rows=rows)
        d = ulp_distance(bits_from_dev(y[torch.from_numpy(rows).cuda()]), y_ref[rows])
        assert_identical_16(d)
        # every accumulator is covered by the exact column checksum
        acc = sq.i8_gemm_i32(xq, wq, layout=layout)
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
    _progress("config 4: the same attention in the fused kernel")
    pq_f = torch.full_like(pq, -128)
    o_f = sq.w8a8_attention(codes[0], codes[1], codes[2], alpha1, alpha2, torch.float16, p_codes=pq_f)
    for h in heads:
        sc_ref = oracle.w8a8_bmm(codes[0][h:h + 1].cpu().numpy(), codes[1][h:h + 1].cpu().numpy(), True, alpha1, F16)
        ref = oracle.softmax_quant_p(sc_ref[0], F16).astype(np.int32)
        got = pq_f[h].cpu().numpy().astype(np.int32)
        diff = np.abs(got - ref)
        assert got.min() >= 0 and diff.max() <= 1 and (diff != 0).mean() <= 1e-3, f"fused: codes of head {h}"
        o_ref = oracle.w8a8_bmm(pq_f[h:h + 1].cpu().numpy(), codes[2][h:h + 1].cpu().numpy(), False, alpha2, F16)
        assert_identical_16(ulp_distance(bits_from_dev(o_f[h]), o_ref[0]), f"fused: output of head {h}")
    # against the unfused library chain over all 768 heads: same scores, row sums in another order
    d_all = (pq_f.view(torch.int8).to(torch.int16) - pq.to(torch.int16)).abs()
    assert int(d_all.max()) <= 1 and float((d_all != 0).float().mean()) <= 1e-3
    del d_all
    assert int(pq_f.min()) >= 0  # every code was written
    _progress("config 4: the fused kernel with the causal mask")
    pq_f.fill_(-128)
    o_c = sq.w8a8_attention(codes[0], codes[1], codes[2], alpha1, alpha2, torch.float16, p_codes=pq_f, causal=True)
    for h in heads:
        sc_ref = oracle.w8a8_bmm(codes[0][h:h + 1].cpu().numpy(), codes[1][h:h + 1].cpu().numpy(), True, alpha1, F16)
        ref = oracle.softmax_quant_p_causal(sc_ref, F16)[0].astype(np.int32)
        got = pq_f[h].cpu().numpy().astype(np.int32)
        diff = np.abs(got - ref)
        assert got.min() >= 0 and diff.max() <= 1 and (diff != 0).mean() <= 1e-3, f"causal: codes of head {h}"
        assert not np.triu(got, 1).any(), f"causal: a hidden key of head {h} got a probability"
        o_ref = oracle.w8a8_bmm(pq_f[h:h + 1].cpu().numpy(), codes[2][h:h + 1].cpu().numpy(), False, alpha2, F16)
        assert_identical_16(ulp_distance(bits_from_dev(o_c[h]), o_ref[0]), f"causal: output of head {h}")
    assert int(pq_f.min()) >= 0 and not bool(pq_f.triu(1).any())  # all heads: every code written, nothing above the diagonal


def test_config5_opt66b_decoder_layer_chain():
    """OPT-66B-shaped decoder layer, batch 4 x sequence 1024 (hidden 9216, FFN 36864, 72 heads), alpha 0.8,
    1% outlier channels x60: LayerNorm with the smoothing factors folded into gamma / beta + per-token
    quantization -> QKV GEMM -> INT8 attention (Q K^T, softmax + P quantization, P V) -> out-proj + residual
    -> LayerNorm + quantization -> FC1 + ReLU -> FC2 + residual.  Every stage runs on the GPU on the previous
    stage's GPU output; each stage is checked against the oracle fed with that same input, on sampled rows /
    heads (exact gates for the GEMMs and quantizers, the +-1 code gate for LayerNorm and softmax).  Head
    splitting / merging between the stages is a torch permute (layout plumbing, no arithmetic)."""
    hid, ffn, n_head, bsz, seq, alpha = 9216, 36864, 72, 4, 1024, 0.8
    d_head, t = hid // n_head, bsz * seq
    g = torch.Generator(device="cuda")
    g.manual_seed(synth.BASE_SEED + 500)

    def dev_weight(c_i, c_o):
        w = torch.empty((c_i, c_o), device="cuda", dtype=torch.float16)
        for r0 in range(0, c_i, 2048):
            w[r0:r0 + 2048] = (torch.randn((min(2048, c_i - r0), c_o), generator=g, device="cuda") * 0.02).to(torch.float16)
        return w

    def ln_params(seed):
        ch = synth.outlier_channels(hid, synth.n_outlier_channels(hid, 0.01), seed)
        gamma = np.ones(hid, np.float32)
        gamma[ch] = 60.0  # the LayerNorm output (what the paper smooths) gets its outlier channels from gamma
        beta = (np.random.default_rng(seed + 1).standard_normal(hid) * 0.1).astype(np.float32)
        return gamma, beta

    def smoothed_layer(x16, gamma, beta, w):
        """Offline part for a LayerNorm -> linear pair: calibrate on 512 tokens, Eq. 4, fold into gamma / beta."""
        xc = torch.nn.functional.layer_norm(x16[:512].float(), (hid,), torch.from_numpy(gamma).cuda(),
                                            torch.from_numpy(beta).cuda(), 1e-5).to(torch.float16)
        s, inv_s = sq.smooth_scales(sq.act_absmax_per_channel(xc).cpu(), sq.weight_absmax_per_in_channel(w).cpu(), alpha)
        wq, ws = sq.prepare_weight(w, s.cuda())
        inv = inv_s.numpy()
        return wq, ws, (gamma * inv).astype(np.float32), (beta * inv).astype(np.float32)

    def check_linear(name, xq, xs, wq, ws, y, bias, res, relu, seed):
        rows = _sample_rows(t, 6, seed)
        ref = oracle.w8a8_linear(xq.cpu().numpy(), xs.cpu().numpy(), wq.cpu().numpy(), ws.cpu().numpy(), F16,
                                 bias=bias, residual_bits=None if res is None else bits_from_dev(res), relu=relu, rows=rows)
        dd = ulp_distance(bits_from_dev(y[torch.from_numpy(rows).cuda()]), ref[rows])
        assert_identical_16(dd)

    def check_ln(name, x16, gamma_f, beta_f, xq, xs, seed):
        rows = _sample_rows(t, 8, seed)
        q_ref, s_ref = oracle.ln_quantize(bits_from_dev(x16[torch.from_numpy(rows).cuda()]), F16, gamma_f, beta_f)
        q = xq[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.int32)
        assert np.abs(q - q_ref.astype(np.int32)).max() <= 1 and (q != q_ref).mean() <= 1e-3, name
        assert np.allclose(xs[torch.from_numpy(rows).cuda()].cpu().numpy(), s_ref, rtol=1e-5), name

    def check_quant(name, x16, xq, xs, seed):
        rows = _sample_rows(t, 8, seed)
        q_ref, s_ref = oracle.quantize_act(bits_from_dev(x16[torch.from_numpy(rows).cuda()]), F16, oracle.PER_TOKEN_DYNAMIC)
        assert np.array_equal(xq[torch.from_numpy(rows).cuda()].cpu().numpy(), q_ref), name
        assert np.array_equal(xs[torch.from_numpy(rows).cuda()].cpu().numpy(), s_ref), name

    _progress("config 5: inputs and offline preparation")
    x = torch.randn((t, hid), generator=g, device="cuda").to(torch.float16)
    gamma1, beta1 = ln_params(synth.BASE_SEED + 510)
    w = dev_weight(hid, 3 * hid)
    wq_qkv, ws_qkv, g1f, b1f = smoothed_layer(x, gamma1, beta1, w)
    w = dev_weight(hid, hid)
    wq_o, ws_o = sq.prepare_weight(w, None)
    del w
    bias_qkv, bias_o = synth.bias(3 * hid, 520), synth.bias(hid, 521)
    bias_1, bias_2 = synth.bias(ffn, 522), synth.bias(hid, 523)

    _progress("config 5: LayerNorm 1 + quantize")
    xq, xs = sq.ln_quantize(x, dev(g1f), dev(b1f))
    check_ln("ln1", x, g1f, b1f, xq, xs, 530)
    _progress("config 5: QKV projection")
    qkv = sq.w8a8_linear(xq, xs, wq_qkv, ws_qkv, torch.float16, bias=dev(bias_qkv))
    check_linear("qkv", xq, xs, wq_qkv, ws_qkv, qkv, bias_qkv, None, False, 531)
    del wq_qkv

    _progress("config 5: per-tensor quantization of Q, K, V and head split")
    codes, steps = [], []
    for i in range(3):
        part = qkv[:, i * hid:(i + 1) * hid]  # [t, hid] view with row stride 3*hid
        cq, cs = sq.quantize_act(part, sq.PER_TENSOR_DYNAMIC)
        rows = _sample_rows(t, 4, 540 + i)
        ref, _ = oracle.quantize_act(bits_from_dev(part[torch.from_numpy(rows).cuda()].contiguous()), F16,
                                     oracle.PER_TENSOR_STATIC, static_scale=np.float32(cs.item()))
        assert np.array_equal(cq[torch.from_numpy(rows).cuda()].cpu().numpy(), ref), f"qkv part {i}"
        codes.append(cq.view(bsz, seq, n_head, d_head).permute(0, 2, 1, 3).contiguous().view(bsz * n_head, seq, d_head))
        steps.append(np.float32(cs.item()))
    del qkv
    heads = [0, 131, bsz * n_head - 1]
    _progress("config 5: attention")
    alpha1 = float(np.float32(steps[0] * steps[1]) / np.float32(np.sqrt(np.float32(d_head))))
    sc = sq.w8a8_bmm(codes[0], codes[1], True, alpha1, torch.float16)
    for h in heads:
        ref = oracle.w8a8_bmm(codes[0][h:h + 1].cpu().numpy(), codes[1][h:h + 1].cpu().numpy(), True, alpha1, F16)
        assert ulp_distance(bits_from_dev(sc[h]), ref[0]).max() <= 1, f"scores head {h}"
    pq = sq.softmax_quant_p(sc)
    for h in heads:
        ref = oracle.softmax_quant_p(bits_from_dev(sc[h]), F16).astype(np.int32)
        diff = np.abs(pq[h].cpu().numpy().astype(np.int32) - ref)
        assert diff.max() <= 1 and (diff != 0).mean() <= 1e-3, f"P head {h}"
    del sc
    alpha2 = float(np.float32(steps[2]) / np.float32(127.0))
    o = sq.w8a8_bmm(pq, codes[2], False, alpha2, torch.float16)
    for h in heads:
        ref = oracle.w8a8_bmm(pq[h:h + 1].cpu().numpy(), codes[2][h:h + 1].cpu().numpy(), False, alpha2, F16)
        assert ulp_distance(bits_from_dev(o[h]), ref[0]).max() <= 1, f"O head {h}"
    del pq, codes
    attn = o.view(bsz, n_head, seq, d_head).permute(0, 2, 1, 3).contiguous().view(t, hid)
    del o

    _progress("config 5: out-proj + residual")
    aq, as_ = sq.quantize_act(attn, sq.PER_TOKEN_DYNAMIC)
    check_quant("attn quant", attn, aq, as_, 550)
    h1 = sq.w8a8_linear(aq, as_, wq_o, ws_o, torch.float16, bias=dev(bias_o), residual=x)
    check_linear("out_proj", aq, as_, wq_o, ws_o, h1, bias_o, x, False, 551)
    del attn, aq, wq_o

    _progress("config 5: LayerNorm 2 + FC1 + ReLU")
    gamma2, beta2 = ln_params(synth.BASE_SEED + 560)
    w = dev_weight(hid, ffn)
    wq_1, ws_1, g2f, b2f = smoothed_layer(h1, gamma2, beta2, w)
    del w
    hq, hs = sq.ln_quantize(h1, dev(g2f), dev(b2f))
    check_ln("ln2", h1, g2f, b2f, hq, hs, 561)
    f1 = sq.w8a8_linear(hq, hs, wq_1, ws_1, torch.float16, bias=dev(bias_1), relu=True)
    check_linear("fc1", hq, hs, wq_1, ws_1, f1, bias_1, None, True, 562)
    del wq_1, hq

    _progress("config 5: FC2 + residual")
    w = dev_weight(ffn, hid)
    wq_2, ws_2 = sq.prepare_weight(w, None)
    del w
    fq, fs = sq.quantize_act(f1, sq.PER_TOKEN_DYNAMIC)
    check_quant("fc1 out quant", f1, fq, fs, 570)
    assert int(fq.min().item()) >= 0  # ReLU output: only the non-negative half of the code range
    out = sq.w8a8_linear(fq, fs, wq_2, ws_2, torch.float16, bias=dev(bias_2), residual=h1)
    check_linear("fc2", fq, fs, wq_2, ws_2, out, bias_2, h1, False, 571)
    assert bool(torch.isfinite(out.float()).all())
