#!/usr/bin/env python3
"""Benchmark of the SmoothQuant W8A8 hot path on one MI355X.

Workload (N=1): the four OPT-175B-shaped linears at hidden 12288 (QKV 12288->36864, out-proj
12288->12288, FC1 12288->49152, FC2 49152->12288) at M = 2048 tokens, per-token dynamic activation
quantization, per-tensor weights, bf16 output.  One step = for each of the four layers:
quantize_act (fp16 activation -> int8 codes + per-token steps) then w8a8_linear (INT8 MFMA GEMM with
the dequantizing epilogue fused); int8 operands use the library's tiled layout.  Inputs (activations,
prepared int8 weights) are resident in HBM
before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0  # MI355X dense INT8 MFMA peak, 5.0 POP/s
PEAK_HBM_GBS = 8000.0


def make_layer(sq, torch, name, t, c_i, c_o, outlier_frac, factor, alpha, smoothed, seed):
    """Synthetic layer with the paper's outlier structure, prepared offline with the library itself."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.randn((t, c_i), generator=g, device="cuda", dtype=torch.float32)
    n_out = int(round(outlier_frac * c_i))
    ch = torch.randperm(c_i, generator=g, device="cuda")[:n_out]
    x[:, ch] *= factor
    x = x.to(torch.float16)
    w = torch.empty((c_i, c_o), device="cuda", dtype=torch.float16)
    rows = 2048
    for r0 in range(0, c_i, rows):  # chunked to bound the fp32 temporary
        w[r0:r0 + rows] = (torch.randn((min(rows, c_i - r0), c_o), generator=g, device="cuda") * 0.02).to(torch.float16)
    inv_s_dev = None
    s_dev = None
    if smoothed:
        xc = torch.randn((512, c_i), generator=g, device="cuda", dtype=torch.float32)
        xc[:, ch] *= factor
        ax = sq.act_absmax_per_channel(xc.to(torch.float16))
        aw = sq.weight_absmax_per_in_channel(w)
        s, inv_s = sq.smooth_scales(ax.cpu(), aw.cpu(), alpha)
        s_dev, inv_s_dev = s.cuda(), inv_s.cuda()
    wq, w_scale = sq.prepare_weight(w, s_dev, layout=sq.TILED)
    del w
    xq = sq.empty_codes(t, c_i, sq.TILED)
    x_scale = torch.empty(t, dtype=torch.float32, device="cuda")
    y = torch.empty((t, c_o), dtype=torch.bfloat16, device="cuda")
    nws = sq.workspace_bytes(sq.OP_W8A8_LINEAR, t, c_i, c_o)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    return dict(name=name, t=t, c_i=c_i, c_o=c_o, x=x, inv_s=inv_s_dev, wq=wq, w_scale=w_scale, xq=xq, x_scale=x_scale,
                y=y, ws=ws, ops=2.0 * t * c_i * c_o)


def run_layer(sq, torch, L):
    sq.quantize_act(L["x"], sq.PER_TOKEN_DYNAMIC, inv_s=L["inv_s"], out=(L["xq"], L["x_scale"]), layout=sq.TILED)
    sq.w8a8_linear(L["xq"], L["x_scale"], L["wq"], L["w_scale"], torch.bfloat16, out=L["y"], workspace=L["ws"], layout=sq.TILED)


def _time_us(torch, fn, iters=10, warm=2):
    for _ in range(warm):
        fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters * 1e3


def other_configs(sq, torch):
    """Latency and roofline fraction of the other benchmark configurations (synthetic inputs of their shapes):
    1 = OPT-125m-shaped static linear, 2 = OPT-13B-shaped FFN pair, 4 = INT8 attention BMMs (batch 8 x 96 heads,
    sequence 2048, head_dim 128), 5 = the linears and attention of an OPT-66B-shaped decoder layer (4 x 1024 tokens)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    out = {}

    def rand16(shape, scale=1.0):
        return (torch.randn(shape, generator=g, device="cuda") * scale).to(torch.float16)

    def linear_pair(t, c_i, c_o, relu=False, static=False):
        x = rand16((t, c_i))
        wq, ws = sq.prepare_weight(rand16((c_i, c_o), 0.02), None, layout=sq.TILED)
        xq = sq.empty_codes(t, c_i, sq.TILED)
        xs = torch.empty(1 if static else t, dtype=torch.float32, device="cuda")
        if static:
            xs.fill_(float(x.abs().max()) / 127.0)
        y = torch.empty((t, c_o), dtype=torch.float16, device="cuda")
        wsp = torch.empty(max(sq.workspace_bytes(sq.OP_W8A8_LINEAR, t, c_i, c_o), 16), dtype=torch.uint8, device="cuda")
        mode = sq.PER_TENSOR_STATIC if static else sq.PER_TOKEN_DYNAMIC
        q_us = _time_us(torch, lambda: sq.quantize_act(x, mode, static_scale=xs if static else None, out=(xq, xs), layout=sq.TILED))
        g_us = _time_us(torch, lambda: sq.w8a8_linear(xq, xs, wq, ws, torch.float16, relu=relu, out=y, workspace=wsp, layout=sq.TILED))
        ops = 2.0 * t * c_i * c_o
        return {"quantize_us": round(q_us, 1), "gemm_us": round(g_us, 1), "tops": round(ops / (q_us + g_us) / 1e6, 1),
                "frac_mfma_peak": round(ops / (q_us + g_us) / 1e6 / PEAK_INT8_TOPS, 4)}

    out["config1_opt125m_static_16x768x3072"] = linear_pair(16, 768, 3072, static=True)
    out["config2_opt13b_fc1_512x5120x20480_relu"] = linear_pair(512, 5120, 20480, relu=True)
    out["config2_opt13b_fc2_512x20480x5120"] = linear_pair(512, 20480, 5120)

    def attention(bh, s_len, d):
        q, k, v = (torch.randint(-127, 128, (bh, s_len, d), dtype=torch.int8, device="cuda", generator=g) for _ in range(3))
        sc = torch.empty((bh, s_len, s_len), dtype=torch.float16, device="cuda")
        pq = torch.empty((bh, s_len, s_len), dtype=torch.int8, device="cuda")
        o = torch.empty((bh, s_len, d), dtype=torch.float16, device="cuda")
        # (the first launches after the multi-GB allocations run slower than the steady state: warm up longer)
        t1 = _time_us(torch, lambda: sq.w8a8_bmm(q, k, True, 2e-5, torch.float16, out=sc), iters=10, warm=5)
        t2 = _time_us(torch, lambda: sq.softmax_quant_p(sc, out=pq), iters=8, warm=2)
        t3 = _time_us(torch, lambda: sq.w8a8_bmm(pq, v, False, 1e-4, torch.float16, out=o), iters=8, warm=2)
        b1 = 2.0 * bh * s_len * d + 2.0 * bh * s_len * s_len
        b2 = 3.0 * bh * s_len * s_len
        b3 = bh * s_len * s_len + 3.0 * bh * s_len * d
        return {"bmm1_us": round(t1, 1), "bmm1_frac_hbm": round(b1 / t1 / 1e3 / PEAK_HBM_GBS, 4),
                "softmax_quant_us": round(t2, 1), "softmax_frac_hbm": round(b2 / t2 / 1e3 / PEAK_HBM_GBS, 4),
                "bmm2_us": round(t3, 1), "bmm2_frac_hbm": round(b3 / t3 / 1e3 / PEAK_HBM_GBS, 4),
                "tops_both_bmms": round(4.0 * bh * s_len * s_len * d / (t1 + t3) / 1e6, 1)}

    out["config4_attention_768x2048x128"] = attention(768, 2048, 128)
    out["config5_opt66b_qkv_4096x9216x27648"] = linear_pair(4096, 9216, 27648)
    out["config5_opt66b_out_proj_4096x9216x9216"] = linear_pair(4096, 9216, 9216)
    out["config5_opt66b_fc1_4096x9216x36864_relu"] = linear_pair(4096, 9216, 36864, relu=True)
    out["config5_opt66b_fc2_4096x36864x9216"] = linear_pair(4096, 36864, 9216)
    out["config5_attention_288x1024x128"] = attention(288, 1024, 128)
    x = rand16((4096, 9216))
    gamma = torch.ones(9216, device="cuda")
    beta = torch.zeros(9216, device="cuda")
    xq = sq.empty_codes(4096, 9216, sq.TILED)
    xs = torch.empty(4096, dtype=torch.float32, device="cuda")
    ln_us = _time_us(torch, lambda: sq.ln_quantize(x, gamma, beta, out=(xq, xs), layout=sq.TILED))
    out["config5_ln_quantize_4096x9216"] = {"us": round(ln_us, 1),
                                            "frac_hbm": round(3.0 * 4096 * 9216 / ln_us / 1e3 / PEAK_HBM_GBS, 4)}
    return out


def cpu_baseline(layers_desc):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload:
    every layer at the full 2048 tokens (quantize + linear with epilogue), about 10-20 s of CPU work."""
    import numpy as np
    import oracle
    from paper_2211_10438_amd import synth
    rows = 2048
    ops = 0.0
    secs = 0.0
    for i, (name, c_i, c_o) in enumerate(layers_desc):
        ch = synth.outlier_channels(c_i, synth.n_outlier_channels(c_i, 0.005), 100 + i)
        x = synth.activations(rows, c_i, ch, 80.0, 200 + i)
        wq = synth.int8_codes((c_o, c_i), 300 + i, -40, 40)  # stand-in codes: the timing does not depend on values
        ws = np.array([0.001], np.float32)
        t0 = time.perf_counter()
        xq, xs = oracle.quantize_act(x, oracle.F16, oracle.PER_TOKEN_DYNAMIC)
        oracle.w8a8_linear(xq, xs, wq, ws, oracle.BF16)
        secs += time.perf_counter() - t0
        ops += 2.0 * rows * c_i * c_o
    return dict(value=ops / secs / 1e12, unit="TOPS", cores=oracle.num_threads(), kind="oracle",
                sample=f"{rows} of 2048 tokens per layer, all four layers, quantize + int32 GEMM + epilogue; {secs:.1f} s")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--probe", action="store_true",
                    help="counter probe for rocprofv3 --pmc: a 512 MiB device copy (known size), two steps of the "
                         "workload and two decode steps at 1 / 16 / 128 tokens, nothing timed, no JSON")
    ap.add_argument("--probe-attention", action="store_true",
                    help="counter probe for rocprofv3 --pmc: a 512 MiB device copy, then the INT8 attention chain "
                         "(scores, softmax + P quantization, P V) at 768 heads x 2048 x 128 twice, nothing timed, no JSON")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one MI355X per box); --gpus must be 1. "
              "Sharding over more GPUs is not built.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2211_10438_amd import binding as sq
    from paper_2211_10438_amd import synth

    sq.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.probe_attention:
        bh, s_len, d = 768, 2048, 128
        g = torch.Generator(device="cuda")
        g.manual_seed(78)
        q, k, v = (torch.randint(-127, 128, (bh, s_len, d), dtype=torch.int8, device="cuda", generator=g) for _ in range(3))
        sc = torch.empty((bh, s_len, s_len), dtype=torch.float16, device="cuda")
        pq = torch.empty((bh, s_len, s_len), dtype=torch.int8, device="cuda")
        o = torch.empty((bh, s_len, d), dtype=torch.float16, device="cuda")
        src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
            sq.w8a8_bmm(q, k, True, 2e-5, torch.float16, out=sc)
            sq.softmax_quant_p(sc, out=pq)
            sq.w8a8_bmm(pq, v, False, 1e-4, torch.float16, out=o)
        torch.cuda.synchronize()
        print("probe done: copy of %d bytes + 2 attention chains at %d heads x %d x %d" % (src.numel(), bh, s_len, d))
        return
    t = args.tokens
    desc = [(l.name, l.c_i, l.c_o) for l in synth.OPT175B_LINEARS]
    layers = []
    for i, (name, c_i, c_o) in enumerate(desc):
        smoothed = name in ("qkv", "fc1")  # inputs that follow a LayerNorm are smoothed; the others use s = 1
        layers.append(make_layer(sq, torch, name, t, c_i, c_o, 0.005, 80.0, 0.5, smoothed, synth.BASE_SEED + 10 * i))
    torch.cuda.synchronize()

    def step():
        for L in layers:
            run_layer(sq, torch, L)

    def make_decode_step(m):
        bufs = []
        for L in layers:
            xs_in = L["x"][:m].contiguous()
            nws = sq.workspace_bytes(sq.OP_W8A8_LINEAR, m, L["c_i"], L["c_o"])
            bufs.append(dict(x=xs_in, xq=sq.empty_codes(m, L["c_i"], sq.TILED),
                             xs=torch.empty(m, dtype=torch.float32, device="cuda"),
                             y=torch.empty((m, L["c_o"]), dtype=torch.bfloat16, device="cuda"),
                             ws=torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")))

        def dstep():
            for L, b in zip(layers, bufs):
                sq.quantize_act(b["x"], sq.PER_TOKEN_DYNAMIC, inv_s=L["inv_s"], out=(b["xq"], b["xs"]), layout=sq.TILED)
                sq.w8a8_linear(b["xq"], b["xs"], L["wq"], L["w_scale"], torch.bfloat16, out=b["y"], workspace=b["ws"],
                               layout=sq.TILED)
        return dstep

    if args.probe:
        src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        dsteps = [make_decode_step(m) for m in (1, 16, 128)]
        for _ in range(2):
            dst.copy_(src)
            step()
            for ds in dsteps:
                ds()
        torch.cuda.synchronize()
        print("probe done: copy of %d bytes + 2 prefill steps + 2 decode steps at 1 / 16 / 128 tokens" % src.numel())
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    total_ops = sum(L["ops"] for L in layers)
    tops = total_ops / (ms_per_step * 1e-3) / 1e12

    # Dominant kernel: the INT8 MFMA GEMM.  Average launch duration measured with events on the stream
    # the kernels run on (torch's current stream is the one the binding passes to the library).
    gemm_ms = 0.0
    quant_ms = 0.0
    for L in layers:
        a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        a.record()
        for _ in range(args.steps):
            sq.quantize_act(L["x"], sq.PER_TOKEN_DYNAMIC, inv_s=L["inv_s"], out=(L["xq"], L["x_scale"]), layout=sq.TILED)
        b.record()
        for _ in range(args.steps):
            sq.w8a8_linear(L["xq"], L["x_scale"], L["wq"], L["w_scale"], torch.bfloat16, out=L["y"], workspace=L["ws"], layout=sq.TILED)
        c.record()
        torch.cuda.synchronize()
        L["quant_us"] = a.elapsed_time(b) / args.steps * 1e3
        L["gemm_us"] = b.elapsed_time(c) / args.steps * 1e3
        gemm_ms += L["gemm_us"] * 1e-3
        quant_ms += L["quant_us"] * 1e-3
    gemm_tops = total_ops / (gemm_ms * 1e-3) / 1e12
    quant_bytes = sum(3.0 * L["t"] * L["c_i"] + 4.0 * L["t"] for L in layers)

    # Decode shapes (Sec. 5.3's generation stage): the same four layers at 1 / 16 / 128 tokens.  Every pass streams
    # all 1.8 GB of int8 weights, far more than any cache holds, so each layer's W comes from HBM every time.
    decode = {}
    for m in (1, 16, 128):
        dstep = make_decode_step(m)
        for _ in range(args.warmup):
            dstep()
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record()
        for _ in range(args.steps):
            dstep()
        d1.record()
        torch.cuda.synchronize()
        dms = d0.elapsed_time(d1) / args.steps
        dbytes = sum(L["c_i"] * L["c_o"] + 4.0 * m * L["c_i"] + 2.0 * m * L["c_o"] for L in layers)
        decode[f"M{m}"] = {"ms_per_step": round(dms, 4), "achieved_GBs": round(dbytes / dms / 1e6, 1),
                           "frac_hbm_peak": round(dbytes / dms / 1e6 / PEAK_HBM_GBS, 4),
                           "tops": round(sum(2.0 * m * L["c_i"] * L["c_o"] for L in layers) / dms / 1e9, 2)}

    # What the INT8 matrix pipes sustain when fed from registers (no memory traffic), on the codes of this workload:
    # the nominal peak assumes 2.4 GHz, the chip holds about 1.6 GHz under a sustained MFMA load.
    probe_data = layers[0]["wq"]
    probe_data = (probe_data._base if probe_data._base is not None else probe_data).reshape(-1)[: 2048 * 49152]
    probe_iters = 20000
    sq.probe_mfma_i8(probe_data, 2048, 2000)
    torch.cuda.synchronize()
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record()
    probe_ops = sq.probe_mfma_i8(probe_data, 2048, probe_iters)
    p1.record()
    torch.cuda.synchronize()
    mfma_only_tops = probe_ops / (p0.elapsed_time(p1) * 1e-3) / 1e12

    # HBM-side traffic of the GEMM launches: measured separately with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on
    # `bench.py --probe` (counters cannot be read from inside this process); the summary is kept under profiles/.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "gemm_i8_opt175b_M2048_hbm_traffic.json")
    if t == 2048 and os.path.exists(tpath):
        with open(tpath) as fh:
            traffic = round(json.load(fh)["gemm_traffic_bytes_per_launch_avg"])

    out = {
        "metric": "W8A8 quant+GEMM+dequant TOPS and % INT8 MFMA peak at OPT-175B layer shapes",
        "value": round(tops, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"opt175b_linears_hidden12288_M{t}: qkv+out_proj+fc1+fc2, per-token dynamic act, "
                               "per-tensor weight, bf16 out, 0.5% outlier channels x80, alpha 0.5"},
        "pct_int8_mfma_peak": round(100.0 * tops / PEAK_INT8_TOPS, 2),
        "roofline": {"bound": "mfma", "kernel": "gemm_i8_kernel (256x384 / 256x256 tiles, INT8 MFMA GEMM + dequant epilogue)",
                     "achieved": round(gemm_tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s",
                     "frac": round(gemm_tops / PEAK_INT8_TOPS, 4), "traffic": traffic,
                     "mfma_only_loop_tops": round(mfma_only_tops, 1),
                     "frac_of_mfma_only_loop": round(gemm_tops / mfma_only_tops, 4),
                     "note": "int8 multiply-accumulate counted as 2 ops; achieved = sum of 2*T*C_i*C_o over the four "
                             "layers / sum of their average GEMM launch durations (HIP events); traffic = HBM-side "
                             "bytes (FETCH_SIZE + WRITE_SIZE, calibrated on a copy) averaged over the four launches; "
                             "mfma_only_loop_tops = register-fed MFMA loop on the same weight codes, 2048 workgroups x 8 "
                             "waves (what the matrix pipes sustain at the clock the chip holds under this load)"},
        "per_layer_us": {L["name"]: {"quantize": round(L["quant_us"], 1), "gemm": round(L["gemm_us"], 1),
                                     "gemm_tops": round(L["ops"] / L["gemm_us"] / 1e6, 1)} for L in layers},
        "quantize_pass": {"bound": "hbm", "achieved_GBs": round(quant_bytes / (quant_ms * 1e-3) / 1e9, 1),
                          "peak_GBs": PEAK_HBM_GBS, "frac": round(quant_bytes / (quant_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
    }
    out["decode"] = {"bound": "hbm", "peak_GBs": PEAK_HBM_GBS,
                     "note": "same four layers, quantize + linear per layer, bytes = int8 W + fp16 x in + codes out/in + "
                             "bf16 y out; weights stream from HBM on every pass (1.8 GB per pass)", **decode}
    layers.clear()
    torch.cuda.empty_cache()
    out["other_configs"] = other_configs(sq, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(desc)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
