#!/usr/bin/env python3
"""Benchmark of the SmoothQuant W8A8 hot path on one MI355X.

Workload (N=1): the four OPT-175B-shaped linears at hidden 12288 (QKV 12288->36864, out-proj
12288->12288, FC1 12288->49152, FC2 49152->12288) at M = 2048 tokens, per-token dynamic activation
quantization, per-tensor weights, bf16 output.  One step = for each of the four layers:
quantize_act (fp16 activation -> int8 codes + per-token steps) then w8a8_linear (INT8 MFMA GEMM with
the dequantizing epilogue fused); int8 operands use the library's tiled layout.  Inputs (activations,
prepared int8 weights) are resident in HBM before the timed region.  Prints ONE JSON line.

Timing protocol: HIP events on the stream the kernels are launched on (torch's current stream is the one the
binding hands to the library).  Every kernel that is bound by HBM is timed over a rotation of buffer sets that
together exceed 512 MB, so that the 256 MB memory-side cache cannot serve the same bytes twice; the step itself
rotates three sets of activations, codes and outputs (3 GB) and streams 1.8 GB of weights.  Per-kernel figures
are the median (and the minimum) over several batches of launches.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0  # MI355X dense INT8 MFMA peak, 5.0 POP/s
PEAK_HBM_GBS = 8000.0
ROTATE_BYTES = 600 << 20  # a rotation of buffer sets covers at least this much


def synth_activation(torch, g, t, c_i, outlier_frac, factor):
    """fp16 [t, c_i]: N(0,1) with round(outlier_frac * c_i) generator-chosen channels multiplied by `factor`."""
    x = torch.randn((t, c_i), generator=g, device="cuda", dtype=torch.float32)
    ch = torch.randperm(c_i, generator=g, device="cuda")[:int(round(outlier_frac * c_i))]
    x[:, ch] *= factor
    return x.to(torch.float16), ch


def synth_weight(torch, g, c_i, c_o):
    w = torch.empty((c_i, c_o), device="cuda", dtype=torch.float16)
    rows = 2048
    for r0 in range(0, c_i, rows):  # chunked to bound the fp32 temporary
        w[r0:r0 + rows] = (torch.randn((min(rows, c_i - r0), c_o), generator=g, device="cuda") * 0.02).to(torch.float16)
    return w


def make_layer(sq, torch, name, t, c_i, c_o, outlier_frac, factor, alpha, smoothed, seed, out_dtype=None, nsets=1, x=None,
               relu=False):
    """Synthetic layer with the paper's outlier structure, prepared offline with the library itself.  `nsets` sets of
    activations / codes / outputs are kept for rotation; `x` overrides the drawn activation of set 0 (a real
    producer's output)."""
    out_dtype = out_dtype or torch.bfloat16
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x0, ch = synth_activation(torch, g, t, c_i, outlier_frac, factor)
    w = synth_weight(torch, g, c_i, c_o)
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
    sets = []
    base = x0 if x is None else x
    for i in range(nsets):
        xi = base if i == 0 else base.roll(i, 0)  # the same rows in another order, at other addresses
        sets.append(dict(x=xi, xq=sq.empty_codes(t, c_i, sq.TILED), x_scale=torch.empty(t, dtype=torch.float32, device="cuda"),
                         y=torch.empty((t, c_o), dtype=out_dtype, device="cuda")))
    nws = sq.workspace_bytes(sq.OP_W8A8_LINEAR, t, c_i, c_o)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    return dict(name=name, t=t, c_i=c_i, c_o=c_o, inv_s=inv_s_dev, wq=wq, w_scale=w_scale, sets=sets, ws=ws, relu=relu,
                out_dtype=out_dtype, ops=2.0 * t * c_i * c_o)


def run_quant(sq, L, i=0):
    S = L["sets"][i % len(L["sets"])]
    sq.quantize_act(S["x"], sq.PER_TOKEN_DYNAMIC, inv_s=L["inv_s"], out=(S["xq"], S["x_scale"]), layout=sq.TILED)


def run_gemm(sq, L, i=0):
    S = L["sets"][i % len(L["sets"])]
    sq.w8a8_linear(S["xq"], S["x_scale"], L["wq"], L["w_scale"], L["out_dtype"], relu=L["relu"], out=S["y"],
                   workspace=L["ws"], layout=sq.TILED)


def time_stats(torch, fn, iters=10, reps=5, warm=2):
    """fn(i) is launched `iters` times between two events, `reps` times over; returns (median, min) of the batch
    averages in microseconds.  `i` counts launches, for buffer rotation."""
    n = 0
    for _ in range(warm):
        fn(n)
        n += 1
    per = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn(n)
            n += 1
        b.record()
        torch.cuda.synchronize()
        per.append(a.elapsed_time(b) / iters * 1e3)
    per.sort()
    return per[len(per) // 2], per[0]


def nsets_for(bytes_per_set):
    return max(3, -(-ROTATE_BYTES // int(bytes_per_set)))


def other_configs(sq, torch):
    """Latency and roofline fraction of the other benchmark configurations, on inputs of their kind: activations with
    outlier channels, smoothing factors on the inputs that follow a LayerNorm, the second FFN layer fed with the first
    one's ReLU output, Q / K / V codes from per-tensor quantized N(0,1) tensors.
    1 = OPT-125m-shaped static linear, 2 = OPT-13B-shaped FFN pair, 4 = INT8 attention (batch 8 x 96 heads,
    sequence 2048, head_dim 128), 5 = the linears and attention of an OPT-66B-shaped decoder layer (4 x 1024 tokens)."""
    out = {}
    f16 = torch.float16

    def linear_entry(L, static=False):
        S0 = L["sets"][0]
        if static:  # O3: calibrated per-tensor step, pure elementwise quantizer
            step = torch.empty(1, dtype=torch.float32, device="cuda")
            sq.quantize_act(S0["x"], sq.PER_TENSOR_DYNAMIC, inv_s=L["inv_s"], out=(S0["xq"], step), layout=sq.TILED)

            def q(i):
                S = L["sets"][i % len(L["sets"])]
                sq.quantize_act(S["x"], sq.PER_TENSOR_STATIC, inv_s=L["inv_s"], static_scale=step, out=(S["xq"], step), layout=sq.TILED)

            def gm(i):
                S = L["sets"][i % len(L["sets"])]
                sq.w8a8_linear(S["xq"], step, L["wq"], L["w_scale"], L["out_dtype"], out=S["y"], workspace=L["ws"], layout=sq.TILED)
        else:
            q = lambda i: run_quant(sq, L, i)
            gm = lambda i: run_gemm(sq, L, i)
        for i in range(len(L["sets"])):
            q(i)  # codes of every set exist before the GEMM is timed
        q_us, q_min = time_stats(torch, q)
        g_us, g_min = time_stats(torch, gm)
        ops = L["ops"]
        return {"quantize_us": round(q_us, 1), "gemm_us": round(g_us, 1), "gemm_us_min": round(g_min, 1),
                "tops": round(ops / (q_us + g_us) / 1e6, 1), "frac_mfma_peak": round(ops / (q_us + g_us) / 1e6 / PEAK_INT8_TOPS, 4)}

    # config 1: 16 tokens, 768 -> 3072, 6 outlier channels x60, alpha 0.5, static per-tensor step
    L = make_layer(sq, torch, "c1", 16, 768, 3072, 6 / 768, 60.0, 0.5, True, 9001, out_dtype=f16)
    out["config1_opt125m_static_16x768x3072"] = linear_entry(L, static=True)
    # config 2: FFN pair at 512 tokens; FC1 smoothed (51 outlier channels x40), FC2 (s = 1) on FC1's ReLU output
    L1 = make_layer(sq, torch, "c2fc1", 512, 5120, 20480, 0.01, 40.0, 0.5, True, 9002, out_dtype=f16, nsets=3, relu=True)
    out["config2_opt13b_fc1_512x5120x20480_relu"] = linear_entry(L1)
    L2 = make_layer(sq, torch, "c2fc2", 512, 20480, 5120, 0.0, 1.0, 0.5, False, 9003, out_dtype=f16, nsets=3,
                    x=L1["sets"][0]["y"])
    out["config2_opt13b_fc2_512x20480x5120"] = linear_entry(L2)
    # The same pair with FC2's input quantizer (static per-tensor step, Table 2's O3) fused into FC1's epilogue
    # (sq_w8a8_linear_q8: the ReLU output leaves FC1 as int8 codes) against FC1 + a separate static quantize launch.
    y_step = (L1["sets"][0]["y"].float().abs().max() / 127.0).reshape(1).contiguous()
    S1, S2 = L1["sets"][0], L2["sets"][0]
    run_quant(sq, L1, 0)

    def fc1_fp16(i):
        sq.w8a8_linear(S1["xq"], S1["x_scale"], L1["wq"], L1["w_scale"], f16, relu=True, out=S1["y"], workspace=L1["ws"], layout=sq.TILED)

    def q_static(i):
        sq.quantize_act(S1["y"], sq.PER_TENSOR_STATIC, static_scale=y_step, out=(S2["xq"], y_step), layout=sq.TILED)

    def fc1_q8(i):
        sq.w8a8_linear_q8(S1["xq"], S1["x_scale"], L1["wq"], L1["w_scale"], y_step, f16, relu=True, out=S2["xq"],
                          workspace=L1["ws"], layout=sq.TILED, out_layout=sq.TILED)

    a_us, _ = time_stats(torch, fc1_fp16)
    b_us, _ = time_stats(torch, q_static)
    c_us, _ = time_stats(torch, fc1_q8)
    out["config2_fc1_with_fc2_quantizer_fused"] = {"fc1_fp16_out_us": round(a_us, 1), "static_quantize_us": round(b_us, 1),
                                                   "fc1_int8_out_us": round(c_us, 1),
                                                   "saved_us": round(a_us + b_us - c_us, 1)}
    del L, L1, L2

    def attention(bh, s_len, d, seed):
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        codes, steps = [], []
        for _ in range(3):  # Q, K, V: N(0,1) fp16, per-tensor step amax / 127
            x = torch.randn((bh * s_len, d), generator=g, device="cuda").to(f16)
            cq, cs = sq.quantize_act(x, sq.PER_TENSOR_DYNAMIC)
            codes.append(cq.view(bh, s_len, d))
            steps.append(float(cs.item()))
        q, k, v = codes
        a1, a2 = steps[0] * steps[1] / d ** 0.5, steps[2] / 127.0
        sc = torch.empty((bh, s_len, s_len), dtype=f16, device="cuda")
        pq = torch.empty((bh, s_len, s_len), dtype=torch.int8, device="cuda")
        o = torch.empty((bh, s_len, d), dtype=f16, device="cuda")
        # (the first launches after the multi-GB allocations run slower than the steady state: warm up longer)
        t1, _ = time_stats(torch, lambda i: sq.w8a8_bmm(q, k, True, a1, f16, out=sc), iters=5, reps=3, warm=4)
        t2, _ = time_stats(torch, lambda i: sq.softmax_quant_p(sc, out=pq), iters=4, reps=3)
        t3, _ = time_stats(torch, lambda i: sq.w8a8_bmm(pq, v, False, a2, f16, out=o), iters=4, reps=3)
        tf, tf_min = time_stats(torch, lambda i: sq.w8a8_attention(q, k, v, a1, a2, f16, out=o), iters=4, reps=3)
        # the same block with the decoder's causal mask (not part of the configuration as stated: reported beside it)
        tc, tc_min = time_stats(torch, lambda i: sq.w8a8_attention(q, k, v, a1, a2, f16, out=o, causal=True), iters=4, reps=3)
        b1 = 2.0 * bh * s_len * d + 2.0 * bh * s_len * s_len
        b2 = 3.0 * bh * s_len * s_len
        b3 = bh * s_len * s_len + 3.0 * bh * s_len * d
        ops = 4.0 * bh * s_len * s_len * d
        return {"fused_us": round(tf, 1), "fused_us_min": round(tf_min, 1), "fused_tops": round(ops / tf / 1e6, 1),
                "fused_speedup_vs_chain": round((t1 + t2 + t3) / tf, 3),
                "fused_causal_us": round(tc, 1), "fused_causal_us_min": round(tc_min, 1),
                "chain_us": round(t1 + t2 + t3, 1),
                "bmm1_us": round(t1, 1), "bmm1_frac_hbm": round(b1 / t1 / 1e3 / PEAK_HBM_GBS, 4),
                "softmax_quant_us": round(t2, 1), "softmax_frac_hbm": round(b2 / t2 / 1e3 / PEAK_HBM_GBS, 4),
                "bmm2_us": round(t3, 1), "bmm2_frac_hbm": round(b3 / t3 / 1e3 / PEAK_HBM_GBS, 4),
                "tops_both_bmms": round(ops / (t1 + t3) / 1e6, 1)}

    out["config4_attention_768x2048x128"] = attention(768, 2048, 128, 9004)
    # config 5: OPT-66B-shaped layer, 4 x 1024 tokens, 1 % outlier channels x60, alpha 0.8; QKV and FC1 follow a
    # LayerNorm (smoothed), out-proj takes the attention output, FC2 the ReLU output of FC1
    t5, hid, ffn = 4096, 9216, 36864
    L = make_layer(sq, torch, "c5qkv", t5, hid, 3 * hid, 0.01, 60.0, 0.8, True, 9005, out_dtype=f16, nsets=3)
    out["config5_opt66b_qkv_4096x9216x27648"] = linear_entry(L)
    del L
    L = make_layer(sq, torch, "c5out", t5, hid, hid, 0.0, 1.0, 0.8, False, 9006, out_dtype=f16, nsets=3)
    out["config5_opt66b_out_proj_4096x9216x9216"] = linear_entry(L)
    del L
    L1 = make_layer(sq, torch, "c5fc1", t5, hid, ffn, 0.01, 60.0, 0.8, True, 9007, out_dtype=f16, nsets=3, relu=True)
    out["config5_opt66b_fc1_4096x9216x36864_relu"] = linear_entry(L1)
    L2 = make_layer(sq, torch, "c5fc2", t5, ffn, hid, 0.0, 1.0, 0.8, False, 9008, out_dtype=f16, nsets=3, x=L1["sets"][0]["y"])
    out["config5_opt66b_fc2_4096x36864x9216"] = linear_entry(L2)
    del L1, L2
    out["config5_attention_288x1024x128"] = attention(288, 1024, 128, 9009)
    # LayerNorm with folded smoothing factors + quantization; gamma carries the outlier channels of its output
    g = torch.Generator(device="cuda")
    g.manual_seed(9010)
    n = nsets_for(3 * t5 * hid)
    xs_in = [torch.randn((t5, hid), generator=g, device="cuda").to(f16) for _ in range(n)]
    gamma = torch.ones(hid, device="cuda")
    gamma[torch.randperm(hid, generator=g, device="cuda")[:92]] = 60.0
    inv = torch.rand(hid, generator=g, device="cuda") + 0.5
    gamma_f, beta_f = (gamma * inv).contiguous(), (torch.randn(hid, generator=g, device="cuda") * 0.1 * inv).contiguous()
    outs = [(sq.empty_codes(t5, hid, sq.TILED), torch.empty(t5, dtype=torch.float32, device="cuda")) for _ in range(n)]
    ln_us, ln_min = time_stats(torch, lambda i: sq.ln_quantize(xs_in[i % n], gamma_f, beta_f, out=outs[i % n], layout=sq.TILED))
    out["config5_ln_quantize_4096x9216"] = {"us": round(ln_us, 1), "us_min": round(ln_min, 1), "buffer_sets": n,
                                            "frac_hbm": round(3.0 * t5 * hid / ln_us / 1e3 / PEAK_HBM_GBS, 4)}
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


def power_probe(sq, torch, seconds=2.0):
    """Is the prefill GEMM bound by its schedule or by the power the chip may draw?  The same launch (2048 x 12288 ->
    36864, tiled operands) on operands of different bit activity, with the shader clock sampled (rocm-smi) while the
    launch repeats for `seconds`.  Prints one JSON line."""
    M, K, N = 2048, 12288, 36864
    ws1 = torch.full((1,), 0.01, device="cuda")
    xs = torch.rand(M, device="cuda")
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")

    def sclk():
        """Current shader clock in MHz from sysfs (no child process: nothing may exec once the GPU is initialised)."""
        import glob
        for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
            try:
                for line in open(path).read().splitlines():
                    if line.rstrip().endswith("*"):
                        return int("".join(c for c in line.split(":")[1] if c.isdigit()))
            except Exception:
                pass
        return None

    def watts(name="power1_input"):
        """Socket power (or its cap) in watts from the hwmon sensor, None if the box does not expose it."""
        import glob
        for path in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/" + name)):
            try:
                return round(int(open(path).read().strip()) / 1e6, 1)
            except Exception:
                pass
        return None

    def codes(kind, shape):
        t = sq.empty_codes(shape[0], shape[1], sq.TILED)
        base = t._base if t._base is not None else t
        if kind == "zeros":
            base.zero_()
        elif kind == "uniform":
            base.random_(-127, 128)
        else:  # Gaussian codes of the given standard deviation (what quantized activations / weights look like)
            sd = float(kind.split("_")[1])
            base.copy_((torch.randn(base.shape, device="cuda") * sd).round().clamp(-127, 127).to(torch.int8))
        return t

    res = {"shape": f"{M}x{K}->{N}", "idle_sclk_mhz": sclk(), "idle_watts": watts(), "power_cap_watts": watts("power1_cap"),
           "cases": {}}
    for kind in ("zeros", "gauss_5", "gauss_20", "uniform"):
        a, b = codes(kind, (M, K)), codes(kind, (N, K))
        fn = lambda i: sq.w8a8_linear(a, xs, b, ws1, torch.bfloat16, out=y, layout=sq.TILED)
        stop, samples, power = [False], [], []

        def sampler():
            while not stop[0]:
                v, w = sclk(), watts()
                if v:
                    samples.append(v)
                if w:
                    power.append(w)
                time.sleep(0.05)
        th = threading.Thread(target=sampler)
        th.start()
        t0, n = time.time(), 0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        while time.time() - t0 < seconds:
            for _ in range(50):
                fn(n)
                n += 1
            torch.cuda.synchronize()
        e1.record()
        torch.cuda.synchronize()
        stop[0] = True
        th.join()
        us = e0.elapsed_time(e1) / n * 1e3
        res["cases"][kind] = {"us": round(us, 1), "tops": round(2.0 * M * N * K / us / 1e6, 1),
                              "frac_int8_peak": round(2.0 * M * N * K / us / 1e6 / PEAK_INT8_TOPS, 4),
                              "sclk_mhz_last": samples[-1] if samples else None, "sclk_mhz_samples": samples[1:6],
                              "watts_last": power[-1] if power else None, "watts_max": max(power) if power else None}
    print(json.dumps(res))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--probe", action="store_true",
                    help="counter probe for rocprofv3 --pmc: a 512 MiB device copy (known size), two steps of the "
                         "workload and two decode steps at 1 / 16 / 128 tokens, nothing timed, no JSON")
    ap.add_argument("--probe-attention", action="store_true",
                    help="counter probe for rocprofv3 --pmc: a 512 MiB device copy, then the INT8 attention chain "
                         "(scores, softmax + P quantization, P V) and the fused kernel at 768 heads x 2048 x 128 twice, "
                         "nothing timed, no JSON")
    ap.add_argument("--power-probe-seconds", type=float, default=2.0)
    ap.add_argument("--power-probe", action="store_true",
                    help="the QKV-shaped GEMM on operands of different bit activity with the shader clock sampled; "
                         "prints its own JSON line")
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
    if args.power_probe:
        power_probe(sq, torch, args.power_probe_seconds)
        return
    if args.probe_attention:
        bh, s_len, d = 768, 2048, 128
        g = torch.Generator(device="cuda")
        g.manual_seed(78)
        q, k, v = ((torch.randn((bh, s_len, d), generator=g, device="cuda") * 30).round().clamp(-127, 127).to(torch.int8)
                   for _ in range(3))
        sc = torch.empty((bh, s_len, s_len), dtype=torch.float16, device="cuda")
        pq = torch.empty((bh, s_len, s_len), dtype=torch.int8, device="cuda")
        o = torch.empty((bh, s_len, d), dtype=torch.float16, device="cuda")
        src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
            sq.w8a8_bmm(q, k, True, 8e-5, torch.float16, out=sc)
            sq.softmax_quant_p(sc, out=pq)
            sq.w8a8_bmm(pq, v, False, 1e-4, torch.float16, out=o)
            sq.w8a8_attention(q, k, v, 8e-5, 1e-4, torch.float16, out=o)
        torch.cuda.synchronize()
        print("probe done: copy of %d bytes + 2 x (attention chain, fused attention) at %d heads x %d x %d" % (src.numel(), bh, s_len, d))
        return
    t = args.tokens
    desc = [(l.name, l.c_i, l.c_o) for l in synth.OPT175B_LINEARS]
    layers = []
    for i, (name, c_i, c_o) in enumerate(desc):
        smoothed = name in ("qkv", "fc1")  # inputs that follow a LayerNorm are smoothed; the others use s = 1
        # enough sets that the quantize pass of this layer, timed alone, rotates over more than the cache holds
        layers.append(make_layer(sq, torch, name, t, c_i, c_o, 0.005, 80.0, 0.5, smoothed, synth.BASE_SEED + 10 * i,
                                 nsets=nsets_for(3 * t * c_i)))
    torch.cuda.synchronize()
    step_no = [0]

    def step():
        i = step_no[0]
        step_no[0] += 1
        for L in layers:
            run_quant(sq, L, i)
            run_gemm(sq, L, i)

    def make_decode_step(m):
        bufs = []
        for L in layers:
            xs_in = L["sets"][0]["x"][:m].contiguous()
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

    # Dominant kernel: the INT8 MFMA GEMM.  Average launch duration from events on the launch stream, median over
    # batches; the quantize pass of each layer likewise, rotating over its buffer sets (> 512 MB together).
    gemm_ms = quant_ms = 0.0
    for L in layers:
        L["quant_us"], L["quant_us_min"] = time_stats(torch, lambda i: run_quant(sq, L, i), iters=args.steps, reps=5)
        L["gemm_us"], L["gemm_us_min"] = time_stats(torch, lambda i: run_gemm(sq, L, i), iters=args.steps, reps=5)
        gemm_ms += L["gemm_us"] * 1e-3
        quant_ms += L["quant_us"] * 1e-3
    gemm_tops = total_ops / (gemm_ms * 1e-3) / 1e12
    quant_bytes = sum(3.0 * L["t"] * L["c_i"] + 4.0 * L["t"] for L in layers)

    # Decode shapes (Sec. 5.3's generation stage): the same four layers at 1 / 16 / 128 tokens.  Every pass streams
    # all 1.8 GB of int8 weights, far more than any cache holds, so each layer's W comes from HBM every time.
    decode = {}
    for m in (1, 16, 64, 128):
        dstep = make_decode_step(m)
        d_us, d_min = time_stats(torch, lambda i: dstep(), iters=args.steps, reps=3, warm=args.warmup)
        dms = d_us * 1e-3
        dbytes = sum(L["c_i"] * L["c_o"] + 4.0 * m * L["c_i"] + 2.0 * m * L["c_o"] for L in layers)
        decode[f"M{m}"] = {"ms_per_step": round(dms, 4), "ms_per_step_min": round(d_min * 1e-3, 4),
                           "achieved_GBs": round(dbytes / dms / 1e6, 1),
                           "frac_hbm_peak": round(dbytes / dms / 1e6 / PEAK_HBM_GBS, 4),
                           "tops": round(sum(2.0 * m * L["c_i"] * L["c_o"] for L in layers) / dms / 1e9, 2)}

    # What the INT8 matrix pipes sustain when fed from registers (no memory traffic), on the codes of this workload:
    # the nominal peak assumes 2.4 GHz, the chip holds less under a sustained MFMA load (power).
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

    # HBM-side traffic of the GEMM launches cannot be read from inside this process: it is the figure measured with
    # rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on `bench.py --probe` and stored under profiles/.
    traffic = None
    traffic_src = None
    tpath = os.path.join(ROOT, "profiles", "gemm_i8_opt175b_M2048_hbm_traffic.json")
    if t == 2048 and os.path.exists(tpath):
        with open(tpath) as fh:
            tj = json.load(fh)
        traffic = round(tj["gemm_traffic_bytes_per_launch_avg"])
        traffic_src = ("stored figure, not measured in this run: profiles/gemm_i8_opt175b_M2048_hbm_traffic.json "
                       "(rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, on `bench.py --probe`, scaled by the same counters on a "
                       "512 MiB copy)" + (", library at " + tj["library_commit"] if "library_commit" in tj else ""))

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
        "roofline": {"bound": "mfma", "kernel": "gemm_i8_kernel (256x384 tiles, 16x16x64 INT8 MFMA, GEMM + dequant epilogue)",
                     "achieved": round(gemm_tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s",
                     "frac": round(gemm_tops / PEAK_INT8_TOPS, 4), "traffic": traffic, "traffic_source": traffic_src,
                     "mfma_only_loop_tops": round(mfma_only_tops, 1),
                     "frac_of_mfma_only_loop": round(gemm_tops / mfma_only_tops, 4),
                     "note": "int8 multiply-accumulate counted as 2 ops; achieved = sum of 2*T*C_i*C_o over the four "
                             "layers / sum of their median GEMM launch durations (HIP events on the launch stream); "
                             "mfma_only_loop_tops = register-fed 16x16x64 MFMA loop on the same weight codes, 2048 workgroups x 8 "
                             "waves: what the matrix pipes sustain at the clock the chip holds under this load (the "
                             "clock is set by the power the operands' bit activity draws: `bench.py --power-probe`)"},
        "per_layer_us": {L["name"]: {"quantize": round(L["quant_us"], 1), "quantize_min": round(L["quant_us_min"], 1),
                                     "quantize_buffer_sets": len(L["sets"]),
                                     "quantize_GBs": round((3.0 * L["t"] * L["c_i"] + 4.0 * L["t"]) / L["quant_us"] / 1e3, 1),
                                     "gemm": round(L["gemm_us"], 1), "gemm_min": round(L["gemm_us_min"], 1),
                                     "gemm_tops": round(L["ops"] / L["gemm_us"] / 1e6, 1)} for L in layers},
        "quantize_pass": {"bound": "hbm", "achieved_GBs": round(quant_bytes / (quant_ms * 1e-3) / 1e9, 1),
                          "peak_GBs": PEAK_HBM_GBS, "frac": round(quant_bytes / (quant_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                          "note": "each layer's launch rotates over buffer sets of more than 512 MB together"},
    }
    out["decode"] = {"bound": "hbm", "peak_GBs": PEAK_HBM_GBS,
                     "note": "same four layers, quantize + linear per layer, bytes = int8 W + fp16 x in + codes out/in + "
                             "bf16 y out; weights stream from HBM on every pass (1.8 GB per pass)", **decode}
    layers.clear()
    torch.cuda.empty_cache()
    if not args.no_other_configs:
        out["other_configs"] = other_configs(sq, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(desc)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
