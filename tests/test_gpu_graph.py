"""The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no synchronisation), so a
decode step can be captured into a HIP graph and replayed.  Every replay is checked against the eager result, with
eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import F16, dev, to_dev_16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("t,c_i,c_o,mode", [(16, 1024, 4096, sq.PER_TOKEN_DYNAMIC),    # weight streaming
                                            (16, 4096, 1024, sq.PER_TOKEN_DYNAMIC),    # split-K tiles + reduction
                                            (128, 4096, 4096, sq.PER_TENSOR_DYNAMIC),  # streaming with a K split, O2 quantizer
                                            (300, 512, 768, sq.PER_TOKEN_DYNAMIC),     # prefill tiles
                                            (2048, 12288, 12288, sq.PER_TOKEN_DYNAMIC)])  # the 256x384 tile (uses scratch memory)
def test_graph_replay_matches_eager(t, c_i, c_o, mode):
    print(f"[case] graph replay t={t} c_i={c_i} c_o={c_o} mode={mode}", flush=True)
    w = synth.weights(c_i, c_o, 4242)
    wq, ws = sq.prepare_weight(to_dev_16(w, F16), None, layout=sq.TILED)
    xs_host = [synth.normal_fp16((t, c_i), 5000 + i) for i in range(3)]
    x = to_dev_16(xs_host[0], F16).clone()
    xq = sq.empty_codes(t, c_i, sq.TILED)
    scale = torch.empty(t if mode == sq.PER_TOKEN_DYNAMIC else 1, dtype=torch.float32, device="cuda")
    y = torch.empty((t, c_o), dtype=torch.float16, device="cuda")
    qws = torch.empty(64, dtype=torch.uint8, device="cuda")
    gws = torch.empty(max(sq.workspace_bytes(sq.OP_W8A8_LINEAR, t, c_i, c_o), 16), dtype=torch.uint8, device="cuda")

    def step():
        sq.quantize_act(x, mode, out=(xq, scale), workspace=qws, layout=sq.TILED)
        sq.w8a8_linear(xq, scale, wq, ws, torch.float16, out=y, workspace=gws, layout=sq.TILED)

    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for i in range(3):
        x.copy_(to_dev_16(xs_host[i], F16))
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        got = y.clone()
        y.zero_()
        step()  # eager, same inputs
        torch.cuda.synchronize()
        assert torch.equal(got, y), f"replay {i} differs from the eager result"
        assert bool(torch.isfinite(y.float()).all()) and float(y.float().abs().max()) > 0.0


def test_graph_replay_attention_chain():
    """Scores (strip kernel) -> softmax + P quantization -> P V captured as one graph."""
    b, s, d = 6, 384, 128
    print(f"[case] graph replay attention b={b} s={s} d={d}", flush=True)
    hosts = [[synth.int8_codes((b, s, d), 7000 + 10 * i + j) for j in range(3)] for i in range(3)]
    q, k, v = (dev(hosts[0][j]).clone() for j in range(3))
    sc = torch.empty((b, s, s), dtype=torch.float16, device="cuda")
    pq = torch.empty((b, s, s), dtype=torch.int8, device="cuda")
    o = torch.empty((b, s, d), dtype=torch.float16, device="cuda")

    def step():
        sq.w8a8_bmm(q, k, True, 3e-4, torch.float16, out=sc)
        sq.softmax_quant_p(sc, out=pq)
        sq.w8a8_bmm(pq, v, False, 1e-3, torch.float16, out=o)

    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for i in range(3):
        for t, h in zip((q, k, v), hosts[i]):
            t.copy_(dev(h))
        o.zero_()
        g.replay()
        torch.cuda.synchronize()
        got, got_p = o.clone(), pq.clone()
        o.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(got, o) and torch.equal(got_p, pq), f"replay {i} differs from the eager result"
        assert float(o.float().abs().max()) > 0.0


def test_graph_replay_fused_attention():
    """The fused attention kernel captured as a graph node, replayed on changing inputs (key count with a masked tail)."""
    b, s_q, s_k, d = 5, 200, 400, 128
    print(f"[case] graph replay fused attention b={b} s_q={s_q} s_k={s_k} d={d}", flush=True)
    hosts = [[synth.int8_codes((b, n, d), 7100 + 10 * i + j) for j, n in enumerate((s_q, s_k, s_k))] for i in range(3)]
    q, k, v = (dev(hosts[0][j]).clone() for j in range(3))
    o = torch.empty((b, s_q, d), dtype=torch.float16, device="cuda")

    def step():
        sq.w8a8_attention(q, k, v, 3e-4, 1e-3, torch.float16, out=o)

    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for i in range(3):
        for t, h in zip((q, k, v), hosts[i]):
            t.copy_(dev(h))
        o.zero_()
        g.replay()
        torch.cuda.synchronize()
        got = o.clone()
        o.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(got, o), f"replay {i} differs from the eager result"
        assert float(o.float().abs().max()) > 0.0
