"""sq_w8a8_linear_noalloc (the entry point for callers that cannot allocate: its K-split scratch is a device
array inside the library) against sq_w8a8_linear with a caller-owned workspace, through the C ABI.  Both run the same
kernels, so outputs must be identical; the first call is also checked against the oracle.  Two calls in a row share
the library's scratch array, the second with a smaller input: stale partial sums of the first must not leak."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_10438_amd import binding as sq
from tests._util import BF16, F16, assert_identical_16, bits_from_dev, dev, ulp_distance

pytestmark = pytest.mark.gpu


def _case(t, c_i, c_o, seed):
    rng = np.random.default_rng(seed)
    xq = rng.integers(-127, 128, (t, c_i), dtype=np.int8)
    wq = rng.integers(-127, 128, (c_o, c_i), dtype=np.int8)
    xs = (rng.random(t, dtype=np.float32) + np.float32(0.5)) * np.float32(2e-3)
    ws = np.array([3e-4], np.float32)
    bias = rng.standard_normal(c_o).astype(np.float32)
    return xq, wq, xs, ws, bias


def _run_pair(t, c_i, c_o, seed, out_dtype, odt):
    print(f"[case] no-alloc linear t={t} c_i={c_i} c_o={c_o}", flush=True)
    need = sq.workspace_bytes(sq.OP_W8A8_LINEAR, t, c_i, c_o)
    assert 0 < need <= sq.lib().sq_static_scratch_bytes(), "the case must exercise the K-split scratch"
    xq, wq, xs, ws, bias = _case(t, c_i, c_o, seed)
    d_xq, d_wq, d_xs, d_ws, d_b = dev(xq), dev(wq), dev(xs), dev(ws), dev(bias)
    want = sq.w8a8_linear(d_xq, d_xs, d_wq, d_ws, out_dtype, bias=d_b, relu=True)
    got = torch.full((t, c_o), float("nan"), dtype=out_dtype, device="cuda")
    sq.w8a8_linear_noalloc(d_xq, d_xs, d_wq, d_ws, got, bias=d_b, relu=True)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16)), "differs from sq_w8a8_linear"
    return xq, wq, xs, ws, bias, got


def test_noalloc_linear_two_calls_shared_scratch():
    # first call: 96 tokens, K split with 15 MB of partial sums
    xq, wq, xs, ws, bias, got = _run_pair(96, 20480, 5120, 901, torch.bfloat16, BF16)
    ref = oracle.w8a8_linear(xq, xs, wq, ws, BF16, bias=bias, relu=True)
    assert_identical_16(ulp_distance(bits_from_dev(got), ref))
    # second call, smaller, ragged token count: reuses the same scratch bytes
    xq, wq, xs, ws, bias, got = _run_pair(40, 2048, 512, 902, torch.float16, F16)
    ref = oracle.w8a8_linear(xq, xs, wq, ws, F16, bias=bias, relu=True)
    assert_identical_16(ulp_distance(bits_from_dev(got), ref))
