"""Attention output P V (V is [k, n], n contiguous: the transposed-operand path of the batched GEMM) at attention-like
shapes: every output element against the oracle, within 1 ulp of the 16-bit type and almost all identical.  The
shapes cover ragged row blocks, contraction lengths that end in a partly filled K step (every tail length), head
dimensions below, at and above one 128-column tile, and codes that reach the largest accumulators."""
import numpy as np
import pytest

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import assert_identical_16, BF16, F16, bits_from_dev, dev, torch_dtype, ulp_distance

pytestmark = pytest.mark.gpu

CASES = [
    (2, 300, 128, 256),    # two full stages, ragged rows
    (3, 129, 64, 272),     # one chunk in the last stage
    (2, 257, 128, 2048),
    (1, 512, 48, 1008),    # seven chunks in the last stage, narrow head
    (2, 260, 272, 384),    # three column tiles, the last one 16 wide
    (1, 1024, 80, 336),
    (5, 384, 128, 640),
    (1, 200, 16, 304),
]


@pytest.mark.parametrize("b,m,n,k", CASES)
@pytest.mark.parametrize("odt", [F16, BF16])
def test_pv_parity(b, m, n, k, odt):
    print(f"[case] pv bmm b={b} m={m} n={n} k={k} out={odt}", flush=True)
    rng = np.random.default_rng(b * 1000 + k)
    a = rng.integers(0, 128, (b, m, k)).astype(np.int8)  # P codes are non-negative
    v = synth.int8_codes((b, k, n), 82 + m)
    alpha = float(np.float32(0.0211 / 127.0))
    ref = oracle.w8a8_bmm(a, v, False, alpha, odt)
    c = sq.w8a8_bmm(dev(a), dev(v), False, alpha, torch_dtype(odt))
    d = ulp_distance(bits_from_dev(c), ref)
    assert_identical_16(d)


def test_pv_signed_saturated_codes_and_untouched_neighbours():
    """Signed +-127 codes on both sides (the call is a general batched product), power-of-two alpha: exact; and
    nothing is written outside [b, m, n]."""
    import torch
    b, m, n, k = 2, 300, 96, 400
    print(f"[case] pv bmm saturated b={b} m={m} n={n} k={k}", flush=True)
    rng = np.random.default_rng(6)
    a = (rng.integers(0, 2, (b, m, k)) * 254 - 127).astype(np.int8)
    v = (rng.integers(0, 2, (b, k, n)) * 254 - 127).astype(np.int8)
    alpha = float(np.float32(2.0 ** -14))
    ref = oracle.w8a8_bmm(a, v, False, alpha, F16)
    guard = torch.full((b * m * n + 2 * 4096,), 0x7BFF, dtype=torch.int16, device="cuda")
    out = guard[4096:4096 + b * m * n].view(torch.float16).view(b, m, n)
    sq.w8a8_bmm(dev(a), dev(v), False, alpha, torch.float16, out=out)
    assert np.array_equal(bits_from_dev(out), ref)
    g = guard.cpu().numpy()
    assert (g[:4096] == 0x7BFF).all() and (g[4096 + b * m * n:] == 0x7BFF).all()
