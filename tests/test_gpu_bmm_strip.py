"""Attention scores Q K^T through the strip kernel (contraction <= 128 bytes, whole 128-column tiles, more than
128 query rows): every output element against the oracle, within 1 ulp of the 16-bit type and almost all
identical.  The shapes cover ragged row blocks (rows past M are computed as copies of row M-1), every number of
32-wide K steps including a half-filled last one, strips split between workgroups (few heads) and full strips
(many heads), and saturated codes."""
import numpy as np
import pytest

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import assert_identical_16, BF16, F16, bits_from_dev, dev, torch_dtype, ulp_distance

pytestmark = pytest.mark.gpu

CASES = [
    (3, 300, 256, 128),    # ragged last row block
    (2, 129, 128, 16),     # one K chunk, one row in the second block
    (1, 1000, 384, 80),    # five K chunks: the third K step is half filled
    (2, 512, 1024, 96),
    (1, 2048, 2048, 128),  # one head: strips are split into single tiles
    (5, 257, 640, 112),
    (40, 384, 1536, 64),   # enough (head, row block) pairs for whole strips of 12 tiles
    (2, 161, 128, 48),
]


@pytest.mark.parametrize("b,m,n,k", CASES)
@pytest.mark.parametrize("odt", [F16, BF16])
def test_strip_scores_parity(b, m, n, k, odt):
    print(f"[case] strip bmm b={b} m={m} n={n} k={k} out={odt}", flush=True)
    a = synth.int8_codes((b, m, k), 71 + b)
    bt = synth.int8_codes((b, n, k), 72 + m)
    alpha = float(np.float32(0.0137 * 0.0121 / np.sqrt(128.0)))
    ref = oracle.w8a8_bmm(a, bt, True, alpha, odt)
    c = sq.w8a8_bmm(dev(a), dev(bt), True, alpha, torch_dtype(odt))
    d = ulp_distance(bits_from_dev(c), ref)
    assert_identical_16(d)


def test_strip_scores_saturated_codes_and_untouched_neighbours():
    """All codes +-127 (largest accumulators), and the kernel writes nothing outside [b, m, n]."""
    import torch
    b, m, n, k = 2, 200, 256, 128
    print(f"[case] strip bmm saturated b={b} m={m} n={n} k={k}", flush=True)
    rng = np.random.default_rng(5)
    a = (rng.integers(0, 2, (b, m, k)) * 254 - 127).astype(np.int8)
    bt = (rng.integers(0, 2, (b, n, k)) * 254 - 127).astype(np.int8)
    alpha = float(np.float32(2.0 ** -12))
    ref = oracle.w8a8_bmm(a, bt, True, alpha, F16)
    guard = torch.full((b * m * n + 2 * 4096,), 0x7BFF, dtype=torch.int16, device="cuda")
    out = guard[4096:4096 + b * m * n].view(torch.float16).view(b, m, n)
    sq.w8a8_bmm(dev(a), dev(bt), True, alpha, torch.float16, out=out)
    assert np.array_equal(bits_from_dev(out), ref)  # power-of-two alpha: the scaling is exact
    g = guard.cpu().numpy()
    assert (g[:4096] == 0x7BFF).all() and (g[4096 + b * m * n:] == 0x7BFF).all()
