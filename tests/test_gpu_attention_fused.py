"""Fused INT8 attention (Sec. 4: both batched matmuls in INT8 around a 16-bit softmax) against the oracle's chain
of the three steps it fuses.  The kernel keeps the probability codes in registers; for the comparison it is asked to
write them out as well.  Gates: codes within one of the oracle's, at most one in a thousand different (exponential
and division are fp32 on the device, fp64 in the oracle); the output identical to the oracle's P V product of the
codes the kernel itself formed (exact integer sums, fixed fp32 epilogue); and the output must not depend on
whether the codes are written out."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_10438_amd import binding as sq
from paper_2211_10438_amd import synth
from tests._util import BF16, F16, assert_identical_16, bits_from_dev, dev, torch_dtype

pytestmark = pytest.mark.gpu


def _codes(shape, seed):
    """Per-tensor quantized N(0,1) values, as Q, K, V are after the static quantizer."""
    x = synth.normal_fp16(shape, seed).astype(np.float32)
    delta = np.float32(np.abs(x).max() / np.float32(127.0))
    return np.clip(np.rint(x / delta), -127, 127).astype(np.int8), delta


# key counts that are not multiples of the 128-key tile exercise the masked last tile (16-key granularity)
CASES = [(2, 128, 128, 128), (3, 300, 384, 128), (2, 33, 256, 64), (5, 257, 640, 64), (1, 1, 128, 128), (4, 512, 1024, 128),
         (3, 130, 400, 128), (2, 64, 48, 64), (2, 200, 144, 128), (1, 40, 16, 128), (2, 96, 1008, 64)]


@pytest.mark.parametrize("b,s_q,s_k,d", CASES)
@pytest.mark.parametrize("odt", [F16, BF16])
def test_fused_attention_vs_oracle_chain(b, s_q, s_k, d, odt):
    print(f"[case] fused attention b={b} s_q={s_q} s_k={s_k} d={d} dtype={odt}", flush=True)
    q, dq = _codes((b, s_q, d), 300 + s_q)
    k, dk = _codes((b, s_k, d), 301 + s_k)
    v, dv = _codes((b, s_k, d), 302 + s_k)
    alpha1 = float(np.float32(dq * dk) / np.float32(np.sqrt(np.float32(d))))
    alpha2 = float(np.float32(dv) / np.float32(127.0))
    tdt = torch_dtype(odt)
    pq = torch.full((b, s_q, s_k), -128, dtype=torch.int8, device="cuda")
    o = sq.w8a8_attention(dev(q), dev(k), dev(v), alpha1, alpha2, tdt, p_codes=pq)
    o_plain = sq.w8a8_attention(dev(q), dev(k), dev(v), alpha1, alpha2, tdt)
    assert torch.equal(o.view(torch.int16), o_plain.view(torch.int16))
    # stage 1 + 2 of the oracle's chain: scores, softmax, codes
    sc_ref = oracle.w8a8_bmm(q, k, True, alpha1, odt)
    pq_ref = oracle.softmax_quant_p(sc_ref, odt).astype(np.int32)
    got = pq.cpu().numpy().astype(np.int32)
    assert got.min() >= 0, "a code was not written"
    diff = np.abs(got - pq_ref)
    assert diff.max() <= 1 and (diff != 0).mean() <= 1e-3, f"codes: max diff {diff.max()}, rate {(diff != 0).mean():.2e}"
    # stage 3 on the kernel's own codes: exact
    o_ref = oracle.w8a8_bmm(pq.cpu().numpy(), v, False, alpha2, odt)
    from tests._util import ulp_distance
    assert_identical_16(ulp_distance(bits_from_dev(o), o_ref))


def test_fused_attention_matches_the_unfused_library_chain():
    """Same quantization points as sq_w8a8_bmm -> sq_softmax_quant_p -> sq_w8a8_bmm: the scores are identical by
    construction, the row sums are accumulated in a different order, so codes may differ by one, rarely."""
    b, s_q, s_k, d = 6, 384, 768, 128
    q, dq = _codes((b, s_q, d), 310)
    k, dk = _codes((b, s_k, d), 311)
    v, dv = _codes((b, s_k, d), 312)
    alpha1 = float(np.float32(dq * dk) / np.float32(np.sqrt(np.float32(d))))
    alpha2 = float(np.float32(dv) / np.float32(127.0))
    sc = sq.w8a8_bmm(dev(q), dev(k), True, alpha1, torch.float16)
    pq_chain = sq.softmax_quant_p(sc)
    pq = torch.empty_like(pq_chain)
    sq.w8a8_attention(dev(q), dev(k), dev(v), alpha1, alpha2, torch.float16, p_codes=pq)
    diff = (pq.to(torch.int32) - pq_chain.to(torch.int32)).abs()
    assert int(diff.max()) <= 1 and float((diff != 0).float().mean()) <= 1e-3


# (b, s_q, s_k, d): square and with earlier keys in front (s_k > s_q); key counts off the 128-key tile; one query
CAUSAL_CASES = [(2, 128, 128, 128), (3, 300, 304, 128), (2, 256, 256, 64), (2, 33, 256, 64), (3, 257, 640, 64), (1, 1, 128, 128),
                (2, 512, 1024, 128), (2, 130, 400, 128), (2, 48, 48, 64), (2, 200, 208, 128), (1, 16, 16, 128), (2, 96, 1008, 64),
                (2, 640, 640, 128), (1, 1, 16, 64)]


@pytest.mark.parametrize("b,s_q,s_k,d", CAUSAL_CASES)
@pytest.mark.parametrize("odt", [F16, BF16])
def test_fused_causal_attention_vs_oracle_chain(b, s_q, s_k, d, odt):
    """The causal form against the oracle's chain scores -> causal softmax + codes -> P V; same gates as above.  The
    code buffer starts at -128 everywhere, so a position the kernel skipped without writing its 0 shows."""
    print(f"[case] fused causal attention b={b} s_q={s_q} s_k={s_k} d={d} dtype={odt}", flush=True)
    q, dq = _codes((b, s_q, d), 320 + s_q)
    k, dk = _codes((b, s_k, d), 321 + s_k)
    v, dv = _codes((b, s_k, d), 322 + s_k)
    alpha1 = float(np.float32(dq * dk) / np.float32(np.sqrt(np.float32(d))))
    alpha2 = float(np.float32(dv) / np.float32(127.0))
    tdt = torch_dtype(odt)
    pq = torch.full((b, s_q, s_k), -128, dtype=torch.int8, device="cuda")
    o = sq.w8a8_attention(dev(q), dev(k), dev(v), alpha1, alpha2, tdt, p_codes=pq, causal=True)
    o_plain = sq.w8a8_attention(dev(q), dev(k), dev(v), alpha1, alpha2, tdt, causal=True)
    assert torch.equal(o.view(torch.int16), o_plain.view(torch.int16))
    sc_ref = oracle.w8a8_bmm(q, k, True, alpha1, odt)
    pq_ref = oracle.softmax_quant_p_causal(sc_ref, odt).astype(np.int32)
    got = pq.cpu().numpy().astype(np.int32)
    assert got.min() >= 0, "a code was not written"
    off = s_k - s_q
    for i in range(s_q):
        assert not got[:, i, i + off + 1:].any(), f"row {i}: a hidden key got a probability"
    diff = np.abs(got - pq_ref)
    assert diff.max() <= 1 and (diff != 0).mean() <= 1e-3, f"codes: max diff {diff.max()}, rate {(diff != 0).mean():.2e}"
    o_ref = oracle.w8a8_bmm(pq.cpu().numpy(), v, False, alpha2, odt)
    from tests._util import ulp_distance
    assert_identical_16(ulp_distance(bits_from_dev(o), o_ref))


def test_fused_causal_attention_tiny_alpha():
    """Scores that all round to (nearly) the same 16-bit value: the mask must still hide keys (it may not rely on a
    hidden score being a large negative number)."""
    b, s_q, s_k, d = 1, 160, 160, 128
    q, _ = _codes((b, s_q, d), 330)
    k, _ = _codes((b, s_k, d), 331)
    v, dv = _codes((b, s_k, d), 332)
    alpha1, alpha2 = 1e-12, float(np.float32(dv) / np.float32(127.0))
    pq = torch.full((b, s_q, s_k), -128, dtype=torch.int8, device="cuda")
    sq.w8a8_attention(dev(q), dev(k), dev(v), alpha1, alpha2, torch.float16, p_codes=pq, causal=True)
    sc_ref = oracle.w8a8_bmm(q, k, True, alpha1, F16)
    pq_ref = oracle.softmax_quant_p_causal(sc_ref, F16).astype(np.int32)
    diff = np.abs(pq.cpu().numpy().astype(np.int32) - pq_ref)
    assert diff.max() <= 1 and (diff != 0).mean() <= 1e-3


def test_fused_causal_attention_matches_the_masked_library_chain():
    """sq_w8a8_bmm -> -inf written at the hidden positions -> sq_softmax_quant_p gives the same codes (within one, rarely)."""
    b, s_q, s_k, d = 4, 384, 512, 128
    q, dq = _codes((b, s_q, d), 340)
    k, dk = _codes((b, s_k, d), 341)
    v, dv = _codes((b, s_k, d), 342)
    alpha1 = float(np.float32(dq * dk) / np.float32(np.sqrt(np.float32(d))))
    alpha2 = float(np.float32(dv) / np.float32(127.0))
    sc = sq.w8a8_bmm(dev(q), dev(k), True, alpha1, torch.float16)
    hidden = torch.ones((s_q, s_k), dtype=torch.bool, device="cuda").triu(diagonal=s_k - s_q + 1)
    sc.masked_fill_(hidden, float("-inf"))
    pq_chain = sq.softmax_quant_p(sc)
    pq = torch.empty_like(pq_chain)
    o = sq.w8a8_attention(dev(q), dev(k), dev(v), alpha1, alpha2, torch.float16, p_codes=pq, causal=True)
    diff = (pq.to(torch.int32) - pq_chain.to(torch.int32)).abs()
    assert int(diff.max()) <= 1 and float((diff != 0).float().mean()) <= 1e-3
    o_chain = sq.w8a8_bmm(pq, dev(v), False, alpha2, torch.float16)
    assert torch.equal(o.view(torch.int16), o_chain.view(torch.int16))
