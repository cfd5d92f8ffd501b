"""The MFMA-only measurement loop: accumulators are linear in the iteration count (exact int32), and argument errors
are caught on the host."""
import ctypes

import pytest
import torch

from paper_2211_10438_amd import binding as sq

pytestmark = pytest.mark.gpu


def test_probe_is_linear_in_iterations():
    print("[case] mfma probe", flush=True)
    wgs = 4
    data = torch.randint(-5, 6, (wgs * 49152,), dtype=torch.int8, device="cuda")
    L = sq.lib()
    sinks = []
    for iters in (1, 7):
        sink = torch.zeros(wgs * 512, dtype=torch.int32, device="cuda")
        st = L.sq_probe_mfma_i8(data.data_ptr(), data.numel(), wgs, iters, sink.data_ptr(), None)
        assert st == 0
        torch.cuda.synchronize()
        sinks.append(sink.cpu())
    assert torch.equal(sinks[1], sinks[0] * 7) and bool(sinks[0].abs().max() > 0)
    assert sq.probe_mfma_i8(data, wgs, 3) == wgs * 8 * 3 * 8 * 65536
    # host-side argument checks
    assert L.sq_probe_mfma_i8(data.data_ptr(), 100, wgs, 1, sinks[0].data_ptr(), None) == 5  # data too small
    assert L.sq_probe_mfma_i8(None, data.numel(), wgs, 1, ctypes.c_void_p(0x1000), None) == 1
