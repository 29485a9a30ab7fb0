"""The probe library on the GPU: every level of the MFMA ceiling probe and the vector-issue probe run and
return rates of the right order (they are measurements, so the checks are bounds, not values)."""
import pytest
import torch

from paper_2502_05431_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_mfma_probe_levels_are_ordered_and_below_the_published_peak():
    sink = torch.zeros(4, dtype=torch.float32, device=DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    ops = torch.randn(65536 // 2, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    rate = [B.probe_mfma(ops, level, sink, warm_ms=30.0) for level in range(5)]
    assert all(200.0 < r < 2600.0 for r in rate), rate
    # every layer of extra work costs something (boxes and runs differ by a few per cent)
    assert rate[1] < 1.03 * rate[0] and rate[2] < 1.03 * rate[1] and rate[3] < 1.03 * rate[2], rate
    assert rate[4] < 1.05 * rate[3], rate
    zeros = torch.zeros(65536 // 2, dtype=torch.bfloat16, device=DEV)
    assert B.probe_mfma(zeros, 0, sink, warm_ms=30.0) > rate[0]      # the clock the chip holds depends on the operand data
    assert float(sink.abs().max()) == 0.0                              # the sink is never written
    with pytest.raises(RuntimeError):
        B.probe_mfma(ops, 5, sink)


def test_vector_issue_probe():
    sink = torch.zeros(4, dtype=torch.float32, device=DEV)
    ns = {w: B.probe_valu_issue(w, sink, warm_ms=20.0) for w in (1, 2, 4)}
    # about 5 cycles per instruction at 2.4 GHz; more wavefronts per SIMD never make a SIMD slower
    assert all(1.0 < v < 6.0 for v in ns.values()), ns
    assert ns[4] < 1.1 * ns[1], ns
    with pytest.raises(RuntimeError):
        B.probe_valu_issue(3, sink)
