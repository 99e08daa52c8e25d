"""The measured-peak probes (include/probe.h) return plausible figures for an MI355X."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_probes_report_plausible_peaks():
    import paper_2603_12440_amd as g
    g.load_library()
    dev = torch.device("cuda:0")
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    for code in (g.BF16, g.F16):
        for refresh in (False, True):
            t = g.probe_mfma_peak(code, sink, min_seconds=0.1, refresh_operands=refresh)
            assert 500.0 < t <= 2516.6 * 1.02, t       # never above the nominal matrix-core peak
    for refresh in (False, True):
        t = g.probe_mfma_peak(g.F8E4M3, sink, min_seconds=0.1, refresh_operands=refresh)
        assert 1000.0 < t <= 5033.2 * 1.02, t
    n = 1 << 30
    buf = torch.ones(n, dtype=torch.uint8, device=dev)
    r = g.probe_read_peak(buf, n, sink, min_seconds=0.1)
    assert 2000.0 < r <= 8000.0 * 1.02, r
    assert float(sink.sum()) == 0.0                     # the sink is never written
