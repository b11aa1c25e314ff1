"""The measurement kernels behind the benchmark's achievable peaks: the copy copies, the work figures are what the
launch does, and the rates are physically possible."""
import pytest
import torch

import paper_2202_00774_amd as sdgp

pytestmark = pytest.mark.gpu


def test_copy_copies_and_reports_both_directions():
    for nbytes in (16, 4096 + 16, (1 << 20) + 48):
        a = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda")
        b = torch.zeros_like(a)
        work = sdgp.sdgp_peak_probe(0, a, b, nbytes)
        torch.cuda.synchronize()
        assert work == 2.0 * nbytes
        assert torch.equal(a, b)
    assert sdgp.sdgp_peak_probe(0, a, b, 0) == 0.0


def test_read_and_matrix_probes_report_their_work():
    a = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16384, dtype=torch.uint8, device="cuda")
    assert sdgp.sdgp_peak_probe(1, a, sink, a.numel()) == float(a.numel())
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    waves = cus * 2 * 4
    assert sdgp.sdgp_peak_probe(2, None, sink, iters=3) == waves * 3 * 8 * 2.0 * 32 * 32 * 16
    assert sdgp.sdgp_peak_probe(3, None, sink, iters=3) == waves * 3 * 8 * 2.0 * 32 * 32 * 32
    torch.cuda.synchronize()


def test_matrix_probe_rate_is_below_the_published_peak():
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    for kind, peak in ((2, 2.6e15), (3, 5.2e15)):
        sdgp.sdgp_peak_probe(kind, None, sink, iters=2000)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        work = sdgp.sdgp_peak_probe(kind, None, sink, iters=20000)
        e1.record()
        torch.cuda.synchronize()
        rate = work / (e0.elapsed_time(e1) * 1e-3)
        assert 0.2 * peak < rate < peak, (kind, rate)
