"""The matrix-rate probe (a measurement utility of the library, not an operation of the paper): it runs,
counts its work as stated in the header, and rejects bad arguments without launching."""
import pytest
import torch

from paper_2512_07011_amd import binding

pytestmark = pytest.mark.gpu


def test_probe_runs_and_reports_a_plausible_rate():
    dev = torch.device("cuda:0")
    wgs, iters = 512, 2000
    ops = torch.randn(4096, generator=torch.Generator().manual_seed(3)).to(dev)
    sink = torch.zeros(wgs * 512, dtype=torch.float32, device=dev)
    fl = binding.mfma_rate_probe(ops, wgs, iters, sink)
    assert fl == wgs * 8 * iters * 16 * 2.0 * 32 * 32 * 16
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    binding.mfma_rate_probe(ops, wgs, iters, sink)
    e1.record()
    torch.cuda.synchronize()
    tflops = fl / (e0.elapsed_time(e1) * 1e-3) / 1e12
    # well above anything the vector units could do, not above the published matrix peak
    assert 300.0 < tflops < 2600.0, tflops
    # every lane has written a finite sum; with zero operands the sums are exactly zero
    assert torch.isfinite(sink).all()
    binding.mfma_rate_probe(torch.zeros(4096, device=dev), wgs, 10, sink)
    torch.cuda.synchronize()
    assert (sink == 0).all()


def test_probe_rejects_bad_arguments():
    dev = torch.device("cuda:0")
    L = binding.lib()
    ops = torch.zeros(4096, device=dev)
    sink = torch.full((512,), 7.0, device=dev)
    nbytes = sink.numel() * 4
    assert L.bsfa_mfma_rate_probe_sink_bytes(1) == 512 * 4
    assert L.bsfa_mfma_rate_probe_sink_bytes(0) == 0
    assert L.bsfa_mfma_rate_probe_flops(0, 5) == 0.0
    assert L.bsfa_mfma_rate_probe(ops.data_ptr(), sink.data_ptr(), nbytes, 2, 10, None) == -5
    assert L.bsfa_mfma_rate_probe(None, sink.data_ptr(), nbytes, 1, 10, None) == -1
    assert L.bsfa_mfma_rate_probe(ops.data_ptr(), sink.data_ptr(), nbytes, 1, 0, None) == -2
    torch.cuda.synchronize()
    assert (sink == 7.0).all()          # nothing was launched
