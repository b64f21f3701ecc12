"""The device-ceiling probes run, stay inside their buffers and report their work."""
import pytest
import torch

from paper_2511_10676_amd import binding as B

pytestmark = pytest.mark.gpu


def test_read_probe_runs_and_rejects_small_sink():
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    guard = torch.full((64,), 7, dtype=torch.uint8, device="cuda")
    B.probe_read(src, sink)
    torch.cuda.synchronize()
    assert int(guard.sum()) == 7 * 64
    with pytest.raises(B.PaepError):
        B.probe_read(src, sink[:1024])


def test_mfma_probe_reports_its_flops():
    sink = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    flops = B.probe_mfma(16, 100, sink)
    torch.cuda.synchronize()
    assert flops == 16 * 8 * 100 * 8 * 2 * 32 * 32 * 16
    assert int(sink.sum()) == 0                      # the probe's result is never stored
    with pytest.raises(B.PaepError):
        B.probe_mfma(4096, 1, sink)                  # sink too small for that many workgroups
