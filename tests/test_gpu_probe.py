"""The benchmark's measurement probes run and the copy probe copies (GPU)."""
import pytest
import torch

import paper_1802_09723_amd as rrm

pytestmark = pytest.mark.gpu


def test_probe_copy_copies_every_vector():
    for nbytes in (16, 16 * 1000, 16 * (256 * 32 * 256 * 4 + 777)):
        src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda")
        dst = torch.zeros_like(src)
        rrm.probe_copy(dst, src, nbytes)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)


def test_probe_mfma_runs_and_rejects_bad_counts():
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    rrm.probe_mfma(rrm.I8, sink, 8, 16)
    rrm.probe_mfma(rrm.BF16, sink, 8, 16)
    torch.cuda.synchronize()
    assert int(sink.abs().sum()) == 0
    with pytest.raises(rrm.RRMError):
        rrm.probe_mfma(rrm.I8, sink, 0, 16)
    with pytest.raises(rrm.RRMError):
        rrm.probe_mfma(rrm.BIN, sink, 8, 16)
