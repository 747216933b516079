"""The AND + popcount rate probe: runs, writes its sink, refuses bad arguments."""
import pytest
import torch

import paper_1709_04060_amd as bs

pytestmark = pytest.mark.gpu


def test_probe_runs_and_writes_sink():
    sink = torch.full((8,), -1, dtype=torch.int32, device="cuda")
    ops = bs.bs_probe_popcount_rate(sink, 8)
    torch.cuda.synchronize()
    assert ops == 8 * 256 * 8 * 32
    # every workgroup stored the XOR of its first lane's 16 counters: each counter is a sum of
    # popcounts of 32-bit words over 8 / 4 * 4 updates, so the XOR is small and non-negative
    h = sink.cpu()
    assert (h >= 0).all() and (h < 32 * 8 * 2).all()


def test_probe_rejects_bad_arguments():
    sink = torch.zeros((4,), dtype=torch.int32, device="cuda")
    for passes in (0, -4, 6):
        with pytest.raises(bs.BsError) as e:
            bs.bs_probe_popcount_rate(sink, passes)
        assert e.value.status == bs.BS_ERR_INVALID_ARG
