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


@pytest.mark.parametrize("nt", [False, True])
def test_stream_read_probe_reads_every_byte_once(nt):
    """The XOR of the workgroups' words equals the XOR of all 32-bit words of the buffer (ragged last slice)."""
    n = (5 * 16384 + 16 * 37) // 4
    g = torch.Generator(device="cpu").manual_seed(7)
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (n,), dtype=torch.int32, generator=g)
    sink = torch.zeros((3,), dtype=torch.int32, device="cuda")
    assert bs.bs_probe_stream_read(src.cuda(), sink, non_temporal=nt) == 4 * n
    torch.cuda.synchronize()
    import numpy as np
    want = int(np.bitwise_xor.reduce(src.numpy().view(np.uint32)))
    got = int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)))
    assert got == want
