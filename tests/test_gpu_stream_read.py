"""The read-only bandwidth yardstick: its XOR of the buffer's 64-bit words proves every word was read once."""
import numpy as np
import pytest
import torch

from paper_2504_03702_amd import binding as ps

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_words", [2, 254, 4096, 1_000_002, 6_291_458])
def test_xor_of_all_words(n_words):
    rng = np.random.default_rng(n_words)
    host = rng.integers(-(1 << 62), 1 << 62, n_words, dtype=np.int64)
    data = torch.from_numpy(host).to("cuda:0")
    sink = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    ps.ps_profile_stream_read(data, sink)
    assert int(sink.cpu()[0]) == int(np.bitwise_xor.reduce(host))
    ps.ps_profile_stream_read(data, sink)            # accumulated into: the second pass cancels the first
    assert int(sink.cpu()[0]) == 0
    # a prefix only
    ps.ps_profile_stream_read(data, sink, nbytes=16 * (n_words // 4))
    assert int(sink.cpu()[0]) == int(np.bitwise_xor.reduce(host[:2 * (n_words // 4)])) if n_words >= 4 else True


def test_rejects_unaligned_sizes_and_pointers():
    data = torch.zeros(64, dtype=torch.int64, device="cuda:0")
    sink = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    with pytest.raises(ps.PsError):
        ps.ps_profile_stream_read(data, sink, nbytes=24)
    with pytest.raises(ps.PsError):
        ps.ps_profile_stream_read(data[1:], sink, nbytes=16)
    ps.ps_profile_stream_read(data, sink, nbytes=0)
    assert int(sink.cpu()[0]) == 0
