"""The streaming-read measurement aid reads every word exactly once: the XOR of the per-wavefront
checksums it leaves equals the XOR of the buffer, at sizes that do and do not fill its unrolled loop."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_words", [4, 4 * 1000, 4 * (256 * 4096 * 8) + 4 * 12345, 4 * 3_000_001])
def test_stream_read_checksum(n_words):
    import torch
    from paper_2502_14051_amd import rocketkv as rk
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    print("[case] stream_read", n_words, flush=True)
    sys.stdout.flush()
    rng = np.random.default_rng(n_words)
    host = rng.integers(0, 2**32, size=n_words, dtype=np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).to("cuda:0")
    sink = rk.stream_read(buf)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert got == np.bitwise_xor.reduce(host)


def test_stream_read_rejects_ragged_size():
    import torch
    from paper_2502_14051_amd import rocketkv as rk
    buf = torch.zeros(6, dtype=torch.int32, device="cuda:0")  # 24 bytes: not a multiple of 16
    with pytest.raises(rk.RocketKVError):
        rk.stream_read(buf)
