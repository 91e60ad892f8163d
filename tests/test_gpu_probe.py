"""The measurement aids read exactly what they claim to.  The streaming read touches every word once:
the XOR of the per-wavefront checksums it leaves equals the XOR of the buffer, at sizes that do and do
not fill its unrolled loop.  The gather probe reads the K and V tiles of the listed pages, once each:
its checksums XOR to that of those tiles (a page listed twice cancels; absent entries add nothing)."""
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


@pytest.mark.parametrize("B,Hkv,pages,row", [(2, 2, 40, 9), (16, 8, 264, 64), (1, 8, 2056, 64), (40, 8, 264, 64)])
def test_stream_gather_checksum(B, Hkv, pages, row):
    import torch
    from paper_2502_14051_amd import rocketkv as rk
    print("[case] stream_gather", B, Hkv, pages, row, flush=True)
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(B * 1000 + row)
    cache = rk.alloc_cache(B, Hkv * 4, Hkv, 128, 16, pages, dev, zero=True)
    cache.k_pool.view(torch.int16).random_(-30000, 30000, generator=g)
    cache.v_pool.view(torch.int16).random_(-30000, 30000, generator=g)
    rng = np.random.default_rng(B + row)
    lst = np.full((B, Hkv, row), -1, dtype=np.int32)
    for b in range(B):
        for h in range(Hkv):
            k = rng.integers(0, row + 1)
            lst[b, h, :k] = np.sort(rng.choice(cache.pages_cap, size=k, replace=False))
    pg = torch.from_numpy(lst).to(dev)
    sink = rk.stream_gather(cache, pg)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    kp = cache.k_pool.view(torch.int32).cpu().numpy().view(np.uint32)   # [pages][Hkv][16][64]
    vp = cache.v_pool.view(torch.int32).cpu().numpy().view(np.uint32)
    want = np.uint32(0)
    for b in range(B):
        for h in range(Hkv):
            for p_ in lst[b, h]:
                if p_ >= 0:
                    pp = b * cache.pages_cap + p_
                    want ^= np.bitwise_xor.reduce(kp[pp, h].ravel()) ^ np.bitwise_xor.reduce(vp[pp, h].ravel())
    assert got == want
