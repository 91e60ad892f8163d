"""The entry point that allocates nothing (`rocketkv_hsa_decode_noalloc`) against `rocketkv_hsa_decode`.

Both run the same kernels with the same launch plan, one on the caller's workspace, the other on the
library's built-in scratch buffer, so the outputs must agree bit for bit (and either is within the
build target's tolerance of the fp64 oracle, which the other GPU tests establish for
rocketkv_hsa_decode).  Two calls in a row share the buffer, the second on a smaller input: whatever
the first left behind must not leak into it.  A shape whose scratch need exceeds the buffer is refused.
"""
import numpy as np
import pytest

from paper_2502_14051_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _case(rk, torch, dev, seed, B, Hkv, G, n, T, k1, n_recent, cap_extra=8):
    w = wl.scaled(wl.CONFIGS["tiny"], batch=B, n_kv_heads=Hkv, n_q_heads=Hkv * G, context=n, token_budget=T,
                  channel_budget=k1, seed=seed)
    d = wl.generate(w)
    lens = np.array([max(1, n - 7 * b) for b in range(B)], dtype=np.int32)  # ragged
    ps = w.page_size
    cap = ((n + ps - 1) // ps + cap_extra + 7) // 8 * 8
    cache = rk.pack_cache(wl.from_bits(d["K"], dev), wl.from_bits(d["V"], dev), lens, w.n_q_heads, ps, pages_cap=cap)
    q = wl.from_bits(d["q"], dev)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    row = rk.pages_row_len(cache, T)

    def outputs():
        return (torch.zeros((B, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev),
                torch.zeros((B, w.n_q_heads), dtype=torch.float32, device=dev),
                torch.full((B, Hkv, row), -7, dtype=torch.int32, device=dev),
                torch.full((B, Hkv, k1), -7, dtype=torch.int32, device=dev))

    ws = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, T)
    want = outputs()
    rk.hsa_decode(cache, q, kmax, kmin, k1, T, n_recent, *want, ws)
    got = outputs()
    rk.hsa_decode_noalloc(cache, q, kmax, kmin, k1, T, n_recent, *got)
    torch.cuda.synchronize()
    for name, a, b in zip(("out", "lse", "pages", "channels"), got, want):
        if a.dtype == torch.bfloat16:
            a, b = a.view(torch.int16), b.view(torch.int16)
        assert torch.equal(a, b), f"{name} differs between the built-in scratch and a caller's workspace"
    return got


def test_noalloc_matches_workspace_call_twice_in_a_row():
    import torch
    from paper_2502_14051_amd import rocketkv as rk

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    # first call: several units, a list split over workgroups (partials and counters in the scratch)
    _case(rk, torch, dev, seed=5, B=3, Hkv=4, G=4, n=2100, T=1024, k1=32, n_recent=1)
    # second call, smaller in every dimension, on the same buffer
    _case(rk, torch, dev, seed=6, B=1, Hkv=2, G=4, n=300, T=64, k1=16, n_recent=0)
    # and the first shape again: the smaller call must have left the buffer usable too
    _case(rk, torch, dev, seed=7, B=3, Hkv=4, G=4, n=2100, T=1024, k1=32, n_recent=1)


def test_noalloc_refuses_a_shape_beyond_its_buffer():
    import torch
    from paper_2502_14051_amd import rocketkv as rk

    dev = torch.device("cuda:0")
    # 1024 units x 1032 pages: the page scores of the multi-launch path alone exceed the buffer.  The
    # call must be refused on the host before anything is launched, so a few physical pages behind an
    # all-zero block table and token summaries of a few bytes stand in for the real buffers.
    B, Hq, Hkv, D, ps, cap = 128, 32, 8, 128, 16, 1032
    bt = torch.zeros((B, cap), dtype=torch.int32, device=dev)
    cache = rk.alloc_cache(B, Hq, Hkv, D, ps, cap, dev, block_table=bt, n_phys_pages=8, zero=True)
    assert rk.workspace_bytes(rk.OP_HSA_DECODE, cache, 1024) > rk.NOALLOC_SCRATCH_BYTES
    q = torch.zeros((B, Hq, D), dtype=torch.bfloat16, device=dev)
    dummy = torch.zeros((64,), dtype=torch.bfloat16, device=dev)
    out = torch.zeros((B, Hq, D), dtype=torch.bfloat16, device=dev)
    with pytest.raises(rk.RocketKVError) as e:
        rk.hsa_decode_noalloc(cache, q, dummy, dummy, 32, 1024, 0, out, None, None, None)
    assert e.value.status == -2 and "scratch" in str(e.value)
    torch.cuda.synchronize()
