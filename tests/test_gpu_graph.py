"""The decode step replayed from a captured HIP graph (the way bench.py issues it) against the same
step launched eagerly on a twin cache: every replay must give the eager result bit for bit, with the
program's own eager work and synchronisations in between."""
import sys

import numpy as np
import pytest

from paper_2502_14051_amd import workloads as wl
from helpers import to_device_cache
from test_gpu_parity import small

pytestmark = pytest.mark.gpu
TM = 1


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2502_14051_amd import rocketkv as rk
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    rk.lib()
    return torch, rk, torch.device("cuda:0")


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


CASES = [
    # name, page size, channels, token budget, context, V layout, multi-turn index
    ("fused channel-major", 16, 32, 256, 3000, 0, False),
    ("fused token-major", 4, 40, 200, 1500, TM, False),
    ("score/pick/attention launches", 2, 128, 96, 1100, TM, False),
    ("fused multi-turn", 16, 32, 128, 2000, TM, True),
]


@pytest.mark.parametrize("name,ps,k1,T,ctx,layout,mt", CASES)
def test_graph_replay_equals_eager(env, name, ps, k1, T, ctx, layout, mt):
    torch, rk, dev = env
    steps = 6
    say("graph replay", name)
    w = small("tiny", batch=2, context=ctx, page_size=ps, channel_budget=k1, token_budget=T, n_heavy=6)
    d = wl.generate(w, with_obs=mt)
    d["seq_lens"] = np.array([ctx, ctx - 61], dtype=np.int32)
    Hq, Hkv = w.n_q_heads, w.n_kv_heads

    def make():
        cps = 16 if mt else ps
        cache, _ = to_device_cache(rk, torch, d, Hq, cps, dev, pages_cap=(ctx + steps + 8 + cps - 1) // cps,
                                   shuffle_rng=np.random.default_rng(3), v_layout=layout)
        if mt:
            N = 512
            index = rk.alloc_index(cache, ps, N + steps + 8)
            ws_s = rk.alloc_workspace(rk.OP_SNAPKV, cache, 32, N)
            rk.snapkv_filter(wl.from_bits(d["qobs"], dev), cache, 32, 63, N, index, ws_s)
            kmax, kmin = rk.alloc_index_summaries(cache, index)
            rk.mt_build_page_summaries(cache, index, kmax, kmin)
            ws = rk.mt_alloc_workspace(cache, index, T)
            row = min(index.pages_cap, (T + ps - 1) // ps)
        else:
            index = None
            kmax, kmin = rk.alloc_summaries(cache)
            rk.build_page_summaries(cache, kmax, kmin)
            ws = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, T)
            row = rk.pages_row_len(cache, T)
        out = torch.zeros((2, Hq, 128), dtype=torch.bfloat16, device=dev)
        pages = torch.zeros((2, Hkv, row), dtype=torch.int32, device=dev)
        return dict(cache=cache, index=index, kmax=kmax, kmin=kmin, ws=ws, out=out, pages=pages)

    A, B = make(), make()
    q = torch.zeros((2, Hq, 128), dtype=torch.bfloat16, device=dev)
    kn = torch.zeros((2, Hkv, 128), dtype=torch.bfloat16, device=dev)
    vn = torch.zeros((2, Hkv, 128), dtype=torch.bfloat16, device=dev)

    def step(S, stream):
        if mt:
            rk.mt_hsa_decode_append(S["cache"], S["index"], q, kn, vn, S["kmax"], S["kmin"], k1, T, 1, S["out"], None,
                                    S["pages"], None, S["ws"], stream)
        else:
            rk.hsa_decode_append(S["cache"], q, kn, vn, S["kmax"], S["kmin"], k1, T, 1, S["out"], None, S["pages"],
                                 None, S["ws"], stream)

    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(A, side)
    torch.cuda.synchronize()
    # capture does not execute: both twins are still at their initial lengths
    assert torch.equal(A["cache"].seq_lens, B["cache"].seq_lens)
    rng = np.random.default_rng(17)
    for s in range(steps):
        q.copy_(wl.from_bits(wl.f32_to_bf16_bits(rng.standard_normal((2, Hq, 128)).astype(np.float32)), dev))
        kn.copy_(wl.from_bits(wl.f32_to_bf16_bits(rng.standard_normal((2, Hkv, 128)).astype(np.float32)), dev))
        vn.copy_(wl.from_bits(wl.f32_to_bf16_bits(rng.standard_normal((2, Hkv, 128)).astype(np.float32)), dev))
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        side.synchronize()
        step(B, None)  # eager, on the current stream
        torch.cuda.synchronize()
        assert torch.equal(A["out"], B["out"]), f"replay {s}: outputs differ"
        assert torch.equal(A["pages"], B["pages"]), f"replay {s}: page lists differ"
        assert torch.equal(A["cache"].seq_lens, B["cache"].seq_lens)
        assert A["cache"].seq_lens.cpu().numpy().tolist() == [ctx + s + 1, ctx - 61 + s + 1]
        if mt:
            assert torch.equal(A["index"].n_indexed, B["index"].n_indexed)
    assert torch.equal(A["cache"].k_pool, B["cache"].k_pool) and torch.equal(A["cache"].v_pool, B["cache"].v_pool)
    assert torch.equal(A["kmax"], B["kmax"]) and torch.equal(A["kmin"], B["kmin"])
    if mt:
        assert torch.equal(A["index"].token_index, B["index"].token_index)


def test_long_decode_256_graph_replays(env, oracle):
    """The long-decode configuration (a cache of 8192 kept tokens, budget 2048, 256 generated tokens)
    driven by one captured step replayed 256 times: every replay equals the eager step on a twin
    cache, pages are crossed 16 times, and the end state agrees with the oracle."""
    from helpers import assert_attention_close
    from test_gpu_parity import check_selection
    torch, rk, dev = env
    steps, n0, T, k1 = 256, 8192, 2048, 32
    w = small("mistral_snap_128k", context=n0 + steps, token_budget=T, channel_budget=k1, n_heavy=32)
    say("256 graph replays", w.name, n0, T)
    full = wl.generate(w)
    Hq, Hkv = w.n_q_heads, w.n_kv_heads
    d0 = dict(q=full["q"], K=np.ascontiguousarray(full["K"][:, :, :n0]), V=np.ascontiguousarray(full["V"][:, :, :n0]),
              seq_lens=np.array([n0], dtype=np.int32))

    def make():
        cache, _ = to_device_cache(rk, torch, d0, Hq, 16, dev, pages_cap=(n0 + steps) // 16 + 1,
                                   shuffle_rng=np.random.default_rng(5))
        kmax, kmin = rk.alloc_summaries(cache)
        rk.build_page_summaries(cache, kmax, kmin)
        row = rk.pages_row_len(cache, T)
        return dict(cache=cache, kmax=kmax, kmin=kmin, ws=rk.alloc_workspace(rk.OP_HSA_DECODE, cache, T),
                    out=torch.zeros((1, Hq, 128), dtype=torch.bfloat16, device=dev),
                    pages=torch.zeros((1, Hkv, row), dtype=torch.int32, device=dev))

    A, B = make(), make()
    q = wl.from_bits(full["q"], dev)
    kn = torch.zeros((1, Hkv, 128), dtype=torch.bfloat16, device=dev)
    vn = torch.zeros((1, Hkv, 128), dtype=torch.bfloat16, device=dev)

    def step(S, stream):
        rk.hsa_decode_append(S["cache"], q, kn, vn, S["kmax"], S["kmin"], k1, T, 1, S["out"], None, S["pages"],
                             None, S["ws"], stream)

    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(A, side)
    torch.cuda.synchronize()
    Kall, Vall = wl.from_bits(full["K"], dev), wl.from_bits(full["V"], dev)
    for s in range(steps):
        kn.copy_(Kall[:, :, n0 + s])
        vn.copy_(Vall[:, :, n0 + s])
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        side.synchronize()
        step(B, None)
        torch.cuda.synchronize()
        assert torch.equal(A["out"], B["out"]), f"replay {s}: outputs differ"
        assert torch.equal(A["pages"], B["pages"]), f"replay {s}: page lists differ"
    assert A["cache"].seq_lens.cpu().numpy().tolist() == [n0 + steps]
    assert torch.equal(A["cache"].k_pool, B["cache"].k_pool) and torch.equal(A["cache"].v_pool, B["cache"].v_pool)
    assert torch.equal(A["kmax"], B["kmax"]) and torch.equal(A["kmin"], B["kmin"])
    # the end state against the oracle
    lens = np.array([n0 + steps], dtype=np.int32)
    want_max, want_min = oracle.build_summaries(full["K"], lens, 16, A["cache"].pages_cap)
    valid = ~np.isnan(want_max)
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(A["kmax"]))[valid], want_max[valid])
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(A["kmin"]))[valid], want_min[valid])
    ds = dict(q=full["q"], K=full["K"], V=full["V"], seq_lens=lens)
    gp = A["pages"].cpu().numpy()
    check_selection(oracle, ds, wl.scaled(w, context=n0 + steps), A["cache"].pages_cap, gp, None, None, 1)
    want_y, _ = oracle.attend_given(full["q"], full["K"], full["V"], lens, 16, gp)
    assert_attention_close(wl.to_bits(A["out"]), want_y, "last replay")


@pytest.mark.parametrize("S,N", [(3000, 512), (40000, 1024)])
def test_snapkv_graph_replays(env, S, N):
    """The SnapKV stage captured once and replayed: every replay over changed inputs must equal the eager
    call on the same inputs, bit for bit.  The 40000-token prompt takes the select of several launches,
    whose histograms in the workspace are cleared by a kernel (a captured memset would not do)."""
    torch, rk, dev = env
    W = 32
    w = small("mistral_snap_128k", batch=2, n_q_heads=4, n_kv_heads=2, context=S, snap_keep=N, window=W, n_heavy=8)
    say("snapkv graph", S, N)
    d = wl.generate(w, with_obs=True)
    src, _ = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev)
    qobs = wl.from_bits(d["qobs"], dev)
    P = (N + 15) // 16

    def fresh():
        return (rk.alloc_cache(w.batch, w.n_q_heads, w.n_kv_heads, 128, 16, P, dev, zero=True),
                torch.full((w.batch, w.n_kv_heads, N), -7, dtype=torch.int32, device=dev),
                rk.alloc_workspace(rk.OP_SNAPKV, src, W, N))

    dst_g, kept_g, ws_g = fresh()
    dst_e, kept_e, ws_e = fresh()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        rk.snapkv_compress(qobs, src, W, 63, N, dst_g, kept_g, ws_g, stream)  # warm
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            rk.snapkv_compress(qobs, src, W, 63, N, dst_g, kept_g, ws_g, stream)
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    for rep in range(3):
        # new queries in place: the captured launches read the same buffers
        qobs.copy_((torch.randn(qobs.shape, generator=gen, device=dev) * (1.0 + rep)).to(torch.bfloat16))
        kept_g.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        rk.snapkv_compress(qobs, src, W, 63, N, dst_e, kept_e, ws_e)
        torch.cuda.synchronize()
        assert torch.equal(kept_g, kept_e), f"replay {rep}: kept indices differ"
        assert torch.equal(dst_g.k_pool, dst_e.k_pool) and torch.equal(dst_g.v_pool, dst_e.v_pool), f"replay {rep}"
        assert torch.equal(dst_g.seq_lens, dst_e.seq_lens)
        assert int((kept_g >= 0).sum()) == w.batch * w.n_kv_heads * N
