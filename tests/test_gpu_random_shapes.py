"""Seeded random configurations of the decode step with token append: head counts, group size, page
size, V layout, budgets, forced recent pages, ragged lengths (short and empty sequences included),
shuffled block tables.  Every case runs a few steps and is checked against the oracle the way the
fixed cases are: both top-k picks within the band, attention on the GPU's own page list, cache and
summaries bit-exact at the end."""
import sys

import numpy as np
import pytest

from paper_2502_14051_amd import workloads as wl
from helpers import assert_attention_close, to_device_cache
from test_gpu_parity import check_selection, small

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2502_14051_amd import rocketkv as rk
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    rk.lib()
    return torch, rk, torch.device("cuda:0")


def draw(seed):
    r = np.random.default_rng(1000 + seed)
    token_major = bool(r.integers(0, 2))
    ps = int(r.choice([1, 2, 3, 4, 5, 8, 16, 32, 64])) if token_major else 16
    G = int(r.choice([1, 2, 3, 4, 6, 8]))
    Hkv = int(r.choice([1, 2, 3, 4]))
    batch = int(r.integers(1, 4))
    ctx = int(r.integers(40, 2600))
    k1 = int(r.choice([1, 8, 32, 33, 64, 100, 128]))
    T = int(r.integers(ps, max(ps + 1, min(ctx, 700))))
    n_recent = int(r.choice([0, 0, 1, 2]))
    steps = int(r.integers(3, 20))
    lens = [ctx] + [int(r.choice([ctx, ctx - 1, max(0, ctx // 3), int(r.integers(0, ctx)), 0]))
                    for _ in range(batch - 1)]
    return dict(token_major=token_major, ps=ps, G=G, Hkv=Hkv, batch=batch, ctx=ctx, k1=k1, T=T,
                n_recent=n_recent, steps=steps, lens=lens, shuffle=bool(r.integers(0, 2)))


@pytest.mark.parametrize("seed", range(48))
def test_random_decode_append(env, oracle, seed):
    torch, rk, dev = env
    p = draw(seed)
    print("[case] random", seed, p, flush=True)
    sys.stdout.flush()
    ps, k1, T, steps, ctx, B = p["ps"], p["k1"], p["T"], p["steps"], p["ctx"], p["batch"]
    w = small("tiny", batch=B, n_q_heads=p["G"] * p["Hkv"], n_kv_heads=p["Hkv"], context=ctx, page_size=ps,
              channel_budget=k1, token_budget=T, n_heavy=4, seed=seed)
    full = wl.generate(wl.scaled(w, context=ctx + steps))
    lens = np.array(p["lens"], dtype=np.int32)
    d0 = dict(full)
    d0["K"] = np.ascontiguousarray(full["K"][:, :, :ctx])
    d0["V"] = np.ascontiguousarray(full["V"][:, :, :ctx])
    d0["seq_lens"] = lens.copy()
    layout = rk.V_TOKEN_MAJOR if p["token_major"] else rk.V_CHANNEL_MAJOR
    rng = np.random.default_rng(seed) if p["shuffle"] else None
    cache, q = to_device_cache(rk, torch, d0, w.n_q_heads, ps, dev, pages_cap=(ctx + steps + ps - 1) // ps,
                               shuffle_rng=rng, v_layout=layout)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    Kref = np.zeros((B, w.n_kv_heads, ctx + steps, 128), dtype=np.uint16)
    Vref = np.zeros_like(Kref)
    for b in range(B):
        Kref[b, :, :lens[b]] = full["K"][b, :, :lens[b]]
        Vref[b, :, :lens[b]] = full["V"][b, :, :lens[b]]
    row = rk.pages_row_len(cache, T)
    out = torch.empty((B, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    pages = torch.empty((B, w.n_kv_heads, row), dtype=torch.int32, device=dev)
    chans = torch.empty((B, w.n_kv_heads, k1), dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, T)
    for s in range(steps):
        kn, vn = full["K"][:, :, ctx + s], full["V"][:, :, ctx + s]
        for b in range(B):
            Kref[b, :, lens[b]] = kn[b]
            Vref[b, :, lens[b]] = vn[b]
        lens += 1
        rk.hsa_decode_append(cache, q, wl.from_bits(kn, dev), wl.from_bits(vn, dev), kmax, kmin, k1, T,
                             p["n_recent"], out, None, pages, chans, ws)
        if s in (0, steps // 2, steps - 1):
            torch.cuda.synchronize()
            assert cache.seq_lens.cpu().numpy().tolist() == lens.tolist()
            ds = dict(q=d0["q"], K=Kref, V=Vref, seq_lens=lens.copy())
            gp, gc = pages.cpu().numpy(), chans.cpu().numpy()
            check_selection(oracle, ds, w, cache.pages_cap, gp, gc, None, p["n_recent"])
            want_y, _ = oracle.attend_given(ds["q"], Kref, Vref, lens, ps, gp)
            assert_attention_close(wl.to_bits(out), want_y, f"seed {seed} step {s}")
    Kg, Vg = rk.unpack_cache(cache)
    Kg, Vg = wl.to_bits(Kg), wl.to_bits(Vg)
    for b in range(B):
        assert np.array_equal(Kg[b, :, :lens[b]], Kref[b, :, :lens[b]])
        assert np.array_equal(Vg[b, :, :lens[b]], Vref[b, :, :lens[b]])
    want_max, want_min = oracle.build_summaries(Kref, lens, ps, cache.pages_cap)
    valid = ~np.isnan(want_max)
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmax))[valid], want_max[valid])
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmin))[valid], want_min[valid])


def draw_snap(seed):
    r = np.random.default_rng(5000 + seed)
    G = int(r.choice([1, 2, 3, 4, 8]))
    W = int(r.choice([w for w in (16, 32, 64, 128) if G * w <= 256]))
    Hkv = int(r.choice([1, 2, 3]))
    batch = int(r.integers(1, 4))
    S = int(r.integers(W + 40, 5200))
    N = int(r.integers(W + 8, max(W + 9, min(S + 200, 1500))))
    ks = int(r.choice([1, 3, 7, 31, 63]))
    lens = [S] + [min(S, int(r.choice([S, S - 1, max(W + 1, S // 2), N, max(1, N - 5), int(r.integers(1, S + 1))])))
                  for _ in range(batch - 1)]
    src_tm, dst_tm = bool(r.integers(0, 2)), bool(r.integers(0, 2))
    dps = int(r.choice([1, 2, 3, 5, 16, 32])) if dst_tm else 16
    return dict(G=G, W=W, Hkv=Hkv, batch=batch, S=S, N=N, ks=ks, lens=lens, src_tm=src_tm, dst_tm=dst_tm,
                dps=dps, shuffle=bool(r.integers(0, 2)))


@pytest.mark.parametrize("seed", range(24))
def test_random_snapkv(env, oracle, seed):
    from helpers import assert_topk_within_band
    from test_gpu_parity import ragged
    torch, rk, dev = env
    p = draw_snap(seed)
    print("[case] random snapkv", seed, p, flush=True)
    sys.stdout.flush()
    S, N, W, B = p["S"], p["N"], p["W"], p["batch"]
    w = small("mistral_snap_128k", batch=B, n_q_heads=p["G"] * p["Hkv"], n_kv_heads=p["Hkv"], context=S,
              snap_keep=N, window=W, n_heavy=6, seed=100 + seed)
    d = ragged(wl.generate(w, with_obs=True), p["lens"])
    rng = np.random.default_rng(seed) if p["shuffle"] else None
    src, _ = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev, shuffle_rng=rng,
                             v_layout=rk.V_TOKEN_MAJOR if p["src_tm"] else rk.V_CHANNEL_MAJOR)
    dps = p["dps"]
    dst = rk.alloc_cache(B, w.n_q_heads, w.n_kv_heads, 128, dps, (N + dps - 1) // dps, dev, zero=True,
                         v_layout=rk.V_TOKEN_MAJOR if p["dst_tm"] else rk.V_CHANNEL_MAJOR)
    kept = torch.full((B, w.n_kv_heads, N), -9, dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_SNAPKV, src, W, N)
    ws.fill_(0xEE)
    rk.workspace_init(ws)
    rk.snapkv_compress(wl.from_bits(d["qobs"], dev), src, W, p["ks"], N, dst, kept, ws)
    torch.cuda.synchronize()
    ref = oracle.snapkv(d["qobs"], d["K"], d["seq_lens"], p["ks"], N, want_votes=True)
    gk = kept.cpu().numpy()
    assert dst.seq_lens.cpu().numpy().tolist() == ref["n_kept"].tolist()
    Kd, Vd = rk.unpack_cache(dst)
    Kd, Vd = wl.to_bits(Kd), wl.to_bits(Vd)
    for b in range(B):
        Sb = int(d["seq_lens"][b])
        cnt = int(ref["n_kept"][b])
        for g in range(w.n_kv_heads):
            row = gk[b, g]
            if Sb <= N:
                assert row[:Sb].tolist() == list(range(Sb)) and (row[Sb:] == -1).all()
            else:
                L = Sb - W
                assert row[N - W:].tolist() == list(range(L, Sb))
                assert_topk_within_band(ref["pooled"][b, g, :L], row[:N - W], N - W, f"kept b{b} g{g}")
            assert np.array_equal(Kd[b, g, :cnt], d["K"][b, g, row[:cnt]])
            assert np.array_equal(Vd[b, g, :cnt], d["V"][b, g, row[:cnt]])


@pytest.mark.parametrize("S,N", [(3000, 512), (20000, 4096), (40000, 4096)])
def test_snapkv_equal_votes_keep_the_lowest_positions(env, oracle, S, N):
    """Every key of the prompt is the same vector: all prefix tokens get exactly the same vote, the
    pooled votes have no finite range to bin, and the tie rule alone decides: the lowest positions
    stay.  (On the GPU this is the top-k's fallback to radix passes with most of a wavefront in one
    counter; the 40000-token prompt goes through the select kernel for long prompts.)"""
    torch, rk, dev = env
    W, ks = 32, 63
    w = small("mistral_snap_128k", batch=1, n_q_heads=8, n_kv_heads=2, context=S, snap_keep=N, window=W,
              n_heavy=0, seed=5)
    print("[case] snapkv equal votes", S, N, flush=True)
    sys.stdout.flush()
    d = wl.generate(w, with_obs=True)
    d["K"][:] = d["K"][:, :, :1, :]  # one key per head, repeated
    src, _ = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev)
    dst = rk.alloc_cache(1, w.n_q_heads, w.n_kv_heads, 128, 16, (N + 15) // 16, dev, zero=True)
    kept = torch.full((1, w.n_kv_heads, N), -9, dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_SNAPKV, src, W, N)
    rk.snapkv_compress(wl.from_bits(d["qobs"], dev), src, W, ks, N, dst, kept, ws)
    torch.cuda.synchronize()
    ref = oracle.snapkv(d["qobs"], d["K"], d["seq_lens"], ks, N)
    want = list(range(N - W)) + list(range(S - W, S))
    for g in range(w.n_kv_heads):
        assert ref["kept"][0, g].tolist() == want
        assert kept[0, g].cpu().numpy().tolist() == want


@pytest.mark.parametrize("token_major,ps", [(False, 16), (True, 16), (True, 4)])
def test_absent_pages_are_skipped(env, oracle, token_major, ps):
    """Block-table entries outside the pool mark absent pages: attention leaves their tokens out (here
    checked as the oracle's attention over the list of the pages that are present), the summary build
    writes neutral zeros for them, and the decode step still runs (its attention equals the oracle's on
    the pages it reports, minus the absent ones)."""
    torch, rk, dev = env
    w = small("tiny", batch=2, n_q_heads=8, n_kv_heads=2, context=900, page_size=ps, token_budget=256, n_heavy=4)
    print("[case] absent pages", token_major, ps, flush=True)
    sys.stdout.flush()
    d = wl.generate(w)
    layout = rk.V_TOKEN_MAJOR if token_major else rk.V_CHANNEL_MAJOR
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, ps, dev, shuffle_rng=np.random.default_rng(3),
                               v_layout=layout)
    P = (w.context + ps - 1) // ps
    rng = np.random.default_rng(17)
    gone = [sorted(rng.choice(P, size=5, replace=False).tolist()) for _ in range(w.batch)]
    bt = cache.block_table.cpu().numpy().copy()
    for b in range(w.batch):
        for i, p in enumerate(gone[b]):
            bt[b, p] = -1 if i % 2 == 0 else int(cache.k_pool.shape[0]) + 7  # below and above the pool
    cache.block_table.copy_(torch.from_numpy(bt).to(dev))
    present = np.full((w.batch, w.n_kv_heads, P), -1, dtype=np.int32)
    for b in range(w.batch):
        keep = [p for p in range(P) if p not in gone[b]]
        present[b, :, :len(keep)] = keep
    # dense decode == attention over the present pages
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((w.batch, w.n_q_heads), dtype=torch.float32, device=dev)
    ws = rk.alloc_workspace(rk.OP_DENSE_DECODE, cache)
    rk.dense_decode(cache, q, out, lse, ws)
    torch.cuda.synchronize()
    want_y, want_lse = oracle.attend_given(d["q"], d["K"], d["V"], d["seq_lens"], ps, present)
    assert_attention_close(wl.to_bits(out), want_y, "dense with absent pages")
    np.testing.assert_allclose(lse.cpu().numpy(), want_lse, rtol=1e-3, atol=1e-3)
    # summaries: zeros in the absent columns, the oracle's values elsewhere
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    torch.cuda.synchronize()
    want_max, want_min = oracle.build_summaries(d["K"], d["seq_lens"], ps, cache.pages_cap)
    gmax, gmin = wl.bf16_bits_to_f64(wl.to_bits(kmax)), wl.bf16_bits_to_f64(wl.to_bits(kmin))
    for b in range(w.batch):
        for p in range(P):
            if p in gone[b]:
                assert (gmax[b, :, :, p] == 0).all() and (gmin[b, :, :, p] == 0).all()
            else:
                assert np.array_equal(gmax[b, :, :, p], want_max[b, :, :, p])
                assert np.array_equal(gmin[b, :, :, p], want_min[b, :, :, p])
    # the decode step: whatever it picks, absent pages contribute nothing
    row = rk.pages_row_len(cache, w.token_budget)
    pages = torch.empty((w.batch, w.n_kv_heads, row), dtype=torch.int32, device=dev)
    wsd = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, w.token_budget)
    rk.hsa_decode(cache, q, kmax, kmin, w.channel_budget, w.token_budget, 0, out, None, pages, None, wsd)
    torch.cuda.synchronize()
    gp = pages.cpu().numpy()
    eff = np.full_like(gp, -1)
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            v = [p for p in gp[b, g] if p >= 0 and p not in gone[b]]
            eff[b, g, :len(v)] = v
    want_y, _ = oracle.attend_given(d["q"], d["K"], d["V"], d["seq_lens"], ps, eff)
    assert_attention_close(wl.to_bits(out), want_y, "decode with absent pages")


@pytest.mark.parametrize("seed", range(12))
def test_random_multi_turn_decode(env, oracle, seed):
    """RocketKV-MT decode over a random index (random subset per (sequence, KV head), random logical
    page size, cache paged independently), a few decode-with-append steps, then the decode checked
    against the oracle on the arrays gathered through the index."""
    from test_gpu_multi_turn import decode_check
    torch, rk, dev = env
    r = np.random.default_rng(9000 + seed)
    lps = int(r.choice([1, 2, 3, 4, 8, 16]))
    cache_ps = int(r.choice([4, 5, 16, 32]))
    G, Hkv, B = int(r.choice([1, 2, 4])), int(r.choice([1, 2, 3])), int(r.integers(1, 4))
    S = int(r.integers(200, 1800))
    k1 = int(r.choice([8, 32, 70, 128]))
    n_idx0 = int(r.integers(20, min(S, 600)))
    T = int(r.integers(lps, max(lps + 1, n_idx0)))
    steps = int(r.integers(2, 9))
    print("[case] random multi-turn", seed, dict(lps=lps, cache_ps=cache_ps, G=G, Hkv=Hkv, B=B, S=S, k1=k1,
                                                 n_idx0=n_idx0, T=T, steps=steps), flush=True)
    sys.stdout.flush()
    w = small("tiny", batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv, context=S + steps, page_size=lps,
              channel_budget=k1, token_budget=T, n_heavy=4, seed=300 + seed)
    full = wl.generate(w)
    lens = np.array([S] + [int(r.integers(n_idx0, S + 1)) for _ in range(B - 1)], dtype=np.int32)
    d0 = dict(q=full["q"], K=np.ascontiguousarray(full["K"][:, :, :S]), V=np.ascontiguousarray(full["V"][:, :, :S]),
              seq_lens=lens.copy())
    cap_tokens = S + steps + 3
    cache, q = to_device_cache(rk, torch, d0, w.n_q_heads, cache_ps, dev,
                               pages_cap=(cap_tokens + cache_ps - 1) // cache_ps,
                               shuffle_rng=np.random.default_rng(seed), v_layout=rk.V_TOKEN_MAJOR)
    index = rk.alloc_index(cache, lps, n_idx0 + steps + 5)
    cap = index.pages_cap * lps
    idx = np.full((B, Hkv, cap), -1, dtype=np.int32)
    n_idx = np.array([n_idx0] + [int(r.integers(0, n_idx0 + 1)) for _ in range(B - 1)], dtype=np.int32)
    for b in range(B):
        for g in range(Hkv):
            idx[b, g, :n_idx[b]] = np.sort(r.choice(int(lens[b]), size=n_idx[b], replace=False))
    index.token_index.copy_(torch.from_numpy(idx).to(dev))
    index.n_indexed.copy_(torch.from_numpy(n_idx).to(dev))
    kmax, kmin = rk.alloc_index_summaries(cache, index)
    rk.mt_build_page_summaries(cache, index, kmax, kmin)
    ws = rk.mt_alloc_workspace(cache, index, T)
    Kfull = np.zeros((B, Hkv, cache.pages_cap * cache_ps, 128), dtype=np.uint16)
    Vfull = np.zeros_like(Kfull)
    for b in range(B):
        Kfull[b, :, :lens[b]] = full["K"][b, :, :lens[b]]
        Vfull[b, :, :lens[b]] = full["V"][b, :, :lens[b]]
    objs = (cache, index, kmax, kmin, ws)
    wlog = wl.scaled(w, page_size=lps)
    decode_check(env, oracle, objs, wlog, full["q"], Kfull, Vfull, n_recent=int(r.integers(0, 2)))
    out = torch.empty((B, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    lens_now = lens.copy()
    for s in range(steps):
        kn, vn = full["K"][:, :, S + s], full["V"][:, :, S + s]
        for b in range(B):
            Kfull[b, :, lens_now[b]] = kn[b]
            Vfull[b, :, lens_now[b]] = vn[b]
        rk.mt_hsa_decode_append(cache, index, q, wl.from_bits(kn, dev), wl.from_bits(vn, dev), kmax, kmin, k1, T,
                                1, out, None, None, None, ws)
        lens_now += 1
    torch.cuda.synchronize()
    assert cache.seq_lens.cpu().numpy().tolist() == lens_now.tolist()
    assert index.n_indexed.cpu().numpy().tolist() == (n_idx + steps).tolist()
    Kc, nl = decode_check(env, oracle, objs, wlog, full["q"], Kfull, Vfull, n_recent=1)
    want_max, want_min = oracle.build_summaries(Kc, nl.astype(np.int32), lps, index.pages_cap)
    valid = ~np.isnan(want_max)
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmax))[valid], want_max[valid])
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmin))[valid], want_min[valid])
