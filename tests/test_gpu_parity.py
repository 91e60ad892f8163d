"""GPU parity: every C-ABI entry point against the fp64 CPU oracle on the same seeded inputs.

Bar: summaries and indices bit-exact (indices up to the 1e-3 band around the selection threshold),
attention within 1e-2 absolute/relative.  Each test prints its case before touching the GPU.
"""
import sys

import numpy as np
import pytest

from paper_2502_14051_amd import workloads as wl
from helpers import (assert_attention_close, assert_topk_within_band, to_device_cache)

pytestmark = pytest.mark.gpu


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


def small(name="tiny", **kw):
    return wl.scaled(wl.CONFIGS[name], **kw)


def ragged(d, lens):
    d = dict(d)
    d["seq_lens"] = np.asarray(lens, dtype=np.int32)
    return d


# ------------------------------------------------------------------ Step 1
@pytest.mark.parametrize("ctx,lens,ps,shuffle", [
    (4096, None, 16, False),
    (1000, (1000, 37), 16, True),      # ragged tail pages, permuted physical pages
    (333, (333, 1), 3, False),         # the paper's own small page sizes
    (130, (130, 129), 1, True),
    (4100, (4100, 4099), 64, False),
])
def test_page_summaries_exact(env, oracle, ctx, lens, ps, shuffle):
    torch, rk, dev = env
    B = 1 if lens is None else len(lens)
    w = small(batch=B, context=ctx, page_size=ps)
    say("summaries", w.name, ctx, lens, ps, shuffle)
    d = wl.generate(w)
    if lens is not None:
        d = ragged(d, lens)
    rng = np.random.default_rng(1) if shuffle else None
    cache, _ = to_device_cache(rk, torch, d, w.n_q_heads, ps, dev, shuffle_rng=rng, extra_pages=5)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    torch.cuda.synchronize()
    want_max, want_min = oracle.build_summaries(d["K"], d["seq_lens"], ps, cache.pages_cap)
    got_max = wl.bf16_bits_to_f64(wl.to_bits(kmax))
    got_min = wl.bf16_bits_to_f64(wl.to_bits(kmin))
    valid = ~np.isnan(want_max)
    assert valid.any()
    assert np.array_equal(got_max[valid], want_max[valid])
    assert np.array_equal(got_min[valid], want_min[valid])
    assert (got_max[~valid] == 0).all()  # untouched columns keep their initial zeros


def test_page_summaries_partial_range(env, oracle):
    torch, rk, dev = env
    w = small(context=2048)
    say("summaries range", w.name)
    d = wl.generate(w)
    cache, _ = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin, first_page=70, n_pages=3)
    torch.cuda.synchronize()
    want_max, _ = oracle.build_summaries(d["K"], d["seq_lens"], 16, cache.pages_cap)
    got = wl.bf16_bits_to_f64(wl.to_bits(kmax))
    assert np.array_equal(got[..., 70:73], want_max[..., 70:73])
    assert (got[..., :70] == 0).all() and (got[..., 73:] == 0).all()


# ------------------------------------------------------------------ Step 2
def check_selection(oracle, d, w, cache_pages_cap, got_pages, got_chans, got_scores, n_recent=0):
    B, Hkv, G, D = w.batch, w.n_kv_heads, w.group, w.head_dim
    ps, k1, T = w.page_size, w.channel_budget, w.token_budget
    ref = oracle.hsa_decode(d["q"], d["K"], d["V"], d["seq_lens"], ps, k1, T, n_recent, want_scores=True)
    exact_sets = 0
    for b in range(B):
        n = int(d["seq_lens"][b])
        P = (n + ps - 1) // ps
        kp = oracle.pages_to_pick(n, ps, T)
        for g in range(Hkv):
            a, s, _ = oracle.channel_select(d["q"][b, g * G:(g + 1) * G], k1)
            if got_chans is not None:
                assert_topk_within_band(a, got_chans[b, g], k1, f"channels b{b} g{g}")
            same_ch = got_chans is None or np.array_equal(got_chans[b, g], ref["chans"][b, g])
            if P == 0:
                assert (got_pages[b, g] == -1).all()
                continue
            # scores the GPU's own channel pick implies, from the oracle's arithmetic
            if got_chans is not None and not same_ch:
                kmax, kmin = oracle.page_summaries(d["K"][b, g, :n], ps)
                sc = oracle.page_scores(s, got_chans[b, g], kmax, kmin)
            else:
                sc = ref["scores"][b, g, :P].copy()
            if got_scores is not None:
                np.testing.assert_allclose(got_scores[b, g, :P], sc, rtol=2e-5,
                                           atol=2e-5 * np.abs(sc).max())
            forced = min(n_recent, kp)
            if forced:
                sc[P - forced:] = np.inf
            assert_topk_within_band(sc, got_pages[b, g], kp, f"pages b{b} g{g}")
            exact_sets += int(np.array_equal(got_pages[b, g, :kp], ref["pages"][b, g, :kp]))
    return ref, exact_sets


SELECT_CASES = [
    # name, overrides, lens, n_recent, shuffle
    ("tiny", {}, None, 0, False),
    ("tiny", dict(token_budget=1024, channel_budget=128), None, 0, False),       # all channels (Quest-like)
    ("tiny", dict(batch=3, context=1500, token_budget=160), (1500, 17, 0), 1, True),
    ("tiny", dict(context=700, page_size=3, channel_budget=70, token_budget=60), None, 0, False),
    ("tiny", dict(context=300, page_size=1, channel_budget=128, token_budget=40), None, 0, False),  # Exact-TopK
    ("llama8b_layer_32k", dict(token_budget=256), None, 0, False),               # P = 2048
    ("llama8b_layer_32k", dict(token_budget=4096, context=32000), None, 2, True),
    ("llama70b_step_b16", dict(batch=2, context=4096, n_layers=1), None, 0, False),  # G = 8
]


@pytest.mark.parametrize("name,over,lens,n_recent,shuffle", SELECT_CASES)
def test_hsa_select(env, oracle, name, over, lens, n_recent, shuffle):
    torch, rk, dev = env
    w = small(name, **over)
    say("select", name, over, lens, n_recent, shuffle)
    d = wl.generate(w)
    if lens is not None:
        d = ragged(d, lens)
    rng = np.random.default_rng(2) if shuffle else None
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, w.page_size, dev, shuffle_rng=rng)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    row = rk.pages_row_len(cache, w.token_budget)
    pages = torch.full((w.batch, w.n_kv_heads, row), -7, dtype=torch.int32, device=dev)
    chans = torch.full((w.batch, w.n_kv_heads, w.channel_budget), -7, dtype=torch.int32, device=dev)
    scores = torch.zeros((w.batch, w.n_kv_heads, cache.pages_cap), dtype=torch.float32, device=dev)
    rk.hsa_select(cache, q, kmax, kmin, w.channel_budget, w.token_budget, n_recent, pages, chans, scores)
    torch.cuda.synchronize()
    p1 = pages.cpu().numpy()
    check_selection(oracle, d, w, cache.pages_cap, p1, chans.cpu().numpy(), scores.cpu().numpy(), n_recent)
    # bit-reproducible
    pages2 = torch.empty_like(pages)
    rk.hsa_select(cache, q, kmax, kmin, w.channel_budget, w.token_budget, n_recent, pages2, None, None)
    torch.cuda.synchronize()
    assert np.array_equal(p1, pages2.cpu().numpy())


def test_select_breaks_ties_towards_lower_index(env, oracle):
    """All keys equal: every page scores the same, so the first kp pages must be picked; all |q|
    equal: the first k1 channels must be picked."""
    torch, rk, dev = env
    say("select ties")
    B, Hkv, G, D, n, ps = 1, 2, 4, 128, 640, 16
    one = wl.f32_to_bf16_bits(np.ones((B, Hkv, n, D), dtype=np.float32))
    d = dict(q=wl.f32_to_bf16_bits(np.ones((B, Hkv * G, D), dtype=np.float32)), K=one, V=one,
             seq_lens=np.array([n], dtype=np.int32))
    cache, q = to_device_cache(rk, torch, d, Hkv * G, ps, dev)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    pages = torch.empty((B, Hkv, 10), dtype=torch.int32, device=dev)
    chans = torch.empty((B, Hkv, 5), dtype=torch.int32, device=dev)
    rk.hsa_select(cache, q, kmax, kmin, 5, 160, 0, pages, chans, None)
    torch.cuda.synchronize()
    assert pages.cpu().numpy()[0, 0].tolist() == list(range(10))
    assert chans.cpu().numpy()[0, 1].tolist() == list(range(5))
    ref = oracle.hsa_decode(d["q"], d["K"], d["V"], d["seq_lens"], ps, 5, 160)
    assert np.array_equal(ref["pages"][:, :, :10], pages.cpu().numpy())


@pytest.mark.parametrize("P,T", [(300, 640), (1000, 1600), (1500, 640), (2600, 1024)])
def test_pick_with_crowded_threshold(env, oracle, P, T):
    """Most pages score exactly the same and the threshold falls among them (far more ties than the
    exact-rank step of the register selection takes on, so it hands over to the radix passes), a few
    pages score higher, a few lower: the higher ones and the lowest-indexed ties must come out, in the
    fused kernel's own selection, for page counts on each of its paths."""
    torch, rk, dev = env
    say("crowded threshold", P, T)
    B, Hkv, G, D, ps = 1, 2, 2, 128, 16
    n = P * ps - 3
    rng = np.random.default_rng(P)
    level = np.ones(P, dtype=np.float32)
    special = rng.choice(P, size=24, replace=False)
    level[special[:12]] = 2.0
    level[special[12:]] = 0.5
    K = np.repeat(level, ps)[:n][None, None, :, None] * np.ones((B, Hkv, 1, D), dtype=np.float32)
    d = dict(q=wl.f32_to_bf16_bits(np.ones((B, Hkv * G, D), dtype=np.float32)), K=wl.f32_to_bf16_bits(K),
             V=wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, n, D)).astype(np.float32)),
             seq_lens=np.array([n], dtype=np.int32))
    cache, q = to_device_cache(rk, torch, d, Hkv * G, ps, dev)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    row = rk.pages_row_len(cache, T)
    out = torch.empty((B, Hkv * G, D), dtype=torch.bfloat16, device=dev)
    pages = torch.empty((B, Hkv, row), dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, T)
    rk.hsa_decode(cache, q, kmax, kmin, 32, T, 0, out, None, pages, None, ws)
    torch.cuda.synchronize()
    kp = T // ps
    big = np.sort(special[:12])
    ties = np.array([p for p in range(P) if level[p] == 1.0])[:kp - 12]
    want = np.sort(np.concatenate([big, ties]))
    got = pages.cpu().numpy()
    for g in range(Hkv):
        assert got[0, g, :kp].tolist() == want.tolist()
    ref = oracle.hsa_decode(d["q"], d["K"], d["V"], d["seq_lens"], ps, 32, T)
    assert np.array_equal(ref["pages"][:, :, :kp], got[:, :, :kp])
    want_y, _ = oracle.attend_given(d["q"], d["K"], d["V"], d["seq_lens"], ps, got)
    assert_attention_close(wl.to_bits(out), want_y, "y, crowded threshold")


# ------------------------------------------------------------------ Step 3 and the dense baseline
ATTEND_CASES = [
    ("tiny", dict(n_heavy=0), None, False),                      # diffuse softmax
    ("tiny", dict(heavy_nats=2.0), None, False),
    ("tiny", dict(batch=3, context=1000, n_heavy=0), (1000, 999, 5), True),
    ("tiny", dict(n_q_heads=4, n_kv_heads=4, context=777, n_heavy=3), None, False),      # MHA, G = 1
    ("tiny", dict(n_q_heads=32, n_kv_heads=2, context=2048, heavy_nats=1.0), None, True),  # G = 16
    ("llama70b_step_b16", dict(batch=2, context=3000, n_layers=1, n_heavy=0), None, False),  # G = 8
    ("tiny", dict(n_q_heads=12, n_kv_heads=2, context=1111, n_heavy=3), None, True),          # G = 6
    ("tiny", dict(batch=33, n_q_heads=32, n_kv_heads=8, context=700, n_heavy=2), None, False),  # 264 units
]


@pytest.mark.parametrize("name,over,lens,shuffle", ATTEND_CASES)
def test_dense_decode(env, oracle, name, over, lens, shuffle):
    torch, rk, dev = env
    w = small(name, **over)
    say("dense", name, over, lens, shuffle)
    d = wl.generate(w)
    if lens is not None:
        d = ragged(d, lens)
    rng = np.random.default_rng(3) if shuffle else None
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev, shuffle_rng=rng, extra_pages=3)
    out = torch.full((w.batch, w.n_q_heads, 128), 7.0, dtype=torch.bfloat16, device=dev)
    lse = torch.zeros((w.batch, w.n_q_heads), dtype=torch.float32, device=dev)
    ws = rk.alloc_workspace(rk.OP_DENSE_DECODE, cache)
    ws.fill_(0xAB)  # whatever the allocation held; initialised once below
    rk.workspace_init(ws)
    rk.dense_decode(cache, q, out, lse, ws)
    torch.cuda.synchronize()
    want_y, want_lse = oracle.dense_decode(d["q"], d["K"], d["V"], d["seq_lens"])
    assert_attention_close(wl.to_bits(out), want_y, "dense y")
    np.testing.assert_allclose(lse.cpu().numpy(), want_lse, rtol=1e-3, atol=1e-3)
    # second call on the same workspace (self-resetting counters) gives the same bits
    out2 = torch.empty_like(out)
    rk.dense_decode(cache, q, out2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("name,over,lens,shuffle", ATTEND_CASES)
def test_attend_on_given_pages(env, oracle, name, over, lens, shuffle):
    torch, rk, dev = env
    w = small(name, **over)
    say("attend", name, over, lens, shuffle)
    d = wl.generate(w)
    if lens is not None:
        d = ragged(d, lens)
    rng = np.random.default_rng(4)
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev, shuffle_rng=rng if shuffle else None)
    row = 21  # odd length: exercises the unpaired last entry
    pages = np.full((w.batch, w.n_kv_heads, row), -1, dtype=np.int32)
    for b in range(w.batch):
        P = (int(d["seq_lens"][b]) + 15) // 16
        for g in range(w.n_kv_heads):
            if P == 0:
                continue
            k = min(P, int(rng.integers(1, row + 1)))
            pick = set(rng.choice(P, size=k, replace=False).tolist())
            if g % 2 == 0:
                pick.add(P - 1)  # make sure partial tail pages are hit
                if len(pick) > min(P, row):
                    pick.discard(min(pick))
            lst = sorted(pick)
            if g % 3 == 1 and len(lst) < row:
                lst.insert(len(lst) // 2, -1)  # holes are skipped, not terminators
            pages[b, g, :len(lst)] = lst
    pt = torch.from_numpy(pages).to(dev)
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((w.batch, w.n_q_heads), dtype=torch.float32, device=dev)
    ws = rk.alloc_workspace(rk.OP_ATTEND, cache, row)
    rk.attend(cache, q, pt, out, lse, ws)
    torch.cuda.synchronize()
    # the oracle stops a row at the first -1: compact valid entries to the front for it
    comp = np.full_like(pages, -1)
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            v = pages[b, g][pages[b, g] >= 0]
            comp[b, g, :len(v)] = v
    want_y, want_lse = oracle.attend_given(d["q"], d["K"], d["V"], d["seq_lens"], 16, comp)
    assert_attention_close(wl.to_bits(out), want_y, "attend y")
    got_lse = lse.cpu().numpy()
    fin = np.isfinite(want_lse)
    np.testing.assert_allclose(got_lse[fin], want_lse[fin], rtol=1e-3, atol=1e-3)
    assert np.isneginf(got_lse[~fin]).all()


# ------------------------------------------------------------------ Algorithm 1 end to end
DECODE_CASES = [
    ("tiny", {}, None, 0, False),
    ("tiny", dict(n_heavy=0), None, 0, True),
    ("tiny", dict(token_budget=8192), None, 0, False),                      # budget >= context: dense
    ("tiny", dict(batch=4, context=1500, token_budget=200, heavy_nats=2.0), (1500, 1499, 16, 0), 1, True),
    ("llama8b_layer_32k", dict(token_budget=256), None, 0, False),
    ("llama8b_layer_32k", dict(token_budget=1024, heavy_nats=2.0), None, 0, False),
    ("llama8b_layer_32k", dict(token_budget=4096, context=32767), None, 0, True),
    ("llama8b_step_b16", dict(batch=4, context=4096, n_layers=1), None, 0, False),   # compacted shape of the bench
    ("llama70b_step_b16", dict(batch=2, context=4096, n_layers=1, heavy_nats=2.0), None, 0, False),
    ("mistral_snap_128k", dict(context=8448), None, 1, False),                 # decode shape after SnapKV + 256 steps
    ("tiny", dict(batch=2, n_q_heads=12, n_kv_heads=2, context=2222, token_budget=300), None, 0, True),   # G = 6
    ("tiny", dict(batch=2, n_q_heads=21, n_kv_heads=3, context=1500, token_budget=128), None, 1, False),  # G = 7
    ("tiny", dict(n_q_heads=8, n_kv_heads=2, context=140000, token_budget=2048, n_heavy=32), None, 0, False),  # > 8192 pages
    # the largest cache the selection takes: 32768 pages, a ragged last page
    ("tiny", dict(n_q_heads=2, n_kv_heads=1, context=32768 * 16 - 5, token_budget=4096, n_heavy=32), None, 1, False),
    # more (sequence, KV head) units than compute units: the four-wavefront launch geometry
    ("tiny", dict(batch=40, n_q_heads=32, n_kv_heads=8, context=1100, token_budget=512, n_heavy=4), None, 0, True),
    # the page counts at which the selection changes its form, on either side of each step: two and five
    # pages per thread in registers, then scores through LDS (512-thread workgroups: 1024 / 2560 pages) ...
    ("tiny", dict(n_q_heads=4, n_kv_heads=2, context=1024 * 16, token_budget=1024, n_heavy=16), None, 0, False),
    ("tiny", dict(n_q_heads=4, n_kv_heads=2, context=1025 * 16 - 3, token_budget=1024, n_heavy=16), None, 1, True),
    ("tiny", dict(n_q_heads=4, n_kv_heads=2, context=2560 * 16, token_budget=1024, n_heavy=16), None, 0, True),
    ("tiny", dict(n_q_heads=4, n_kv_heads=2, context=2561 * 16 - 9, token_budget=1024, n_heavy=16), None, 2, False),
    ("tiny", dict(n_q_heads=4, n_kv_heads=2, context=8192 * 16, token_budget=2048, n_heavy=16), None, 0, False),
    # ... and the same steps for the 256-thread workgroups of launches with more than 256 units
    # (512 / 1280 pages; `tile`: the host generator draws a third of the batch and the rest are copies,
    # which keeps it to seconds at 264 units)
    ("tiny", dict(batch=33, tile=11, n_q_heads=8, n_kv_heads=8, context=512 * 16, token_budget=512, n_heavy=4), None, 0, False),
    ("tiny", dict(batch=33, tile=11, n_q_heads=8, n_kv_heads=8, context=513 * 16 - 1, token_budget=512, n_heavy=4), None, 1, False),
    ("tiny", dict(batch=33, tile=11, n_q_heads=8, n_kv_heads=8, context=1280 * 16, token_budget=512, n_heavy=4), None, 0, False),
    ("tiny", dict(batch=33, tile=11, n_q_heads=8, n_kv_heads=8, context=1281 * 16 - 7, token_budget=512, n_heavy=4), None, 0, False),
]


@pytest.mark.parametrize("name,over,lens,n_recent,shuffle", DECODE_CASES)
def test_hsa_decode(env, oracle, name, over, lens, n_recent, shuffle):
    torch, rk, dev = env
    over = dict(over)
    tile = over.pop("tile", 1)
    w = small(name, **over)
    say("decode", name, over, lens, n_recent, shuffle, "tile", tile)
    if tile > 1:
        d = wl.generate(wl.scaled(w, batch=w.batch // tile))
        d = {k: (np.concatenate([v] * tile, axis=0) if isinstance(v, np.ndarray) and v.ndim >= 1 and
                 v.shape[0] == w.batch // tile else v) for k, v in d.items()}
    else:
        d = wl.generate(w)
    if lens is not None:
        d = ragged(d, lens)
    rng = np.random.default_rng(5) if shuffle else None
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev, shuffle_rng=rng)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    row = rk.pages_row_len(cache, w.token_budget)
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((w.batch, w.n_q_heads), dtype=torch.float32, device=dev)
    pages = torch.empty((w.batch, w.n_kv_heads, row), dtype=torch.int32, device=dev)
    chans = torch.empty((w.batch, w.n_kv_heads, w.channel_budget), dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, w.token_budget)
    ws.fill_(0xCD)
    rk.workspace_init(ws)
    rk.hsa_decode(cache, q, kmax, kmin, w.channel_budget, w.token_budget, n_recent, out, lse, pages,
                  chans, ws)
    torch.cuda.synchronize()
    gp, gc = pages.cpu().numpy(), chans.cpu().numpy()
    ref, exact = check_selection(oracle, d, w, cache.pages_cap, gp, gc, None, n_recent)
    # (i) Step 3 re-evaluated by the oracle on the GPU's own page list
    want_y, want_lse = oracle.attend_given(d["q"], d["K"], d["V"], d["seq_lens"], 16, gp)
    assert_attention_close(wl.to_bits(out), want_y, "y on GPU list")
    fin = np.isfinite(want_lse)
    np.testing.assert_allclose(lse.cpu().numpy()[fin], want_lse[fin], rtol=1e-3, atol=1e-3)
    # (ii) end to end wherever the lists agree (always, unless a threshold tie fell in the band)
    same = (gp == ref["pages"][:, :, :row]).all(axis=-1)
    assert same.mean() > 0.9
    got = wl.bf16_bits_to_f64(wl.to_bits(out)).reshape(w.batch, w.n_kv_heads, w.group, 128)
    want = ref["y"].reshape(w.batch, w.n_kv_heads, w.group, 128)
    assert (np.abs(got - want)[same] <= 1e-2 + 1e-2 * np.abs(want[same])).all()
    # empty sequences give zeros and -inf
    for b in range(w.batch):
        if d["seq_lens"][b] == 0:
            assert (got[b] == 0).all() and np.isneginf(lse.cpu().numpy()[b]).all()


def test_budget_covering_context_equals_dense_bits(env):
    """Token budget >= context picks every page: the result is the dense kernel's, bit for bit."""
    torch, rk, dev = env
    w = small("tiny", context=2000, token_budget=2000, n_heavy=0)
    say("decode==dense", w.name)
    d = wl.generate(w)
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    out = torch.empty((1, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    out_d = torch.empty_like(out)
    ws = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, w.token_budget)
    rk.hsa_decode(cache, q, kmax, kmin, 32, w.token_budget, 0, out, None, None, None, ws)
    wsd = rk.alloc_workspace(rk.OP_DENSE_DECODE, cache)
    rk.dense_decode(cache, q, out_d, None, wsd)
    torch.cuda.synchronize()
    a = wl.bf16_bits_to_f64(wl.to_bits(out))
    b = wl.bf16_bits_to_f64(wl.to_bits(out_d))
    assert np.abs(a - b).max() <= 2e-3  # same math, possibly different split points


# ------------------------------------------------------------------ append (summaries follow new keys)
def test_append_keeps_cache_and_summaries_current(env, oracle):
    torch, rk, dev = env
    w = small("tiny", batch=2, context=100, n_heavy=0)
    steps = 40
    say("append", w.name, steps)
    full = wl.generate(wl.scaled(w, context=100 + steps))
    d0 = dict(full)
    d0["K"] = np.ascontiguousarray(full["K"][:, :, :100])
    d0["V"] = np.ascontiguousarray(full["V"][:, :, :100])
    lens0 = np.array([100, 83], dtype=np.int32)
    d0["seq_lens"] = lens0
    cache, q = to_device_cache(rk, torch, d0, w.n_q_heads, 16, dev, pages_cap=16,
                               shuffle_rng=np.random.default_rng(6))
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    Kref = np.zeros((2, w.n_kv_heads, 100 + steps, 128), dtype=np.uint16)
    Vref = np.zeros_like(Kref)
    for b in range(2):
        Kref[b, :, :lens0[b]] = full["K"][b, :, :lens0[b]]
        Vref[b, :, :lens0[b]] = full["V"][b, :, :lens0[b]]
    lens = lens0.copy()
    for s in range(steps):
        kn = full["K"][:, :, 100 + s]
        vn = full["V"][:, :, 100 + s]
        for b in range(2):
            Kref[b, :, lens[b]] = kn[b]
            Vref[b, :, lens[b]] = vn[b]
        rk.append_kv(cache, wl.from_bits(kn, dev), wl.from_bits(vn, dev), kmax, kmin)
        lens += 1
    torch.cuda.synchronize()
    assert cache.seq_lens.cpu().numpy().tolist() == lens.tolist()
    Kg, Vg = rk.unpack_cache(cache)
    Kg, Vg = wl.to_bits(Kg), wl.to_bits(Vg)
    for b in range(2):
        assert np.array_equal(Kg[b, :, :lens[b]], Kref[b, :, :lens[b]])
        assert np.array_equal(Vg[b, :, :lens[b]], Vref[b, :, :lens[b]])
    want_max, want_min = oracle.build_summaries(Kref, lens, 16, cache.pages_cap)
    valid = ~np.isnan(want_max)
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmax))[valid], want_max[valid])
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmin))[valid], want_min[valid])
    # a full sequence is left alone
    cache.seq_lens.fill_(cache.pages_cap * 16)
    rk.append_kv(cache, wl.from_bits(kn, dev), wl.from_bits(vn, dev), kmax, kmin)
    torch.cuda.synchronize()
    assert (cache.seq_lens.cpu().numpy() == cache.pages_cap * 16).all()


# ------------------------------------------------------------------ Stage 1
SNAP_CASES = [
    # name, overrides, lens, pool kernel, shuffle
    ("mistral_snap_128k", dict(context=4096, snap_keep=1024, n_heavy=16), None, 63, False),
    ("mistral_snap_128k", dict(batch=3, context=3000, snap_keep=512, n_heavy=8), (3000, 2999, 400), 63, True),
    ("mistral_snap_128k", dict(context=2500, snap_keep=300, n_heavy=0, n_q_heads=8, n_kv_heads=8), None, 7, False),
    ("mistral_snap_128k", dict(context=2000, snap_keep=256, n_heavy=4), None, 1, False),
    ("llama70b_step_b16", dict(batch=1, context=2048, snap_keep=512, n_layers=1, n_heavy=8), None, 63, False),
    ("mistral_snap_128k", dict(context=1536, snap_keep=640, window=128, n_heavy=8,
                               n_q_heads=4, n_kv_heads=2), None, 63, False),  # multi-turn window size
    # a prompt beyond 32768 tokens: the radix-select kernel instead of the register-resident top-k
    ("mistral_snap_128k", dict(context=40000, snap_keep=2048, n_heavy=16, n_q_heads=4, n_kv_heads=2), None, 63, False),
    # the same kernel on ragged lengths (a row that ends inside a 16-byte group, a prompt below the keep budget)
    ("mistral_snap_128k", dict(batch=3, context=50003, snap_keep=1000, n_heavy=12, n_q_heads=2, n_kv_heads=1),
     (50003, 33001, 700), 31, True),
    # the longest prompt a source cache can hold (32768 pages), ending inside a page
    ("mistral_snap_128k", dict(context=32768 * 16 - 3, snap_keep=2048, n_heavy=16, n_q_heads=1, n_kv_heads=1),
     None, 63, False),
    # more than 64 units of such prompts: one workgroup per unit and a single launch (fewer units take
    # several workgroups per unit over several launches, as in the two cases above)
    ("mistral_snap_128k", dict(batch=13, context=33000, snap_keep=512, window=16, n_heavy=6, n_q_heads=5, n_kv_heads=5),
     None, 15, False),
]


@pytest.mark.parametrize("name,over,lens,ks,shuffle", SNAP_CASES)
def test_snapkv_compress(env, oracle, name, over, lens, ks, shuffle):
    torch, rk, dev = env
    w = small(name, **over)
    say("snapkv", name, over, lens, ks, shuffle)
    d = wl.generate(w, with_obs=True)
    if lens is not None:
        d = ragged(d, lens)
    N, W = w.snap_keep, w.window
    rng = np.random.default_rng(7) if shuffle else None
    src, _ = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev, shuffle_rng=rng)
    dst = rk.alloc_cache(w.batch, w.n_q_heads, w.n_kv_heads, 128, 16, (N + 15) // 16, dev, zero=True)
    kept = torch.full((w.batch, w.n_kv_heads, N), -9, dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_SNAPKV, src, W, N)
    ws.fill_(0xEE)
    rk.workspace_init(ws)
    rk.snapkv_compress(wl.from_bits(d["qobs"], dev), src, W, ks, N, dst, kept, ws)
    torch.cuda.synchronize()
    ref = oracle.snapkv(d["qobs"], d["K"], d["seq_lens"], ks, N, want_votes=True)
    gk = kept.cpu().numpy()
    assert dst.seq_lens.cpu().numpy().tolist() == ref["n_kept"].tolist()
    Kd, Vd = rk.unpack_cache(dst)
    Kd, Vd = wl.to_bits(Kd), wl.to_bits(Vd)
    n_same = 0
    for b in range(w.batch):
        S = int(d["seq_lens"][b])
        cnt = int(ref["n_kept"][b])
        for g in range(w.n_kv_heads):
            row = gk[b, g]
            if S <= N:
                assert row[:S].tolist() == list(range(S)) and (row[S:] == -1).all()
            else:
                L = S - W
                assert row[N - W:].tolist() == list(range(L, S))
                assert_topk_within_band(ref["pooled"][b, g, :L], row[:N - W], N - W, f"kept b{b} g{g}")
            n_same += int(np.array_equal(row, ref["kept"][b, g]))
            # the destination cache holds exactly the rows the GPU said it kept, in that order
            assert np.array_equal(Kd[b, g, :cnt], d["K"][b, g, row[:cnt]])
            assert np.array_equal(Vd[b, g, :cnt], d["V"][b, g, row[:cnt]])
    assert n_same >= 0.8 * w.batch * w.n_kv_heads


def test_snapkv_then_decode_pipeline(env, oracle):
    """Stage 1 then stage 2 on the compacted cache, as the method runs them (Section 3.2)."""
    torch, rk, dev = env
    w = small("llama8b_step_b16", batch=2, context=4096, snap_keep=1024, token_budget=256, n_layers=1,
              n_heavy=16)
    say("pipeline", w.name)
    d = wl.generate(w, with_obs=True)
    src, q = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev)
    dst = rk.alloc_cache(w.batch, w.n_q_heads, w.n_kv_heads, 128, 16, w.snap_keep // 16, dev, zero=True)
    kept = torch.empty((w.batch, w.n_kv_heads, w.snap_keep), dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_SNAPKV, src, w.window, w.snap_keep)
    rk.snapkv_compress(wl.from_bits(d["qobs"], dev), src, w.window, w.pool_kernel, w.snap_keep, dst, kept, ws)
    kmax, kmin = rk.alloc_summaries(dst)
    rk.build_page_summaries(dst, kmax, kmin)
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    pages = torch.empty((w.batch, w.n_kv_heads, 16), dtype=torch.int32, device=dev)
    ws2 = rk.alloc_workspace(rk.OP_HSA_DECODE, dst, w.token_budget)
    rk.hsa_decode(dst, q, kmax, kmin, 32, w.token_budget, 0, out, None, pages, None, ws2)
    torch.cuda.synchronize()
    gk = kept.cpu().numpy()
    Kc = np.stack([np.stack([d["K"][b, g, gk[b, g]] for g in range(w.n_kv_heads)]) for b in range(w.batch)])
    Vc = np.stack([np.stack([d["V"][b, g, gk[b, g]] for g in range(w.n_kv_heads)]) for b in range(w.batch)])
    dc = dict(q=d["q"], K=Kc, V=Vc, seq_lens=np.full(w.batch, w.snap_keep, dtype=np.int32))
    wc = wl.scaled(w, context=w.snap_keep)
    check_selection(oracle, dc, wc, dst.pages_cap, pages.cpu().numpy(), None, None)
    want_y, _ = oracle.attend_given(dc["q"], Kc, Vc, dc["seq_lens"], 16, pages.cpu().numpy())
    assert_attention_close(wl.to_bits(out), want_y, "pipeline y")
    # planted tokens survive both stages: HSA over the compacted cache matches dense over the prompt
    yd, _ = oracle.dense_decode(d["q"], d["K"], d["V"], d["seq_lens"])
    assert np.median(np.abs(wl.bf16_bits_to_f64(wl.to_bits(out)) - yd)) < 2e-2


# ------------------------------------------------------------------ decode step with the new token folded in
@pytest.mark.parametrize("name,over,lens0,shuffle", [
    ("tiny", dict(batch=3, context=300, token_budget=96, heavy_nats=2.0), (250, 239, 0), True),
    ("llama8b_step_b16", dict(batch=2, context=4200, n_layers=1, token_budget=1024), (4090, 4096), False),
    ("llama70b_step_b16", dict(batch=1, context=600, n_layers=1, token_budget=128, n_heavy=4), (555,), False),
    # the receiving page in the second round of the two-round register selection, crossing a page boundary
    ("tiny", dict(batch=2, context=700 * 16 + 40, token_budget=512, n_heavy=8), (700 * 16 - 10, 520 * 16 + 3), False),
    # five rounds: receiving pages in rounds 2 and 4
    ("tiny", dict(batch=2, context=2100 * 16 + 40, token_budget=512, n_heavy=8), (1500 * 16 - 10, 2100 * 16 - 3), True),
    # scores through LDS (more than 2560 pages)
    ("tiny", dict(batch=2, context=3000 * 16 + 40, token_budget=512, n_heavy=8), (3000 * 16 - 10, 2600 * 16), False),
    # more than 256 units: the four-wavefront kernel, which takes the receiving page's old bounds from the
    # page's own rows; every slot of a page and both sides of a page boundary, with and without a block table
    ("tiny", dict(batch=33, n_q_heads=8, n_kv_heads=8, context=420, token_budget=128, n_heavy=2),
     tuple(300 + (7 * i) % 61 for i in range(33)), False),
    ("tiny", dict(batch=33, n_q_heads=16, n_kv_heads=8, context=420, token_budget=96, n_heavy=2),
     tuple([0, 1, 15, 16, 17] + [200 + (11 * i) % 97 for i in range(28)]), True),
])
def test_decode_append_equals_append_then_decode(env, oracle, name, over, lens0, shuffle):
    """rocketkv_hsa_decode_append must leave everything exactly as rocketkv_append_kv followed by
    rocketkv_hsa_decode does, step after step, across page boundaries; and both must match the oracle
    on the grown cache."""
    torch, rk, dev = env
    w = small(name, **over)
    steps = 20
    say("decode+append", name, over, lens0, shuffle)
    full = wl.generate(w)
    lens0 = np.asarray(lens0, dtype=np.int32)
    B, Hkv = w.batch, w.n_kv_heads
    cap = int(lens0.max()) + steps + 5
    base = dict(full)
    base["seq_lens"] = lens0

    def fresh():
        c, q = to_device_cache(rk, torch, base, w.n_q_heads, 16, dev, pages_cap=(cap + 15) // 16,
                               shuffle_rng=np.random.default_rng(8) if shuffle else None)
        kx, kn = rk.alloc_summaries(c)
        rk.build_page_summaries(c, kx, kn)
        return c, q, kx, kn

    A, q, Akx, Akn = fresh()
    Bc, _, Bkx, Bkn = fresh()
    row = rk.pages_row_len(A, w.token_budget)
    wsA = rk.alloc_workspace(rk.OP_HSA_DECODE, A, w.token_budget)
    wsB = rk.alloc_workspace(rk.OP_HSA_DECODE, Bc, w.token_budget)
    outA = torch.empty((B, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    outB = torch.empty_like(outA)
    pgA = torch.empty((B, Hkv, row), dtype=torch.int32, device=dev)
    pgB = torch.empty_like(pgA)
    rng = np.random.default_rng(9)
    Kref = full["K"].copy()
    Vref = full["V"].copy()
    Kref = np.concatenate([Kref, np.zeros((B, Hkv, cap, 128), dtype=np.uint16)], axis=2)
    Vref = np.concatenate([Vref, np.zeros((B, Hkv, cap, 128), dtype=np.uint16)], axis=2)
    lens = lens0.copy()
    for s in range(steps):
        kn_new = wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, 128)).astype(np.float32) * 1.5)
        vn_new = wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, 128)).astype(np.float32))
        for b in range(B):
            Kref[b, :, lens[b]] = kn_new[b]
            Vref[b, :, lens[b]] = vn_new[b]
        lens += 1
        kt, vt = wl.from_bits(kn_new, dev), wl.from_bits(vn_new, dev)
        rk.hsa_decode_append(A, q, kt, vt, Akx, Akn, w.channel_budget, w.token_budget, 1, outA, None, pgA,
                             None, wsA)
        rk.append_kv(Bc, kt, vt, Bkx, Bkn)
        rk.hsa_decode(Bc, q, Bkx, Bkn, w.channel_budget, w.token_budget, 1, outB, None, pgB, None, wsB)
        torch.cuda.synchronize()
        assert A.seq_lens.cpu().numpy().tolist() == lens.tolist(), f"step {s}"
        assert torch.equal(pgA, pgB), f"step {s}: page lists differ"
        assert torch.equal(outA, outB), f"step {s}: outputs differ"
    assert torch.equal(Akx, Bkx) and torch.equal(Akn, Bkn)
    KA, VA = rk.unpack_cache(A)
    KB, VB = rk.unpack_cache(Bc)
    KA, VA, KB, VB = (wl.to_bits(t) for t in (KA, VA, KB, VB))
    for b in range(B):
        assert np.array_equal(KA[b, :, :lens[b]], Kref[b, :, :lens[b]])
        assert np.array_equal(VA[b, :, :lens[b]], Vref[b, :, :lens[b]])
        assert np.array_equal(KB[b, :, :lens[b]], Kref[b, :, :lens[b]])
    # oracle on the grown cache
    nmax = int(lens.max())
    d = dict(q=full["q"], K=np.ascontiguousarray(Kref[:, :, :nmax]), V=np.ascontiguousarray(Vref[:, :, :nmax]),
             seq_lens=lens)
    gp = pgA.cpu().numpy()
    check_selection(oracle, d, w, A.pages_cap, gp, None, None, n_recent=1)
    want_y, _ = oracle.attend_given(d["q"], d["K"], d["V"], lens, 16, gp)
    assert_attention_close(wl.to_bits(outA), want_y, "decode+append y")
    want_max, want_min = oracle.build_summaries(d["K"], lens, 16, A.pages_cap)
    valid = ~np.isnan(want_max)
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(Akx))[valid], want_max[valid])
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(Akn))[valid], want_min[valid])
