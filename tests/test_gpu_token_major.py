"""GPU parity for caches with token-major V tiles at any page size: the operating points the
adaptive decomposition of Section 3.6 yields (pages of 2-4 tokens, 60-76 channels), the Exact-TopK
setting of Section 4.1 (pages of one token, every channel) and the Quest-like setting (every
channel, pages of 16), all through the same entry points and against the same fp64 oracle.
"""
import sys

import numpy as np
import pytest

from paper_2502_14051_amd import workloads as wl
from helpers import assert_attention_close, assert_topk_within_band, to_device_cache
from test_gpu_parity import check_selection, ragged, small

pytestmark = pytest.mark.gpu
TM = 1  # ROCKETKV_V_TOKEN_MAJOR


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


DENSE_TM = [
    # page size, overrides, lens, shuffle
    (1, dict(context=300, n_heavy=2), None, False),
    (2, dict(batch=2, context=1001, n_heavy=0), (1001, 64), True),
    (3, dict(batch=3, context=1000), (1000, 999, 5), True),
    (4, dict(n_q_heads=4, n_kv_heads=4, context=777, n_heavy=3), None, False),         # G = 1
    (5, dict(n_q_heads=32, n_kv_heads=2, context=2048, heavy_nats=1.0), None, False),  # G = 16
    (16, dict(batch=2, context=4100), (4100, 0), False),
    (33, dict(context=3000, n_heavy=0), None, True),
    (64, dict(context=2100), None, False),
]


@pytest.mark.parametrize("ps,over,lens,shuffle", DENSE_TM)
def test_dense_decode_token_major(env, oracle, ps, over, lens, shuffle):
    torch, rk, dev = env
    w = small("tiny", page_size=ps, **over)
    say("dense token-major", ps, over, lens, shuffle)
    d = wl.generate(w)
    if lens is not None:
        d = ragged(d, lens)
    rng = np.random.default_rng(30 + ps) if shuffle else None
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, ps, dev, shuffle_rng=rng, extra_pages=3, v_layout=TM)
    out = torch.full((w.batch, w.n_q_heads, 128), 7.0, dtype=torch.bfloat16, device=dev)
    lse = torch.zeros((w.batch, w.n_q_heads), dtype=torch.float32, device=dev)
    ws = rk.alloc_workspace(rk.OP_DENSE_DECODE, cache)
    ws.fill_(0xAB)
    rk.workspace_init(ws)
    rk.dense_decode(cache, q, out, lse, ws)
    torch.cuda.synchronize()
    want_y, want_lse = oracle.dense_decode(d["q"], d["K"], d["V"], d["seq_lens"])
    assert_attention_close(wl.to_bits(out), want_y, "dense y")
    fin = np.isfinite(want_lse)
    np.testing.assert_allclose(lse.cpu().numpy()[fin], want_lse[fin], rtol=1e-3, atol=1e-3)
    assert np.isneginf(lse.cpu().numpy()[~fin]).all()
    out2 = torch.empty_like(out)
    rk.dense_decode(cache, q, out2, None, ws)  # workspace left ready by the first call
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("ps,row", [(1, 37), (3, 21), (4, 50), (16, 9), (7, 64)])
def test_attend_on_given_pages_token_major(env, oracle, ps, row):
    torch, rk, dev = env
    w = small("tiny", batch=3, context=900, page_size=ps, n_heavy=4)
    say("attend token-major", ps, row)
    d = ragged(wl.generate(w), (900, 899, 10))
    rng = np.random.default_rng(40 + ps)
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, ps, dev, shuffle_rng=rng, v_layout=TM)
    pages = np.full((w.batch, w.n_kv_heads, row), -1, dtype=np.int32)
    for b in range(w.batch):
        P = (int(d["seq_lens"][b]) + ps - 1) // ps
        for g in range(w.n_kv_heads):
            k = min(P, int(rng.integers(1, row + 1)))
            pick = set(rng.choice(P, size=k, replace=False).tolist())
            if g % 2 == 0:
                pick.add(P - 1)  # the partial tail page
                if len(pick) > min(P, row):
                    pick.discard(min(pick))
            lst = sorted(pick)
            if g % 3 == 1 and len(lst) < row:
                lst.insert(len(lst) // 2, -1)  # a hole is skipped, it does not end the row
            pages[b, g, :len(lst)] = lst
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((w.batch, w.n_q_heads), dtype=torch.float32, device=dev)
    ws = rk.alloc_workspace(rk.OP_ATTEND, cache, row)
    rk.attend(cache, q, torch.from_numpy(pages).to(dev), out, lse, ws)
    torch.cuda.synchronize()
    comp = np.full_like(pages, -1)
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            v = pages[b, g][pages[b, g] >= 0]
            comp[b, g, :len(v)] = v
    want_y, want_lse = oracle.attend_given(d["q"], d["K"], d["V"], d["seq_lens"], ps, comp)
    assert_attention_close(wl.to_bits(out), want_y, "attend y")
    np.testing.assert_allclose(lse.cpu().numpy(), want_lse, rtol=1e-3, atol=1e-3)


def decode_and_check(env, oracle, w, d, n_recent, shuffle_seed, v_layout=TM):
    torch, rk, dev = env
    ps = w.page_size
    rng = np.random.default_rng(shuffle_seed) if shuffle_seed else None
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, ps, dev, shuffle_rng=rng, v_layout=v_layout)
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
    rk.hsa_decode(cache, q, kmax, kmin, w.channel_budget, w.token_budget, n_recent, out, lse, pages, chans, ws)
    torch.cuda.synchronize()
    gp, gc = pages.cpu().numpy(), chans.cpu().numpy()
    ref, _ = check_selection(oracle, d, w, cache.pages_cap, gp, gc, None, n_recent)
    want_y, want_lse = oracle.attend_given(d["q"], d["K"], d["V"], d["seq_lens"], ps, gp)
    assert_attention_close(wl.to_bits(out), want_y, "y on GPU list")
    fin = np.isfinite(want_lse)
    np.testing.assert_allclose(lse.cpu().numpy()[fin], want_lse[fin], rtol=1e-3, atol=1e-3)
    width = min(row, ref["pages"].shape[-1])  # the oracle's rows are as long as its longest pick
    assert (gp[:, :, width:] == -1).all()
    same = (gp[:, :, :width] == ref["pages"][:, :, :width]).all(axis=-1)
    assert same.mean() > 0.9
    got = wl.bf16_bits_to_f64(wl.to_bits(out)).reshape(w.batch, w.n_kv_heads, w.group, 128)
    want = ref["y"].reshape(w.batch, w.n_kv_heads, w.group, 128)
    assert (np.abs(got - want)[same] <= 1e-2 + 1e-2 * np.abs(want[same])).all()
    return out, gp


def test_decode_at_the_decomposed_operating_point(env, oracle):
    """Section 3.6 end to end: the split of a 64x compression decides keep budget, page size,
    channel count and attended tokens; Stage 2 then runs at exactly that point."""
    torch, rk, dev = env
    S, t = 32768, 512
    sp = rk.decompose(S, t, 128)
    assert sp["page_size"] == 3  # the worked example of the section
    w = small("llama8b_step_b16", batch=2, n_layers=1, context=sp["keep_budget"], page_size=sp["page_size"],
              channel_budget=sp["channel_budget"], token_budget=sp["attend_tokens"], n_heavy=12)
    say("decode at decomposed point", sp)
    decode_and_check(env, oracle, w, wl.generate(w), 0, 51)


DECODE_TM = [
    # page size, channels, token budget, overrides, lens, n_recent
    (1, 128, 64, dict(context=600, n_heavy=6), None, 0),                                   # Exact-TopK
    (16, 128, 256, dict(context=4096, n_heavy=8), None, 0),                                # Quest-like
    (2, 60, 128, dict(batch=3, context=1500, heavy_nats=2.0), (1500, 1499, 1), 1),
    (4, 72, 200, dict(n_q_heads=8, n_kv_heads=8, context=2000), None, 2),                  # MHA
    (3, 76, 8192, dict(context=700), None, 0),                                             # budget covers all
    (8, 32, 512, dict(n_q_heads=64, n_kv_heads=8, context=3000, n_heavy=0), None, 0),      # G = 8
    (5, 48, 200, dict(batch=2, n_q_heads=12, n_kv_heads=4, context=1700), None, 0),        # G = 3
    (1, 4, 4000, dict(context=8000, n_heavy=20), None, 0),   # list too long for LDS: separate launches
    (1, 16, 500, dict(context=12000, n_heavy=10), None, 0),  # more than 8192 pages: scores through the workspace
]


@pytest.mark.parametrize("ps,k1,T,over,lens,n_recent", DECODE_TM)
def test_hsa_decode_token_major(env, oracle, ps, k1, T, over, lens, n_recent):
    w = small("tiny", page_size=ps, channel_budget=k1, token_budget=T, **over)
    say("decode token-major", ps, k1, T, over, lens, n_recent)
    d = wl.generate(w)
    if lens is not None:
        d = ragged(d, lens)
    decode_and_check(env, oracle, w, d, n_recent, 60 + ps)


def test_layouts_agree_at_page_16(env, oracle):
    """The same cache in both V layouts: same selection, results within rounding of each other."""
    torch, rk, dev = env
    w = small("llama8b_step_b16", batch=2, n_layers=1, context=4096, n_heavy=8)
    say("layouts agree", w.name)
    d = wl.generate(w)
    out_c, pg_c = decode_and_check(env, oracle, w, d, 0, 0, v_layout=0)
    out_t, pg_t = decode_and_check(env, oracle, w, d, 0, 0, v_layout=TM)
    assert np.array_equal(pg_c, pg_t)
    a, b = wl.bf16_bits_to_f64(wl.to_bits(out_c)), wl.bf16_bits_to_f64(wl.to_bits(out_t))
    assert np.abs(a - b).max() <= 4e-3


@pytest.mark.parametrize("ps,k1,T,ctx", [
    (3, 62, 96, 400),      # small summaries: append launch, one selection launch, attention
    (2, 128, 96, 1100),    # large summaries: the score launch takes the token in, then top-k, attention
    (1, 128, 64, 700),     # Exact-TopK setting, every step opens a new page
    (1, 40, 500, 9000),    # more than 8192 pages: the scores go through memory, with the token taken in
])
def test_decode_append_token_major(env, oracle, ps, k1, T, ctx):
    """A run of decode steps with the new token folded in, small pages."""
    torch, rk, dev = env
    steps = 20
    w = small("tiny", batch=2, context=ctx, page_size=ps, channel_budget=k1, token_budget=T, n_heavy=5)
    say("decode+append token-major", ps, k1, T, ctx, steps)
    full = wl.generate(wl.scaled(w, context=ctx + steps))
    lens = np.array([ctx, ctx - 89], dtype=np.int32)
    d0 = dict(full)
    d0["K"] = np.ascontiguousarray(full["K"][:, :, :ctx])
    d0["V"] = np.ascontiguousarray(full["V"][:, :, :ctx])
    d0["seq_lens"] = lens.copy()
    cache, q = to_device_cache(rk, torch, d0, w.n_q_heads, ps, dev, pages_cap=(ctx + steps + ps - 1) // ps,
                               shuffle_rng=np.random.default_rng(70), v_layout=TM)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    Kref = np.zeros((2, w.n_kv_heads, ctx + steps, 128), dtype=np.uint16)
    Vref = np.zeros_like(Kref)
    for b in range(2):
        Kref[b, :, :lens[b]] = full["K"][b, :, :lens[b]]
        Vref[b, :, :lens[b]] = full["V"][b, :, :lens[b]]
    row = rk.pages_row_len(cache, T)
    out = torch.empty((2, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    pages = torch.empty((2, w.n_kv_heads, row), dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, T)
    for s in range(steps):
        kn, vn = full["K"][:, :, ctx + s], full["V"][:, :, ctx + s]
        for b in range(2):
            Kref[b, :, lens[b]] = kn[b]
            Vref[b, :, lens[b]] = vn[b]
        lens += 1
        rk.hsa_decode_append(cache, q, wl.from_bits(kn, dev), wl.from_bits(vn, dev), kmax, kmin, k1, T, 1,
                             out, None, pages, None, ws)
        if s % 7 == 6 or s == steps - 1:
            torch.cuda.synchronize()
            assert cache.seq_lens.cpu().numpy().tolist() == lens.tolist()
            ds = dict(q=d0["q"], K=Kref, V=Vref, seq_lens=lens.copy())
            gp = pages.cpu().numpy()
            check_selection(oracle, ds, w, cache.pages_cap, gp, None, None, 1)
            want_y, _ = oracle.attend_given(ds["q"], Kref, Vref, lens, ps, gp)
            assert_attention_close(wl.to_bits(out), want_y, f"step {s}")
    Kg, Vg = rk.unpack_cache(cache)
    Kg, Vg = wl.to_bits(Kg), wl.to_bits(Vg)
    for b in range(2):
        assert np.array_equal(Kg[b, :, :lens[b]], Kref[b, :, :lens[b]])
        assert np.array_equal(Vg[b, :, :lens[b]], Vref[b, :, :lens[b]])
    want_max, want_min = oracle.build_summaries(Kref, lens, ps, cache.pages_cap)
    valid = ~np.isnan(want_max)
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmax))[valid], want_max[valid])
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmin))[valid], want_min[valid])


@pytest.mark.parametrize("src_layout,dst_layout,dps", [(0, TM, 3), (TM, TM, 2), (TM, 0, 16), (0, TM, 16)])
def test_snapkv_into_token_major(env, oracle, src_layout, dst_layout, dps):
    """Stage 1 writing the cache Stage 2 will use at its own page size."""
    torch, rk, dev = env
    w = small("mistral_snap_128k", batch=2, context=3000, snap_keep=500, n_heavy=8)
    say("snapkv layouts", src_layout, dst_layout, dps)
    d = ragged(wl.generate(w, with_obs=True), (3000, 2999))
    N, W = w.snap_keep, w.window
    src, _ = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev, shuffle_rng=np.random.default_rng(80),
                             v_layout=src_layout)
    dst = rk.alloc_cache(w.batch, w.n_q_heads, w.n_kv_heads, 128, dps, (N + dps - 1) // dps, dev, zero=True,
                         v_layout=dst_layout)
    kept = torch.full((w.batch, w.n_kv_heads, N), -9, dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_SNAPKV, src, W, N)
    rk.snapkv_compress(wl.from_bits(d["qobs"], dev), src, W, w.pool_kernel, N, dst, kept, ws)
    torch.cuda.synchronize()
    ref = oracle.snapkv(d["qobs"], d["K"], d["seq_lens"], w.pool_kernel, N, want_votes=True)
    gk = kept.cpu().numpy()
    assert dst.seq_lens.cpu().numpy().tolist() == ref["n_kept"].tolist()
    Kd, Vd = rk.unpack_cache(dst)
    Kd, Vd = wl.to_bits(Kd), wl.to_bits(Vd)
    for b in range(w.batch):
        L = int(d["seq_lens"][b]) - W
        for g in range(w.n_kv_heads):
            row = gk[b, g]
            assert_topk_within_band(ref["pooled"][b, g, :L], row[:N - W], N - W, f"kept b{b} g{g}")
            assert np.array_equal(Kd[b, g, :N], d["K"][b, g, row])
            assert np.array_equal(Vd[b, g, :N], d["V"][b, g, row])


@pytest.mark.parametrize("mode", ["pairs", "constant", "spread"])
def test_split_selection_breaks_ties_towards_lower_index(env, oracle, mode):
    """Large summaries take the score launch + top-k launch; its pick must resolve exact ties the way
    Algorithm 1's argtopk is read here (larger score, then lower page), whether the value-binned
    search decides or, for scores without a range, the radix passes behind it."""
    torch, rk, dev = env
    w = small("tiny", context=1100, page_size=1, channel_budget=128, token_budget=150, n_heavy=0)
    say("split select ties", mode)
    d = wl.generate(w)
    K = d["K"].copy()
    if mode == "pairs":
        K[:, :, 1::2] = K[:, :, 0:-1:2]          # every key twice: every score twice
    elif mode == "constant":
        K[:] = K[:, :, :1]                       # one key everywhere: every score equal
    d["K"] = K
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, 1, dev, v_layout=TM)
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    row = rk.pages_row_len(cache, w.token_budget)
    pages = torch.empty((1, w.n_kv_heads, row), dtype=torch.int32, device=dev)
    scores = torch.empty((1, w.n_kv_heads, cache.pages_cap), dtype=torch.float32, device=dev)
    rk.hsa_select(cache, q, kmax, kmin, 128, w.token_budget, 0, pages, None, scores)
    torch.cuda.synchronize()
    gp, gs = pages.cpu().numpy(), scores.cpu().numpy()
    for g in range(w.n_kv_heads):
        # exact expectation from the GPU's own fp32 scores: stable sort, larger first, lower index first
        sc = gs[0, g, :1100]
        want = np.sort(np.argsort(-sc.astype(np.float64), kind="stable")[:150])
        assert np.array_equal(gp[0, g, :150], want), (mode, g)
    check_selection(oracle, d, w, cache.pages_cap, gp, None, gs)


@pytest.mark.parametrize("ps,k1,ctx,why", [(4, 32, 1000, "fused launch"), (2, 128, 1100, "score/pick/attention launches")])
def test_append_to_a_full_cache_is_a_plain_decode(env, oracle, ps, k1, ctx, why):
    """A sequence that already holds pages_cap * page_size tokens is left unchanged by the append and
    still gets its attention result; its neighbour in the batch takes the token as usual."""
    torch, rk, dev = env
    T = 96
    say("append to full cache, token-major", ps, k1, why)
    cap_pages = ((ctx + ps - 1) // ps + 7) // 8 * 8
    full_len = cap_pages * ps
    w = small("tiny", batch=2, context=full_len, page_size=ps, channel_budget=k1, token_budget=T, n_heavy=4)
    d = wl.generate(w)
    d["seq_lens"] = np.array([full_len, full_len - 10], dtype=np.int32)
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, ps, dev, pages_cap=cap_pages, v_layout=TM)
    assert cache.pages_cap == cap_pages
    kmax, kmin = rk.alloc_summaries(cache)
    rk.build_page_summaries(cache, kmax, kmin)
    row = rk.pages_row_len(cache, T)
    out = torch.empty((2, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    pages = torch.empty((2, w.n_kv_heads, row), dtype=torch.int32, device=dev)
    ws = rk.alloc_workspace(rk.OP_HSA_DECODE, cache, T)
    rng = np.random.default_rng(5)
    kn = wl.f32_to_bf16_bits(rng.standard_normal((2, w.n_kv_heads, 128)).astype(np.float32))
    vn = wl.f32_to_bf16_bits(rng.standard_normal((2, w.n_kv_heads, 128)).astype(np.float32))
    k_before = cache.k_pool.clone()
    rk.hsa_decode_append(cache, q, wl.from_bits(kn, dev), wl.from_bits(vn, dev), kmax, kmin, k1, T, 0, out, None,
                         pages, None, ws)
    torch.cuda.synchronize()
    assert cache.seq_lens.cpu().numpy().tolist() == [full_len, full_len - 9]
    K = d["K"].copy()
    V = d["V"].copy()
    K[1, :, full_len - 10] = kn[1]
    V[1, :, full_len - 10] = vn[1]
    lens = np.array([full_len, full_len - 9], dtype=np.int32)
    gp = pages.cpu().numpy()
    dd = dict(q=d["q"], K=K, V=V, seq_lens=lens)
    check_selection(oracle, dd, w, cache.pages_cap, gp, None, None)
    want_y, _ = oracle.attend_given(d["q"], K, V, lens, ps, gp)
    assert_attention_close(wl.to_bits(out), want_y, "y")
    # sequence 0's rows are untouched
    Kg, _ = rk.unpack_cache(cache)
    assert np.array_equal(wl.to_bits(Kg)[0], d["K"][0, :, :full_len])
    # and the workspace is ready for the next call: same inputs, same bits
    out2 = torch.empty_like(out)
    rk.hsa_decode(cache, q, kmax, kmin, k1, T, 0, out2, None, None, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
