"""GPU parity for RocketKV-MT (Section 3.5): nothing is evicted, Stage 2 works through an index of
the tokens Stage 1 filtered for the turn, and the filter runs again over the whole cache at the next
turn.  By construction a logical sequence is what the eviction variant would have copied out, so the
oracle is the same fp64 code applied to the arrays gathered through the index."""
import sys

import numpy as np
import pytest

from paper_2502_14051_amd import workloads as wl
from helpers import assert_attention_close, assert_topk_within_band, to_device_cache
from test_gpu_parity import check_selection, small

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


def gather(arr, idx, lens):
    """arr [B][Hkv][S][D] gathered through idx [B][Hkv][cap] -> [B][Hkv][max len][D] (zero padded)."""
    B, Hkv = idx.shape[:2]
    out = np.zeros((B, Hkv, int(max(lens.max(), 1)), arr.shape[-1]), dtype=arr.dtype)
    for b in range(B):
        for g in range(Hkv):
            out[b, g, :lens[b]] = arr[b, g, idx[b, g, :lens[b]]]
    return out


def check_filter(oracle, qobs, K, lens, ks, N, W, got_idx, got_n):
    ref = oracle.snapkv(qobs, K, lens, ks, N, want_votes=True)
    assert got_n.tolist() == ref["n_kept"].tolist()
    for b in range(len(lens)):
        S = int(lens[b])
        for g in range(K.shape[1]):
            row = got_idx[b, g]
            if S <= N:
                assert row[:S].tolist() == list(range(S))
            else:
                L = S - W
                assert row[N - W:N].tolist() == list(range(L, S))
                assert_topk_within_band(ref["pooled"][b, g, :L], row[:N - W], N - W, f"filter b{b} g{g}")
    return ref


def decode_check(env, oracle, rk_objs, w_logical, q_bits, Kfull, Vfull, n_recent=0):
    """mt_hsa_decode against the oracle on the gathered arrays."""
    torch, rk, dev = env
    cache, index, kmax, kmin, ws = rk_objs
    k1, T = w_logical.channel_budget, w_logical.token_budget
    row = min(index.pages_cap, (T + index.page_size - 1) // index.page_size)
    out = torch.empty((cache.batch, cache.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((cache.batch, cache.n_q_heads), dtype=torch.float32, device=dev)
    pages = torch.empty((cache.batch, cache.n_kv_heads, row), dtype=torch.int32, device=dev)
    chans = torch.empty((cache.batch, cache.n_kv_heads, k1), dtype=torch.int32, device=dev)
    rk.mt_hsa_decode(cache, index, wl.from_bits(q_bits, dev), kmax, kmin, k1, T, n_recent, out, lse, pages, chans, ws)
    torch.cuda.synchronize()
    idx = index.token_index.cpu().numpy()
    nl = index.n_indexed.cpu().numpy()
    Kc, Vc = gather(Kfull, idx, nl), gather(Vfull, idx, nl)
    dc = dict(q=q_bits, K=Kc, V=Vc, seq_lens=nl.astype(np.int32))
    gp = pages.cpu().numpy()
    check_selection(oracle, dc, w_logical, index.pages_cap, gp, chans.cpu().numpy(), None, n_recent)
    want_y, want_lse = oracle.attend_given(q_bits, Kc, Vc, dc["seq_lens"], index.page_size, gp)
    assert_attention_close(wl.to_bits(out), want_y, "mt y")
    fin = np.isfinite(want_lse)
    np.testing.assert_allclose(lse.cpu().numpy()[fin], want_lse[fin], rtol=1e-3, atol=1e-3)
    return Kc, nl


@pytest.mark.parametrize("lps,cache_ps,k1,T,N", [
    (16, 16, 32, 128, 400),     # one fused launch per step
    (3, 16, 70, 90, 400),
    (4, 5, 128, 64, 400),       # cache paged differently from the logical sequence
    (1, 16, 128, 64, 600),      # large logical summaries: append, score, top-k and attention launches
])
def test_two_turns(env, oracle, lps, cache_ps, k1, T, N):
    torch, rk, dev = env
    B, S1, steps, M2, W, ks = 2, 2000, 6, 900, 32, 63
    S2 = S1 + steps + M2
    say("multi-turn", lps, cache_ps, k1, T)
    # the whole conversation's K/V, with planted tokens that matter to the SECOND turn's queries
    w2 = small("mistral_snap_128k", batch=B, context=S2, snap_keep=N, n_heavy=24, heavy_nats=8.0)
    conv = wl.generate(w2, with_obs=True)
    # the first turn's queries come from an unrelated draw
    w1 = small("mistral_snap_128k", batch=B, context=S1, snap_keep=N, n_heavy=0, seed=4242)
    turn1 = wl.generate(w1, with_obs=True)
    Hkv, Hq = w2.n_kv_heads, w2.n_q_heads
    cap_tokens = S2 + 16

    def cache_with(n_tokens, lens):
        d = dict(K=np.ascontiguousarray(conv["K"][:, :, :n_tokens]), V=np.ascontiguousarray(conv["V"][:, :, :n_tokens]),
                 q=conv["q"], seq_lens=np.asarray(lens, dtype=np.int32))
        c, _ = to_device_cache(rk, torch, d, Hq, cache_ps, dev,
                               pages_cap=(cap_tokens + cache_ps - 1) // cache_ps,
                               shuffle_rng=np.random.default_rng(90 + lps), v_layout=TM)
        return c

    # ---------------- turn 1: filter the prompt, decode a few tokens ----------------
    lens1 = np.array([S1, S1 - 77], dtype=np.int32)
    cache = cache_with(S1, lens1)
    index = rk.alloc_index(cache, lps, N + steps + 8)
    snap_src = cache
    if cache_ps != 16:
        # Stage 1 reads pages of 16: filter on a page-16 copy of the same tokens, decode on the other
        d16 = dict(K=np.ascontiguousarray(conv["K"][:, :, :S1]), V=np.ascontiguousarray(conv["V"][:, :, :S1]),
                   q=conv["q"], seq_lens=lens1)
        snap_src, _ = to_device_cache(rk, torch, d16, Hq, 16, dev, v_layout=TM)
    ws_snap = rk.alloc_workspace(rk.OP_SNAPKV, snap_src, W, N)
    k_before = cache.k_pool.clone()
    rk.snapkv_filter(wl.from_bits(turn1["qobs"], dev), snap_src, W, ks, N, index, ws_snap)
    torch.cuda.synchronize()
    assert torch.equal(k_before, cache.k_pool)  # nothing is evicted or moved
    idx1 = index.token_index.cpu().numpy().copy()
    n1 = index.n_indexed.cpu().numpy().copy()
    K1 = np.ascontiguousarray(conv["K"][:, :, :S1])
    check_filter(oracle, turn1["qobs"], K1, lens1, ks, N, W, idx1, n1)

    kmax, kmin = rk.alloc_index_summaries(cache, index)
    rk.mt_build_page_summaries(cache, index, kmax, kmin)
    ws = rk.mt_alloc_workspace(cache, index, T)
    wlog = wl.scaled(w2, page_size=lps, channel_budget=k1, token_budget=T)
    objs = (cache, index, kmax, kmin, ws)
    # full-cache arrays as the GPU holds them: sequence 1 is shorter, generated tokens follow its end
    Kfull = np.zeros((B, Hkv, cap_tokens, 128), dtype=np.uint16)
    Vfull = np.zeros_like(Kfull)
    for b in range(B):
        Kfull[b, :, :lens1[b]] = conv["K"][b, :, :lens1[b]]
        Vfull[b, :, :lens1[b]] = conv["V"][b, :, :lens1[b]]
    Kc, nl = decode_check(env, oracle, objs, wlog, turn1["q"], Kfull, Vfull)
    want_max, want_min = oracle.build_summaries(Kc, nl.astype(np.int32), lps, index.pages_cap)
    valid = ~np.isnan(want_max)
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmax))[valid], want_max[valid])
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmin))[valid], want_min[valid])

    lens = lens1.copy()
    out = torch.empty((B, Hq, 128), dtype=torch.bfloat16, device=dev)
    for s in range(steps):
        kn, vn = conv["K"][:, :, S1 + s], conv["V"][:, :, S1 + s]
        for b in range(B):
            Kfull[b, :, lens[b]] = kn[b]
            Vfull[b, :, lens[b]] = vn[b]
        if s % 2 == 0:
            rk.mt_append_kv(cache, index, wl.from_bits(kn, dev), wl.from_bits(vn, dev), kmax, kmin)
        else:
            rk.mt_hsa_decode_append(cache, index, wl.from_bits(turn1["q"], dev), wl.from_bits(kn, dev),
                                    wl.from_bits(vn, dev), kmax, kmin, k1, T, 1, out, None, None, None, ws)
        lens += 1
    torch.cuda.synchronize()
    assert cache.seq_lens.cpu().numpy().tolist() == lens.tolist()
    assert index.n_indexed.cpu().numpy().tolist() == (n1 + steps).tolist()
    idx_now = index.token_index.cpu().numpy()
    for b in range(B):
        assert (idx_now[b, :, n1[b]:n1[b] + steps] == np.arange(lens1[b], lens1[b] + steps)).all()
        assert np.array_equal(idx_now[b, :, :n1[b]], idx1[b, :, :n1[b]])
    Kg, Vg = rk.unpack_cache(cache)
    Kg, Vg = wl.to_bits(Kg), wl.to_bits(Vg)
    for b in range(B):
        assert np.array_equal(Kg[b, :, :lens[b]], Kfull[b, :, :lens[b]])
        assert np.array_equal(Vg[b, :, :lens[b]], Vfull[b, :, :lens[b]])
    Kc, nl = decode_check(env, oracle, objs, wlog, turn1["q"], Kfull, Vfull, n_recent=1)
    want_max, want_min = oracle.build_summaries(Kc, nl.astype(np.int32), lps, index.pages_cap)
    valid = ~np.isnan(want_max)
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmax))[valid], want_max[valid])
    assert np.array_equal(wl.bf16_bits_to_f64(wl.to_bits(kmin))[valid], want_min[valid])

    # ---------------- turn 2: the next prompt has been written behind the history; filter again over
    # ---------------- the whole cache
    lens2 = np.array([S2, S2], dtype=np.int32)
    cache2 = cache_with(S2, lens2)  # sequence 0's history is exactly what turn 1 left in `cache`
    src2 = cache2
    if cache_ps != 16:
        d16 = dict(K=np.ascontiguousarray(conv["K"][:, :, :S2]), V=np.ascontiguousarray(conv["V"][:, :, :S2]),
                   q=conv["q"], seq_lens=lens2)
        src2, _ = to_device_cache(rk, torch, d16, Hq, 16, dev, v_layout=TM)
    index2 = rk.alloc_index(cache2, lps, N + 8)
    ws_snap2 = rk.alloc_workspace(rk.OP_SNAPKV, src2, W, N)
    rk.snapkv_filter(wl.from_bits(conv["qobs"], dev), src2, W, ks, N, index2, ws_snap2)
    torch.cuda.synchronize()
    idx2 = index2.token_index.cpu().numpy()
    n2 = index2.n_indexed.cpu().numpy()
    K2 = np.ascontiguousarray(conv["K"][:, :, :S2])
    check_filter(oracle, conv["qobs"], K2, lens2, ks, N, W, idx2, n2)
    # tokens of the first prompt that turn 1 passed over are back in play
    back = 0
    for g in range(Hkv):
        old = set(idx1[0, g, :n1[0]].tolist())
        back += sum(1 for t in idx2[0, g, :n2[0]] if t < S1 and t not in old)
    assert back > 0
    kmax2, kmin2 = rk.alloc_index_summaries(cache2, index2)
    rk.mt_build_page_summaries(cache2, index2, kmax2, kmin2)
    ws2 = rk.mt_alloc_workspace(cache2, index2, T)
    decode_check(env, oracle, (cache2, index2, kmax2, kmin2, ws2), wlog, conv["q"], K2,
                 np.ascontiguousarray(conv["V"][:, :, :S2]))


def test_empty_and_full_logical_sequences(env, oracle):
    """Edge cases of the index: a sequence with nothing indexed gives zeros and -inf; a full index row
    or a full cache leaves the sequence unchanged on append while the others take the token."""
    torch, rk, dev = env
    say("multi-turn edge cases")
    B, S, T, k1, lps = 3, 640, 64, 32, 4
    w = small("tiny", batch=B, context=S, page_size=lps, channel_budget=k1, token_budget=T, n_heavy=4)
    d = wl.generate(w)
    d["seq_lens"] = np.array([S, S, S - 5], dtype=np.int32)
    # sequence 1's cache is exactly full (pages_cap * 16 == S); sequence 2 has room
    cache, q = to_device_cache(rk, torch, d, w.n_q_heads, 16, dev, pages_cap=S // 16, v_layout=TM)
    assert cache.pages_cap * 16 == S
    index = rk.alloc_index(cache, lps, 96)
    cap = index.pages_cap * lps
    idx = np.full((B, w.n_kv_heads, cap), -1, dtype=np.int32)
    n_idx = np.array([0, 40, cap], dtype=np.int32)   # empty / partly filled / full index row
    rng = np.random.default_rng(8)
    for b in range(B):
        for g in range(w.n_kv_heads):
            idx[b, g, :n_idx[b]] = np.sort(rng.choice(int(d["seq_lens"][b]), size=n_idx[b], replace=False))
    index.token_index.copy_(torch.from_numpy(idx).to(dev))
    index.n_indexed.copy_(torch.from_numpy(n_idx).to(dev))
    kmax, kmin = rk.alloc_index_summaries(cache, index)
    rk.mt_build_page_summaries(cache, index, kmax, kmin)
    ws = rk.mt_alloc_workspace(cache, index, T)
    out = torch.full((B, w.n_q_heads, 128), 3.0, dtype=torch.bfloat16, device=dev)
    lse = torch.zeros((B, w.n_q_heads), dtype=torch.float32, device=dev)
    row = min(index.pages_cap, (T + lps - 1) // lps)
    pages = torch.empty((B, w.n_kv_heads, row), dtype=torch.int32, device=dev)
    kn = wl.f32_to_bf16_bits(rng.standard_normal((B, w.n_kv_heads, 128)).astype(np.float32))
    vn = wl.f32_to_bf16_bits(rng.standard_normal((B, w.n_kv_heads, 128)).astype(np.float32))
    rk.mt_hsa_decode_append(cache, index, q, wl.from_bits(kn, dev), wl.from_bits(vn, dev), kmax, kmin, k1, T, 0,
                            out, lse, pages, None, ws)
    torch.cuda.synchronize()
    # sequence 0: empty index, room in both -> the new token becomes its only logical token
    # sequence 1: cache full -> unchanged; sequence 2: index full -> unchanged
    got_n = index.n_indexed.cpu().numpy().tolist()
    got_len = cache.seq_lens.cpu().numpy().tolist()
    assert got_n[1:] == [40, cap] and got_len[1:] == [S, S - 5]
    # (sequence 0's cache is full as well, so its empty index stays empty)
    assert (got_n[0], got_len[0]) == (0, S)
    y = wl.bf16_bits_to_f64(wl.to_bits(out))
    assert (y[0] == 0).all() and np.isneginf(lse.cpu().numpy()[0]).all()
    idx_now = index.token_index.cpu().numpy()
    assert np.array_equal(idx_now, idx)
    # sequences 1 and 2 against the oracle on their gathered rows
    for b in (1, 2):
        Kc = np.stack([d["K"][b, g, idx[b, g, :n_idx[b]]] for g in range(w.n_kv_heads)])[None]
        Vc = np.stack([d["V"][b, g, idx[b, g, :n_idx[b]]] for g in range(w.n_kv_heads)])[None]
        gp = pages.cpu().numpy()[b:b + 1]
        want_y, want_lse = oracle.attend_given(d["q"][b:b + 1], Kc, Vc, n_idx[b:b + 1], lps, gp)
        assert_attention_close(wl.to_bits(out)[b:b + 1], want_y, f"y b{b}")
        wb = wl.scaled(w, batch=1)
        check_selection(oracle, dict(q=d["q"][b:b + 1], K=Kc, V=Vc, seq_lens=n_idx[b:b + 1]), wb, index.pages_cap,
                        gp, None, None)
