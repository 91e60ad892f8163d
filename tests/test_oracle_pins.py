"""Pins for the CPU oracle (no GPU).

Each test ties a part of ``oracle/`` to something other than itself: a library
routine on a special case that reduces to a textbook definition, a bound the
paper states, brute force on tiny inputs, or numbers the paper prints.
Citations are to arXiv 2502.14051.
"""
import os

import numpy as np
import pytest
import torch

from paper_2502_14051_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_bits(rng, shape, scale=1.0):
    return wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32) * scale)


def torch_dense(q, K, V, seq_lens):
    """softmax(q K^T / sqrt(D)) V with torch fp64 library ops, explicit GQA repeat."""
    qf = torch.from_numpy(wl.bf16_bits_to_f64(q))
    Kf = torch.from_numpy(wl.bf16_bits_to_f64(K))
    Vf = torch.from_numpy(wl.bf16_bits_to_f64(V))
    B, Hq, D = qf.shape
    Hkv = Kf.shape[1]
    G = Hq // Hkv
    ys, lses = [], []
    for b in range(B):
        n = int(seq_lens[b])
        Kb = Kf[b, :, :n].repeat_interleave(G, dim=0)     # [Hq][n][D]
        Vb = Vf[b, :, :n].repeat_interleave(G, dim=0)
        logits = torch.einsum("hd,hnd->hn", qf[b], Kb) / np.sqrt(D)
        ys.append(torch.einsum("hn,hnd->hd", torch.softmax(logits, dim=-1), Vb))
        lses.append(torch.logsumexp(logits, dim=-1))
    return torch.stack(ys).numpy(), torch.stack(lses).numpy()


# ---------------------------------------------------------------- top-k
def brute_topk(v, k):
    order = sorted(range(len(v)), key=lambda i: (-v[i], i))
    return sorted(order[:k])


def test_topk_matches_full_sort_with_planted_ties(oracle):
    rng = np.random.default_rng(0)
    for n, k in [(1, 1), (7, 3), (64, 64), (64, 10), (33, 0), (50, 49)]:
        v = np.round(rng.standard_normal(n), 1)  # coarse values: many exact ties
        got = oracle.topk(v, k)
        assert got.tolist() == brute_topk(v.tolist(), k)
    v = np.zeros(16)
    assert oracle.topk(v, 5).tolist() == [0, 1, 2, 3, 4]  # all tied -> lowest indices


def test_pages_to_pick_rule(oracle):
    # budget >= context -> every page (dense); otherwise whole pages within budget, at least one
    assert oracle.pages_to_pick(4096, 16, 4096) == 256
    assert oracle.pages_to_pick(4096, 16, 10 ** 6) == 256
    assert oracle.pages_to_pick(17, 16, 17) == 2
    assert oracle.pages_to_pick(4096, 16, 256) == 16
    assert oracle.pages_to_pick(4096, 16, 250) == 15
    assert oracle.pages_to_pick(4096, 16, 3) == 1
    assert oracle.pages_to_pick(0, 16, 256) == 0
    assert oracle.pages_to_pick(100, 3, 30) == 10


# ---------------------------------------------------------------- Step 1
@pytest.mark.parametrize("n,ps", [(64, 16), (50, 16), (7, 3), (5, 1), (16, 16), (3, 16)])
def test_summaries_bound_and_attained(oracle, n, ps):
    """Section 3.4 Step 1: K_min <= K_j <= K_max channel-wise within a page, both attained."""
    rng = np.random.default_rng(n * 31 + ps)
    D = 8
    K = rand_bits(rng, (n, D))
    kmax, kmin = oracle.page_summaries(K, ps)
    Kf = wl.bf16_bits_to_f64(K)
    P = (n + ps - 1) // ps
    assert kmax.shape == (D, P)
    for p in range(P):
        blk = Kf[p * ps:min((p + 1) * ps, n)]
        assert np.array_equal(kmax[:, p], blk.max(axis=0))  # numpy reduction, not the oracle's loop
        assert np.array_equal(kmin[:, p], blk.min(axis=0))
        assert (blk <= kmax[:, p]).all() and (blk >= kmin[:, p]).all()


# ---------------------------------------------------------------- Step 2
@pytest.mark.parametrize("G", [1, 4, 8])
@pytest.mark.parametrize("n,ps", [(96, 16), (90, 16), (40, 3), (33, 1)])
def test_page_score_upper_bounds_group_logit(oracle, G, n, ps):
    """Section 3.4 Step 2: with every channel kept the page score is the largest value the
    group-summed logit can take inside the page's min/max box, hence >= the value at every key
    of the page; with one token per page it is attained."""
    rng = np.random.default_rng(G * 1000 + n + ps)
    D = 16
    q = rand_bits(rng, (G, D))
    K = rand_bits(rng, (n, D))
    a, s, i1 = oracle.channel_select(q, D)
    assert i1.tolist() == list(range(D))
    kmax, kmin = oracle.page_summaries(K, ps)
    score = oracle.page_scores(s, i1, kmax, kmin)
    qsum = wl.bf16_bits_to_f64(q).sum(axis=0)
    logit = wl.bf16_bits_to_f64(K) @ qsum
    for j in range(n):
        assert score[j // ps] >= logit[j] - 1e-9 * (1 + abs(logit[j]))
    if ps == 1:
        np.testing.assert_allclose(score, logit, rtol=1e-12, atol=1e-12)
    else:
        # strictness: some page is strictly above all of its keys (box corner is not a key)
        page_best = np.array([logit[p * ps:min((p + 1) * ps, n)].max() for p in range(len(score))])
        assert (score > page_best + 1e-6).any()


def test_channel_select_is_topk_of_abs_sum_and_sign_of_sum(oracle):
    """Algorithm 1, first two assignments: |q| summed over the group ranks channels; q summed
    over the group gives the sign.  Heads are built so the two sums disagree."""
    D, G, k1 = 8, 2, 3
    qf = np.zeros((G, D), dtype=np.float32)
    qf[0] = [4, -4, 1, 0.5, 3, -1, 0.25, 2]
    qf[1] = [-4, 3, 1, 0.5, 3, -2, 0.25, -2]
    # |q| sums: 8 7 2 1 6 3 .5 4 ; q sums: 0 -1 2 1 6 -3 .5 0
    a, s, i1 = oracle.channel_select(wl.f32_to_bf16_bits(qf), k1)
    assert a.tolist() == [8, 7, 2, 1, 6, 3, 0.5, 4]
    assert s.tolist() == [0, -1, 2, 1, 6, -3, 0.5, 0]
    assert i1.tolist() == [0, 1, 4]
    # sign rule (Algorithm 1: g >= 0 -> K_max, g < 0 -> K_min), one page with max=+1, min=-1:
    kmax = np.ones((D, 1))
    kmin = -np.ones((D, 1))
    score = oracle.page_scores(s, i1, kmax, kmin)
    # channel 0: s=0 -> 0 ; channel 1: s=-1 uses K_min=-1 -> +1 ; channel 4: s=6 uses K_max -> 6
    assert score.tolist() == [7.0]


def test_partial_channels_equal_full_channels_on_masked_query(oracle):
    """Dropping the non-selected channels (Section 3.4 Step 2, 'ignore others') is the same as a
    full-channel score of a query whose other channels are zero."""
    rng = np.random.default_rng(5)
    G, D, n, ps, k1 = 4, 32, 200, 16, 8
    q = rand_bits(rng, (G, D), scale=np.exp(rng.standard_normal(D)))
    K = rand_bits(rng, (n, D))
    a, s, i1 = oracle.channel_select(q, k1)
    kmax, kmin = oracle.page_summaries(K, ps)
    part = oracle.page_scores(s, i1, kmax, kmin)
    qm = q.copy()
    mask = np.ones(D, dtype=bool)
    mask[i1] = False
    qm[:, mask] = 0
    a2, s2, i_all = oracle.channel_select(qm, D)
    full = oracle.page_scores(s2, i_all, kmax, kmin)
    np.testing.assert_allclose(part, full, rtol=1e-13, atol=1e-13)
    # and the kept channels are the k1 largest of a by an independent sort
    assert sorted(np.argsort(-a, kind="stable")[:k1].tolist()) == i1.tolist()


def test_exact_topk_special_case(oracle):
    """Appendix A.3 Exact-TopK: page size 1 and every channel kept turn the selection into the
    exact top-T of the group-summed logits."""
    rng = np.random.default_rng(7)
    B, Hkv, G, D, n, T = 2, 2, 4, 16, 120, 20
    q = rand_bits(rng, (B, Hkv * G, D))
    K = rand_bits(rng, (B, Hkv, n, D))
    V = rand_bits(rng, (B, Hkv, n, D))
    r = oracle.hsa_decode(q, K, V, [n, n], ps=1, k1=D, T=T)
    qf = wl.bf16_bits_to_f64(q).reshape(B, Hkv, G, D)
    Kf = wl.bf16_bits_to_f64(K)
    for b in range(B):
        for g in range(Hkv):
            logit = Kf[b, g] @ qf[b, g].sum(axis=0)
            assert r["pages"][b, g, :T].tolist() == brute_topk(logit.tolist(), T)
            assert (r["pages"][b, g, T:] == -1).all()


# ---------------------------------------------------------------- Step 3
@pytest.mark.parametrize("Hkv,G", [(1, 1), (2, 4), (1, 8)])
@pytest.mark.parametrize("lens,ps", [((64, 64), 16), ((50, 23), 16), ((10, 1), 3)])
def test_budget_covering_context_is_dense_attention(oracle, Hkv, G, lens, ps):
    """Token budget >= context: every page is picked and HSA is plain softmax attention
    (Table 1 Full-KV row); checked against torch's softmax / einsum in fp64."""
    rng = np.random.default_rng(Hkv * 100 + G * 10 + ps)
    B, D, ncap = len(lens), 16, max(lens)
    q = rand_bits(rng, (B, Hkv * G, D))
    K = rand_bits(rng, (B, Hkv, ncap, D))
    V = rand_bits(rng, (B, Hkv, ncap, D))
    want_y, want_lse = torch_dense(q, K, V, lens)
    r = oracle.hsa_decode(q, K, V, lens, ps=ps, k1=4, T=ncap)
    np.testing.assert_allclose(r["y"], want_y, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(r["lse"], want_lse, rtol=1e-12, atol=1e-12)
    yd, lsed = oracle.dense_decode(q, K, V, lens)
    np.testing.assert_allclose(yd, want_y, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lsed, want_lse, rtol=1e-12, atol=1e-12)
    for b, n in enumerate(lens):
        P = (n + ps - 1) // ps
        assert r["pages"][b, 0, :P].tolist() == list(range(P))


def test_sparse_attention_equals_dense_over_the_gathered_tokens(oracle):
    """Step 3 restricted to a page list == library softmax attention over exactly those tokens."""
    rng = np.random.default_rng(11)
    G, D, n, ps = 4, 16, 75, 16
    q = rand_bits(rng, (G, D))
    K = rand_bits(rng, (n, D))
    V = rand_bits(rng, (n, D))
    pages = [1, 4]  # page 4 is the partial tail (tokens 64..74)
    y, lse = oracle.attend_pages(q, K, V, ps, pages)
    tok = list(range(16, 32)) + list(range(64, 75))
    want_y, want_lse = torch_dense(q[None], K[tok][None, None], V[tok][None, None], [len(tok)])
    np.testing.assert_allclose(y, want_y[0], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lse, want_lse[0], rtol=1e-12, atol=1e-12)


def test_tiny_invariants(oracle):
    """Tiny inputs: weights sum to one (V = 1 gives y = 1), outputs lie inside the picked values'
    range, the picked pages are the brute-force top pages of the returned scores."""
    rng = np.random.default_rng(13)
    B, Hkv, G, D, n, ps, k1, T = 1, 2, 2, 8, 64, 4, 3, 16
    q = rand_bits(rng, (B, Hkv * G, D))
    K = rand_bits(rng, (B, Hkv, n, D))
    V = rand_bits(rng, (B, Hkv, n, D))
    ones = wl.f32_to_bf16_bits(np.ones((B, Hkv, n, D), dtype=np.float32))
    r1 = oracle.hsa_decode(q, K, ones, [n], ps, k1, T)
    np.testing.assert_allclose(r1["y"], 1.0, rtol=1e-13)
    r = oracle.hsa_decode(q, K, V, [n], ps, k1, T, want_scores=True)
    Vf = wl.bf16_bits_to_f64(V)
    for g in range(Hkv):
        pages = r["pages"][0, g, :T // ps]
        assert pages.tolist() == brute_topk(r["scores"][0, g, :n // ps].tolist(), T // ps)
        tok = np.concatenate([np.arange(p * ps, (p + 1) * ps) for p in pages])
        lo, hi = Vf[0, g, tok].min(axis=0), Vf[0, g, tok].max(axis=0)
        for h in range(G):
            y = r["y"][0, g * G + h]
            assert (y >= lo - 1e-12).all() and (y <= hi + 1e-12).all()


def test_recent_pages_are_forced(oracle):
    rng = np.random.default_rng(17)
    B, Hkv, G, D, n, ps = 1, 1, 2, 8, 70, 8
    q = rand_bits(rng, (B, Hkv * G, D))
    K = rand_bits(rng, (B, Hkv, n, D))
    K[0, 0, 56:] = 0  # make the last two pages unattractive
    K[0, 0, :56] = wl.f32_to_bf16_bits(np.abs(wl.bf16_bits_to_f32(K[0, 0, :56])) *
                                       np.sign(wl.bf16_bits_to_f32(q[0]).sum(0))[None, :] + 0)
    V = rand_bits(rng, (B, Hkv, n, D))
    r0 = oracle.hsa_decode(q, K, V, [n], ps, D, 24, n_recent=0)
    r2 = oracle.hsa_decode(q, K, V, [n], ps, D, 24, n_recent=2)
    assert 8 not in r0["pages"][0, 0, :3] and 7 not in r0["pages"][0, 0, :3]
    assert r2["pages"][0, 0, :3].tolist()[-2:] == [7, 8]
    assert r2["pages"][0, 0, 0] == r0["pages"][0, 0, 0] or r2["pages"][0, 0, 0] in r0["pages"][0, 0, :3]


def test_empty_sequence(oracle):
    rng = np.random.default_rng(19)
    q = rand_bits(rng, (2, 4, 8))
    K = rand_bits(rng, (2, 2, 16, 8))
    V = rand_bits(rng, (2, 2, 16, 8))
    r = oracle.hsa_decode(q, K, V, [0, 16], 4, 4, 8)
    assert (r["y"][0] == 0).all() and np.isneginf(r["lse"][0]).all()
    assert (r["pages"][0] == -1).all()
    assert np.isfinite(r["y"][1]).all()


def test_planted_heavy_pages_are_recalled(oracle):
    """Workload-level plausibility (Section 3.1's heavy hitters): when the page budget covers the
    planted tokens, HSA picks every one of their pages and reproduces dense attention closely."""
    w = wl.CONFIGS["tiny"]
    d = wl.generate(w)
    r = oracle.hsa_decode(d["q"], d["K"], d["V"], d["seq_lens"], w.page_size, w.channel_budget,
                          w.token_budget)
    for g in range(w.n_kv_heads):
        hp = np.unique(d["heavy"][0, g] // w.page_size)
        assert np.isin(hp, r["pages"][0, g]).all()
    yd, _ = oracle.dense_decode(d["q"], d["K"], d["V"], d["seq_lens"])
    assert np.abs(yd - r["y"]).max() < 1e-3


# ---------------------------------------------------------------- batch wrappers
def test_attend_given_batch_against_library(oracle):
    """The batch re-evaluation of Step 3 on a supplied list (several sequences of different lengths,
    several KV heads, a GQA group, rows cut short by -1) equals torch's fp64 softmax attention over
    exactly the listed tokens of the right (sequence, KV head), head by head."""
    rng = np.random.default_rng(101)
    B, Hkv, G, D, ps, ncap, cap = 3, 2, 4, 16, 4, 40, 6
    lens = [37, 18, 40]
    q = rand_bits(rng, (B, Hkv * G, D))
    K = rand_bits(rng, (B, Hkv, ncap, D))
    V = rand_bits(rng, (B, Hkv, ncap, D))
    pages = np.full((B, Hkv, cap), -1, dtype=np.int32)
    rows = {(0, 0): [0, 3, 9], (0, 1): [1, 2, 4, 8, 9], (1, 0): [4], (1, 1): [0, 2, 3, 4],
            (2, 0): [], (2, 1): [0, 1, 5, 6, 7, 9]}  # page 9 of 37 tokens / page 4 of 18 are partial tails
    for (b, g), r in rows.items():
        pages[b, g, :len(r)] = r
    # what follows a -1 must be ignored, whatever it holds
    pages[1, 0, 2] = 1
    y, lse = oracle.attend_given(q, K, V, lens, ps, pages)
    for (b, g), r in rows.items():
        tok = [j for p_ in r for j in range(p_ * ps, min((p_ + 1) * ps, lens[b]))]
        sl = slice(g * G, (g + 1) * G)
        if not tok:
            assert (y[b, sl] == 0).all() and np.isneginf(lse[b, sl]).all()
            continue
        want_y, want_lse = torch_dense(q[b:b + 1, sl], K[b, g][tok][None, None], V[b, g][tok][None, None], [len(tok)])
        np.testing.assert_allclose(y[b, sl], want_y[0], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(lse[b, sl], want_lse[0], rtol=1e-12, atol=1e-12)


def test_attend_given_on_the_full_list_is_dense_and_on_the_picked_list_is_hsa(oracle):
    """Two fixed points of the wrapper: the list of every page gives full attention (torch), and the
    list Algorithm 1 picked gives Algorithm 1's own y."""
    rng = np.random.default_rng(103)
    B, Hkv, G, D, ps, ncap = 2, 2, 4, 16, 8, 64
    lens = [64, 41]
    q = rand_bits(rng, (B, Hkv * G, D))
    K = rand_bits(rng, (B, Hkv, ncap, D))
    V = rand_bits(rng, (B, Hkv, ncap, D))
    every = np.full((B, Hkv, ncap // ps), -1, dtype=np.int32)
    for b, n in enumerate(lens):
        P = (n + ps - 1) // ps
        every[b, :, :P] = np.arange(P)
    y, lse = oracle.attend_given(q, K, V, lens, ps, every)
    want_y, want_lse = torch_dense(q, K, V, lens)
    np.testing.assert_allclose(y, want_y, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lse, want_lse, rtol=1e-12, atol=1e-12)
    r = oracle.hsa_decode(q, K, V, lens, ps=ps, k1=6, T=24)
    y2, lse2 = oracle.attend_given(q, K, V, lens, ps, r["pages"])
    np.testing.assert_array_equal(y2, r["y"])
    np.testing.assert_array_equal(lse2, r["lse"])


def test_build_summaries_batch_against_numpy(oracle):
    """Batch Step 1 into rows of pages_cap > P columns: every written column is numpy's max / min over
    the page's valid tokens of the right (sequence, KV head); columns at and beyond P stay untouched."""
    rng = np.random.default_rng(107)
    B, Hkv, D, ps, ncap, cap = 3, 2, 8, 4, 30, 12
    lens = [30, 9, 0]
    K = rand_bits(rng, (B, Hkv, ncap, D))
    kmax, kmin = oracle.build_summaries(K, lens, ps, pages_cap=cap)
    Kf = wl.bf16_bits_to_f64(K)
    for b, n in enumerate(lens):
        P = (n + ps - 1) // ps
        for g in range(Hkv):
            for p_ in range(P):
                blk = Kf[b, g, p_ * ps:min((p_ + 1) * ps, n)]  # [tokens][D]
                np.testing.assert_array_equal(kmax[b, g, :, p_], blk.max(axis=0))
                np.testing.assert_array_equal(kmin[b, g, :, p_], blk.min(axis=0))
            assert np.isnan(kmax[b, g, :, P:]).all() and np.isnan(kmin[b, g, :, P:]).all()


def test_snapkv_batch_ragged_against_library(oracle):
    """Batch Stage 1 with several sequences of different lengths (one short enough to be kept whole),
    two KV heads and a GQA group: each (sequence, KV head) equals the torch rebuild on its own slices
    (Section 3.3: window-summed, group-summed causal softmax, max-pool, top-(N-W) plus the window)."""
    rng = np.random.default_rng(109)
    B, Hkv, G, W, D, Scap, N, ks = 3, 2, 2, 4, 16, 70, 20, 5
    lens = [70, 18, 43]
    qobs = rand_bits(rng, (B, Hkv * G, W, D), scale=2.0)
    K = rand_bits(rng, (B, Hkv, Scap, D), scale=2.0)
    r = oracle.snapkv(qobs, K, lens, ks=ks, N=N, want_votes=True)
    assert r["n_kept"].tolist() == [N, 18, N]
    for b, S in enumerate(lens):
        for g in range(Hkv):
            if S <= N:
                assert r["kept"][b, g, :S].tolist() == list(range(S)) and (r["kept"][b, g, S:] == -1).all()
                continue
            L = S - W
            probs = torch_window_probs(qobs[b, g * G:(g + 1) * G], K[b, g], S, W)
            gv = probs[:, :, :L].sum(dim=(0, 1))
            np.testing.assert_allclose(r["gv"][b, g, :L], gv.numpy(), rtol=1e-11, atol=1e-14)
            gv_o = torch.from_numpy(r["gv"][b, g, :L].copy())
            pooled = torch.nn.functional.max_pool1d(gv_o[None, None], ks, stride=1, padding=ks // 2)[0, 0]
            np.testing.assert_array_equal(r["pooled"][b, g, :L], pooled.numpy())
            assert r["kept"][b, g].tolist() == brute_topk(r["pooled"][b, g, :L].tolist(), N - W) + list(range(L, S))


# ---------------------------------------------------------------- SnapKV
def torch_window_probs(qobs, K, S, W):
    """Causal softmax rows of the last W positions, torch fp64.  qobs: [H][W][D], K: [S][D]."""
    qf = torch.from_numpy(wl.bf16_bits_to_f64(qobs))
    Kf = torch.from_numpy(wl.bf16_bits_to_f64(K[:S]))
    logits = torch.einsum("hwd,sd->hws", qf, Kf) / np.sqrt(qf.shape[-1])
    pos = torch.arange(S)[None, None, :]
    lim = (S - W + torch.arange(W))[None, :, None]
    logits = logits.masked_fill(pos > lim, float("-inf"))
    return torch.softmax(logits, dim=-1)


def test_snapkv_identity_when_prompt_fits(oracle):
    rng = np.random.default_rng(23)
    qobs = rand_bits(rng, (1, 2, 4, 8))
    K = rand_bits(rng, (1, 1, 20, 8))
    r = oracle.snapkv(qobs, K, [20], ks=7, N=32)
    assert r["n_kept"].tolist() == [20]
    assert r["kept"][0, 0, :20].tolist() == list(range(20)) and (r["kept"][0, 0, 20:] == -1).all()


@pytest.mark.parametrize("G", [1, 4])
def test_snapkv_votes_and_selection_against_library(oracle, G):
    """Section 3.3: votes are window-summed (and group-summed) causal softmax probabilities of the
    prefix columns; pooling is a stride-1 max-pool; the kept set is the top-(N-W) of the pooled
    votes plus the window.  Each stage is rebuilt with torch library ops."""
    rng = np.random.default_rng(29 + G)
    Hkv, W, D, S, N, ks = 2, 4, 16, 90, 24, 5
    qobs = rand_bits(rng, (1, Hkv * G, W, D), scale=2.0)
    K = rand_bits(rng, (1, Hkv, S, D), scale=2.0)
    r = oracle.snapkv(qobs, K, [S], ks=ks, N=N, want_votes=True)
    L = S - W
    for g in range(Hkv):
        probs = torch_window_probs(qobs[0, g * G:(g + 1) * G], K[0, g], S, W)  # [G][W][S]
        np.testing.assert_allclose(probs.sum(-1).numpy(), 1.0, rtol=1e-12)
        gv = probs[:, :, :L].sum(dim=(0, 1))
        np.testing.assert_allclose(r["gv"][0, g, :L], gv.numpy(), rtol=1e-11, atol=1e-14)
        # total mass: prefix votes + window columns == G * W
        np.testing.assert_allclose(r["gv"][0, g, :L].sum() + probs[:, :, L:].sum().item(), G * W,
                                   rtol=1e-12)
        gv_o = torch.from_numpy(r["gv"][0, g, :L].copy())
        pooled = torch.nn.functional.max_pool1d(gv_o[None, None], ks, stride=1, padding=ks // 2)[0, 0]
        np.testing.assert_array_equal(r["pooled"][0, g, :L], pooled.numpy())
        assert (r["pooled"][0, g, :L] >= r["gv"][0, g, :L]).all()
        want = brute_topk(r["pooled"][0, g, :L].tolist(), N - W) + list(range(L, S))
        assert r["kept"][0, g].tolist() == want
    assert r["n_kept"].tolist() == [N]


def test_snapkv_pool1_mha_is_plain_topk_of_window_mass(oracle):
    """Kernel size 1 and group size 1 reduce the stage to the original per-head rule: top-k of the
    window-summed attention probabilities (torch.topk on torch's softmax)."""
    rng = np.random.default_rng(31)
    W, D, S, N = 8, 16, 200, 40
    qobs = rand_bits(rng, (1, 1, W, D), scale=2.0)
    K = rand_bits(rng, (1, 1, S, D), scale=2.0)
    r = oracle.snapkv(qobs, K, [S], ks=1, N=N)
    probs = torch_window_probs(qobs[0], K[0, 0], S, W)
    mass = probs[0, :, :S - W].sum(0)
    top = torch.topk(mass, N - W).indices.sort().values.tolist()
    assert r["kept"][0, 0].tolist() == top + list(range(S - W, S))


def test_snapkv_keeps_planted_tokens_and_their_neighbourhood(oracle):
    w = wl.scaled(wl.CONFIGS["mistral_snap_128k"], context=4096, snap_keep=1024, n_heavy=4,
                  n_kv_heads=2, n_q_heads=8)
    d = wl.generate(w, with_obs=True)
    r = oracle.snapkv(d["qobs"], d["K"], d["seq_lens"], ks=w.pool_kernel, N=w.snap_keep)
    L = w.context - w.window
    for g in range(w.n_kv_heads):
        kept = set(r["kept"][0, g].tolist())
        assert len(kept) == w.snap_keep and set(range(L, w.context)) <= kept
        for pos in d["heavy"][0, g]:
            if pos >= L:
                continue
            lo, hi = max(0, pos - 31), min(L - 1, pos + 31)
            assert set(range(lo, hi + 1)) <= kept


# ---------------------------------------------------------------- Section 3.6
def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def test_decomposition_worked_example(oracle):
    g = read_golden("decompose_c64.txt")
    d = oracle.decompose(g["c"])
    assert round(d["r"], 2) == g["r"]
    assert round(d["stage1"], 1) == g["stage1"]
    assert round(d["stage2"], 1) == g["stage2"]
    assert d["page"] == g["page"]
    assert round(d["head_ratio"], 1) == g["head_ratio"]


def test_decomposition_clamps_and_recombines(oracle):
    for c in [1.0, 2.0, 16.0, 400.0, 1024.0, 2.0 ** 12]:
        d = oracle.decompose(c)
        assert 0.2 <= d["r"] <= 0.8
        np.testing.assert_allclose(d["stage1"] * d["stage2"], c, rtol=1e-12)
        np.testing.assert_allclose(d["page"] * d["head_ratio"], d["stage2"], rtol=1e-12)
    assert oracle.decompose(2.0 ** 12)["r"] == 0.8  # 0.2 + 0.06*12 = 0.92 -> clamped
    assert oracle.decompose(1.0)["r"] == 0.2


def test_decomposed_operating_point_reproduces_the_budget(oracle):
    """Appendix A.3 splits the budget t evenly: Step 2 reads keep/page summary rows of `channels`
    elements (one of max/min per channel), i.e. keep*channels/(page*2D) key/value pairs = t/2, and
    Step 3 attends to t/2 tokens.  The integer point must reproduce that up to its own rounding,
    and its ratios must be the ones the section prints for c = 64."""
    g = read_golden("decompose_c64.txt")
    S, t, D = 64 * 1024, 1024, 128
    p = oracle.decompose_budget(S, t, D)
    assert p["page"] == g["page"]
    assert round(S / p["keep"], 1) == g["stage1"]
    assert abs(D / p["channels"] - g["head_ratio"]) < 0.05
    assert p["attend_tokens"] == t // 2
    for S, t in [(32768, 256), (32768, 512), (32768, 4096), (131072, 1024), (131072, 16384), (8192, 512)]:
        p = oracle.decompose_budget(S, t, D)
        step2_pairs = p["keep"] * p["channels"] / (p["page"] * 2.0 * D)
        assert abs(step2_pairs - t / 2) <= 0.02 * t / 2 + 1, (S, t, p)
        assert p["attend_tokens"] == t // 2
    # no compression asked for: nothing evicted, every channel, single-token pages
    p = oracle.decompose_budget(1000, 4096, D)
    assert (p["page"], p["keep"], p["channels"]) == (1, 1000, D)


def test_cost_model_bounds_the_buffers_of_the_operating_point(oracle):
    """Table 1: storage 1/c^r + 2/c^((1+r)/2) and traffic 1/c relative to the full KV cache.  Checked
    against bytes counted from the integer operating point: kept K/V plus the K_max/K_min pair must
    stay within the printed storage term (the pair costs 1/page of the kept K/V, half of what the
    table books for it), the two steps' traffic must add up to S/c key/value pairs, and the
    multi-turn row differs from the eviction row by exactly the first-stage saving."""
    D = 128
    for S, t in [(32768, 512), (32768, 2048), (131072, 1024), (65536, 1024)]:
        c = S / t
        m = oracle.cost_model(c)
        sp = oracle.decompose(c)
        p = oracle.decompose_budget(S, t, D)
        full = S * 2 * D                                         # elements of K and V
        kept = p["keep"] * 2 * D
        aux = 2 * D * -(-p["keep"] // p["page"])                 # K_max and K_min rows
        assert (kept + aux) / full <= m["storage"] * 1.01
        assert (kept + 2 * aux) / full >= m["storage"] * 0.75    # the table's own (doubled) accounting
        step2 = p["keep"] * p["channels"] / (p["page"] * 2.0 * D)
        assert abs((step2 + p["attend_tokens"]) / S - m["traffic"]) <= 0.03 * m["traffic"]
        np.testing.assert_allclose(m["storage_mt"] - m["storage"], 1.0 - 1.0 / sp["stage1"], rtol=1e-12)
        np.testing.assert_allclose(m["traffic"] * c, 1.0, rtol=1e-12)
    # c = 64, from the ratios the section prints: 1/10.3 + 2/(10.3 * sqrt(6.2)) = 0.175
    g = read_golden("decompose_c64.txt")
    want = 1.0 / g["stage1"] + 2.0 / (g["stage1"] * g["stage2"] ** 0.5)
    assert abs(oracle.cost_model(g["c"])["storage"] - want) < 2e-3


def test_kv_size_example_matches_byte_accounting():
    g = read_golden("kv_size_example.txt")
    total = (g["layers"] * g["batch"] * g["kv_heads"] * g["context"] * g["head_dim"]
             * g["bytes_per_elem"] * 2)
    assert total / 2 ** 30 == g["approx_gib"]
