"""Recall and output error against the token budget, on the seeded synthetic single-layer workload
(32768-token context, planted heavy tokens), for the settings the paper compares in Section 4.1:

  hsa         pages of 16 tokens, 32 of 128 channels (the benchmark's setting)
  quest-like  pages of 16 tokens, every channel
  exact-topk  pages of one token, every channel
  decomposed  page size and channel count from the adaptive decomposition of Section 3.6 for the
              budget at hand (token budget t = 2 x attended tokens)

Every row comes from the library's own kernels on one GPU: `recall` is the share of the planted heavy
tokens whose page was picked, `rel_err` the relative L2 distance of the sparse attention output from
the full-KV dense output.  A diagnostic, not a benchmark:  python -m paper_2502_14051_amd.recall_curve
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--budgets", type=str, default="128,256,512,1024,2048,4096")
    ap.add_argument("--context", type=int, default=32768)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    import torch
    from . import rocketkv as rk
    from . import workloads as wl

    dev = torch.device("cuda:0")
    w = wl.scaled(wl.CONFIGS["llama8b_layer_32k"], context=args.context)
    B, Hq, Hkv, D = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    d = wl.generate_device(w, 0, dev)
    q, heavy = d["q"].contiguous(), d["heavy"].cpu().numpy()  # heavy: [B][Hkv][n_heavy] positions
    lens = d["seq_lens"].cpu().numpy()

    def cache_for(ps, token_major):
        c = rk.pack_cache(d["K"], d["V"], lens, Hq, ps,
                          v_layout=rk.V_TOKEN_MAJOR if token_major else rk.V_CHANNEL_MAJOR)
        kmax, kmin = rk.alloc_summaries(c)
        rk.build_page_summaries(c, kmax, kmin)
        return c, kmax, kmin

    base, bmax, bmin = cache_for(16, False)
    dense = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=dev)
    rk.dense_decode(base, q, dense, None, rk.alloc_workspace(rk.OP_DENSE_DECODE, base))
    torch.cuda.synchronize()
    ref = dense.float()
    caches = {(16, False): (base, bmax, bmin)}
    rows = []
    for T in (int(x) for x in args.budgets.split(",")):
        sp = rk.decompose(args.context, 2 * T, D)
        settings = [("hsa", 16, 32, False), ("quest-like", 16, D, False), ("exact-topk", 1, D, True),
                    ("decomposed", sp["page_size"], sp["channel_budget"], True)]
        for name, ps, k1, tm in settings:
            if (ps, tm) not in caches:
                caches[(ps, tm)] = cache_for(ps, tm)
            c, kmax, kmin = caches[(ps, tm)]
            row = rk.pages_row_len(c, T)
            out = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=dev)
            pages = torch.empty((B, Hkv, row), dtype=torch.int32, device=dev)
            rk.hsa_decode(c, q, kmax, kmin, k1, T, 0, out, None, pages, None, rk.alloc_workspace(rk.OP_HSA_DECODE, c, T))
            torch.cuda.synchronize()
            gp = pages.cpu().numpy()
            hit = tot = 0
            for b in range(B):
                for g in range(Hkv):
                    picked = set(gp[b, g][gp[b, g] >= 0].tolist())
                    hp = heavy[b, g] // ps
                    hit += sum(1 for p in hp if int(p) in picked)
                    tot += len(hp)
            err = float((out.float() - ref).norm() / ref.norm())
            rows.append(dict(setting=name, token_budget=T, page_size=ps, channels=k1, recall=round(hit / max(tot, 1), 4),
                             rel_err=round(err, 5)))
    if args.json:
        print(json.dumps(rows))
        return
    print(f"context {args.context}, {Hq} query / {Hkv} KV heads, {heavy.shape[-1]} planted heavy tokens per KV head")
    print(f"{'setting':12s} {'budget':>7s} {'page':>5s} {'chan':>5s} {'recall':>7s} {'rel_err':>9s}")
    for r in rows:
        print(f"{r['setting']:12s} {r['token_budget']:7d} {r['page_size']:5d} {r['channels']:5d} {r['recall']:7.3f} {r['rel_err']:9.5f}")


if __name__ == "__main__":
    main()
