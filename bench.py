#!/usr/bin/env python3
"""Benchmark of the RocketKV decode hot path on one MI355X.

Workload (benchmark configs[2], the shape the >=70 %-of-HBM target is stated on):
Llama3.1-8B-shaped decode step, 32 layers x (32 query / 8 KV heads, head_dim 128), batch 16,
32768-token bf16 context per sequence, SnapKV-compressed to 4096 tokens per (sequence, KV head),
then hybrid sparse attention with token budget 1024, page size 16, channel budget 32.

One "step" = one decode step of the attention path of every layer: rocketkv_hsa_decode_append, which
takes in the new token's K/V (folding the key into the tail page's min/max summary) and runs
Algorithm 1 (channel pick, page scores, page top-k, exact attention over the picked pages) in one
launch per layer.  Projections, MLPs and
weights are outside the path and not run.  Inputs are seeded synthetic data resident in HBM; the
one-time SnapKV stage and the summary build run untimed in set-up, through the same library.

Prints one JSON line: metric / value / unit, the roofline of the dominant kernel, the CPU oracle
baseline, and secondary measurements (per-stage times, the decomposed operating point, the
multi-turn variant).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published peak
# HBM bytes per launch of the fused kernel on the default workload, from rocprofv3 FETCH_SIZE /
# WRITE_SIZE counters: read at run time from the committed summary of that counter run (its line
# "roofline.traffic: kernel=<name> batch=<B> bytes_per_launch=<N>"), never a literal here.
PMC_SUMMARY = os.path.join(ROOT, "profiles", "bench_llama8b_step_b16_pmc.txt")


def measured_traffic(batch):
    """(kernel name, HBM bytes per launch) recorded for this batch size, or (None, None)."""
    try:
        for line in open(PMC_SUMMARY):
            if line.startswith("roofline.traffic:"):
                f = dict(kv.split("=", 1) for kv in line.split(":", 1)[1].split(";"))
                f = {k.strip(): v.strip() for k, v in f.items()}
                if int(f["batch"]) == batch:
                    return f["kernel"], int(f["bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        pass
    return None, None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = workload's)")
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--dense-layers", type=int, default=8,
                    help="layers whose uncompressed cache is kept for the full-KV comparison")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--kernel-reps", type=int, default=20)
    ap.add_argument("--no-decomposed", action="store_true",
                    help="skip the secondary measurement at the operating point of the adaptive decomposition")
    ap.add_argument("--q-variants", type=int, default=4,
                    help="distinct query sets cycled over the timed steps, so that consecutive steps pick "
                         "different pages (1..window)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a known-size reference "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (one process, one MI355X); "
              "--gpus > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2502_14051_amd import rocketkv as rk
    from paper_2502_14051_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    rk.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    w = wl.CONFIGS["llama8b_step_b16"]
    if args.layers:
        w = wl.scaled(w, n_layers=args.layers)
    if args.batch:
        w = wl.scaled(w, batch=args.batch)
    B, Hq, Hkv, D, G = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.group
    ps, k1, T, N, W = w.page_size, w.channel_budget, w.token_budget, w.snap_keep, w.window
    units = B * Hkv
    total_steps = args.warmup + args.steps + 8

    def hsa_bytes_at(P_, ps_, k1_, T_):
        """Algorithmic bytes of one decode-with-append step over P_ pages (all units)."""
        kp_ = min(P_, max(1, T_ // ps_))
        return units * ((kp_ * ps_ * D * 2 * 2 + 2 * G * D * 2) + (k1_ * ((P_ + 7) // 8 * 8) * 2 + G * D * 2 + kp_ * 4)
                        + (2 * D * 2 + 2 * D * 2 * 2))
    room_pages = (total_steps + ps - 1) // ps + 1
    pages_cap = (N // ps + room_pages + 7) // 8 * 8
    n_dense = min(args.dense_layers, w.n_layers)
    n_var = max(1, min(args.q_variants, W))

    # ------------------------------------------------------------------ set-up (untimed)
    t_setup = time.time()
    layers = []
    dense_layers = []
    snap_ws = None
    snap_ms = []
    for layer in range(w.n_layers):
        d = wl.generate_device(w, layer, dev, with_obs=True)
        src = rk.pack_cache(d["K"], d["V"], d["seq_lens"].cpu().numpy(), Hq, ps)
        dst = rk.alloc_cache(B, Hq, Hkv, D, ps, pages_cap, dev, zero=True)
        if snap_ws is None:
            snap_ws = rk.alloc_workspace(rk.OP_SNAPKV, src, W, N)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        rk.snapkv_compress(d["qobs"], src, W, w.pool_kernel, N, dst, None, snap_ws)
        e1.record()
        kmax, kmin = rk.alloc_summaries(dst)
        rk.build_page_summaries(dst, kmax, kmin)
        torch.cuda.synchronize()
        snap_ms.append(e0.elapsed_time(e1))
        gen = torch.Generator(device=dev)
        gen.manual_seed(77_000 + layer)
        new_k = torch.randn((B, Hkv, D), generator=gen, device=dev).bfloat16()
        new_v = torch.randn((B, Hkv, D), generator=gen, device=dev).bfloat16()
        # query sets of later steps: rows of the observation window, i.e. the layer's q plus fresh
        # noise of the same per-channel scales (consecutive decode queries are correlated, not equal)
        qv = [d["q"].contiguous()] + [d["qobs"][:, :, W - j, :].contiguous() for j in range(1, n_var)]
        L = dict(cache=dst, kmax=kmax, kmin=kmin, q=qv[0], qv=qv, new_k=new_k, new_v=new_v,
                 out=torch.empty((B, Hq, D), dtype=torch.bfloat16, device=dev),
                 ws=rk.alloc_workspace(rk.OP_HSA_DECODE, dst, T))
        layers.append(L)
        if layer < n_dense:
            dense_layers.append(dict(cache=src, q=L["q"], qobs=d["qobs"],
                                     out=torch.empty((B, Hq, D), dtype=torch.bfloat16, device=dev),
                                     ws=rk.alloc_workspace(rk.OP_DENSE_DECODE, src)))
        del d
        if layer >= n_dense:
            del src
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    if args.calib_copy_mib:
        src_c = torch.ones((args.calib_copy_mib << 20,), dtype=torch.uint8, device=dev)
        dst_c = torch.empty_like(src_c)
        torch.cuda.synchronize()
        dst_c.copy_(src_c)
        torch.cuda.synchronize()
        del src_c, dst_c

    stream = torch.cuda.Stream()  # default priority; all timed work runs on it

    # Every step appends one new key/value row per layer.  The rows are fixed synthetic buffers (their
    # values do not change the work done), so a captured step can be replayed as is.
    # Step i runs with query set i mod n_var (one captured graph per set), so the pages picked change
    # from step to step as they do in a real decode.
    def one_step(v=0):
        for L in layers:
            rk.hsa_decode_append(L["cache"], L["qv"][v], L["new_k"], L["new_v"], L["kmax"], L["kmin"], k1, T, 0,
                                 L["out"], None, None, None, L["ws"], stream)

    graphs = []
    with torch.cuda.stream(stream):
        one_step()  # eager once: surfaces launch errors before capture
        stream.synchronize()
        if not args.no_graph:
            for v in range(n_var):
                g_ = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g_, stream=stream):
                    one_step(v)
                graphs.append(g_)
    graph = graphs[0] if graphs else None

    with torch.cuda.stream(stream):
        def run_step(i):
            if graphs:
                graphs[i % n_var].replay()
            else:
                one_step(i % n_var)

        for i in range(args.warmup):
            run_step(i)
        stream.synchronize()
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        t0 = time.perf_counter()
        marks[0].record(stream)
        for i in range(args.steps):
            run_step(args.warmup + i)
            marks[i + 1].record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
    dev_ms = marks[0].elapsed_time(marks[-1])
    per_step_ms = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)])
    ms_per_step = max(dev_ms, 0.0) / args.steps
    us_layer = ms_per_step * 1e3 / w.n_layers
    n_now = int(layers[0]["cache"].seq_lens[0].item())
    P_now = (n_now + ps - 1) // ps

    # ------------------------------------------------------------------ dominant kernel alone
    # gathered attention over the page lists of the last step, through rocketkv_attend
    row = rk.pages_row_len(layers[0]["cache"], T)
    lists = []
    for L in layers:
        pg = torch.empty((B, Hkv, row), dtype=torch.int32, device=dev)
        rk.hsa_select(L["cache"], L["q"], L["kmax"], L["kmin"], k1, T, 0, pg, None, None, stream)
        lists.append(pg)
    att_ws = rk.alloc_workspace(rk.OP_ATTEND, layers[0]["cache"], row)

    def timed_graph(fn, reps):
        with torch.cuda.stream(stream):
            fn()
            stream.synchronize()
            g = None
            if not args.no_graph:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    fn()
            for _ in range(2):
                g.replay() if g is not None else fn()
            stream.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(reps):
                g.replay() if g is not None else fn()
            b.record(stream)
            stream.synchronize()
        return a.elapsed_time(b) / reps

    def attend_all():
        for L, pg in zip(layers, lists):
            rk.attend(L["cache"], L["q"], pg, L["out"], None, att_ws, stream)

    def select_all():
        for L, pg in zip(layers, lists):
            rk.hsa_select(L["cache"], L["q"], L["kmax"], L["kmin"], k1, T, 0, pg, None, None, stream)

    def decode_all():
        for L in layers:
            rk.hsa_decode(L["cache"], L["q"], L["kmax"], L["kmin"], k1, T, 0, L["out"], None, None, None,
                          L["ws"], stream)

    def append_all():
        for L in layers:
            rk.append_kv(L["cache"], L["new_k"], L["new_v"], L["kmax"], L["kmin"], stream)

    attend_us = timed_graph(attend_all, args.kernel_reps) * 1e3 / w.n_layers
    # the floor under the attention routine: the same page lists, the same work split and loads, nothing computed
    gather_sink = rk.stream_gather(layers[0]["cache"], lists[0])

    def gather_all():
        for L, pg in zip(layers, lists):
            rk.stream_gather(L["cache"], pg, gather_sink, stream)

    gather_us = timed_graph(gather_all, args.kernel_reps) * 1e3 / w.n_layers
    select_us = timed_graph(select_all, args.kernel_reps) * 1e3 / w.n_layers
    decode_us = timed_graph(decode_all, args.kernel_reps) * 1e3 / w.n_layers
    n_before = int(layers[0]["cache"].seq_lens[0].item())
    append_us = timed_graph(append_all, 2) * 1e3 / w.n_layers
    for L in layers:  # undo the appends of that probe
        L["cache"].seq_lens.fill_(n_before)

    def dense_all():
        for Ld in dense_layers:
            rk.dense_decode(Ld["cache"], Ld["q"], Ld["out"], None, Ld["ws"], stream)

    dense_us = timed_graph(dense_all, max(3, args.kernel_reps // 4)) * 1e3 / max(1, n_dense)

    # measured read ceiling: a plain streaming read of the same uncompressed pools (2 GiB per layer)
    read_gbs = None
    if n_dense > 0:
        sink = torch.empty((rk.lib().rocketkv_stream_read_sink_bytes(),), dtype=torch.uint8, device=dev)
        pools = [t for Ld in dense_layers for t in (Ld["cache"].k_pool, Ld["cache"].v_pool)]

        def read_all():
            for t in pools:
                rk.stream_read(t, sink, stream)

        read_ms = timed_graph(read_all, 3)
        read_gbs = sum(t.numel() * t.element_size() for t in pools) / (read_ms * 1e-3) / 1e9

    # The secondary measurements below run over at least eight layers each, so that a replay touches
    # several times the 256 MB of last-level cache and every launch reads from HBM as in a full model.
    # ------------------------------------------------------------------ the method's own operating point
    # Same model shape and the same traffic budget, but split the way Section 3.6 prescribes: the
    # token budget t counts Step 2 and Step 3 together (t = 2T), and the decomposition of c = S / t
    # gives the SnapKV keep budget, the page size and the channel count.  Token-major V layout, the
    # selection split into a score launch and a top-k launch, token-gather attention.
    dec_pt = None
    if not args.no_decomposed and n_dense > 0:
        sp = rk.decompose(w.context, 2 * T, D)
        ps2, k12, T2, N2 = sp["page_size"], sp["channel_budget"], sp["attend_tokens"], sp["keep_budget"]
        cap2 = ((N2 + total_steps + 8 + ps2 - 1) // ps2 + 7) // 8 * 8
        pl = []
        snap2_ws = rk.alloc_workspace(rk.OP_SNAPKV, dense_layers[0]["cache"], W, N2)
        for Ld in dense_layers:
            dst2 = rk.alloc_cache(B, Hq, Hkv, D, ps2, cap2, dev, zero=True, v_layout=rk.V_TOKEN_MAJOR)
            rk.snapkv_compress(Ld["qobs"], Ld["cache"], W, w.pool_kernel, N2, dst2, None, snap2_ws)
            km2, kn2 = rk.alloc_summaries(dst2)
            rk.build_page_summaries(dst2, km2, kn2)
            pl.append(dict(cache=dst2, kmax=km2, kmin=kn2, q=Ld["q"], out=Ld["out"],
                           new_k=layers[0]["new_k"], new_v=layers[0]["new_v"],
                           ws=rk.alloc_workspace(rk.OP_HSA_DECODE, dst2, T2)))
        torch.cuda.synchronize()

        def dec_pt_all():
            for L in pl:
                rk.hsa_decode_append(L["cache"], L["q"], L["new_k"], L["new_v"], L["kmax"], L["kmin"], k12, T2, 0,
                                     L["out"], None, None, None, L["ws"], stream)

        def dec_pt_plain():
            for L in pl:
                rk.hsa_decode(L["cache"], L["q"], L["kmax"], L["kmin"], k12, T2, 0, L["out"], None, None, None,
                              L["ws"], stream)

        pt_plain_us = timed_graph(dec_pt_plain, args.kernel_reps) * 1e3 / len(pl)
        pt_us = timed_graph(dec_pt_all, max(2, args.kernel_reps // 2)) * 1e3 / len(pl)
        n2 = int(pl[0]["cache"].seq_lens[0].item())
        P2 = (n2 + ps2 - 1) // ps2
        kp2 = min(P2, max(1, T2 // ps2))
        pt_bytes = units * (kp2 * ps2 * D * 2 * 2 + 2 * G * D * 2            # Step 3: K and V rows, q, out
                            + k12 * ((P2 + 7) // 8 * 8) * 2 + P2 * 4 * 2 + kp2 * 4 * 2  # Step 2: rows, scores, list
                            + 2 * D * 2 + 2 * D * 2 * 2)                        # the appended token
        pt_gbs = pt_bytes / (pt_us * 1e-6) / 1e9
        dec_pt = {"paper_equivalent_budget": round(T2 + P2 * k12 / (2.0 * D), 1),
                  "workload": f"same shape, t = {2 * T} split by Section 3.6: SnapKV keeps {N2}, page {ps2}, "
                              f"k1 {k12}, {T2} tokens attended, token-major V, {len(pl)} layers",
                  "us_per_layer_step": round(pt_us, 3), "us_per_layer_step_no_append": round(pt_plain_us, 3),
                  "bytes_per_layer_step": pt_bytes, "achieved_GBs": round(pt_gbs, 1),
                  "frac_of_hbm_peak": round(pt_gbs / HBM_PEAK_GBS, 4),
                  "speedup_vs_dense_full_kv": round(dense_us / pt_us, 2)}
        del pl

    # ------------------------------------------------------------------ the multi-turn variant
    # RocketKV-MT (Section 3.5) at the headline's budgets: nothing evicted, the 32768-token cache stays
    # whole (token-major V), SnapKV only writes an index of 4096 tokens, Algorithm 1 runs over that
    # logical sequence and gathers rows from the big cache.
    mt_pt = None
    if not args.no_decomposed and n_dense > 0:
        ml = []
        snapf_ws = None
        for Ld in dense_layers:
            Kf, Vf = rk.unpack_cache(Ld["cache"])
            full = rk.pack_cache(Kf[:, :, :w.context], Vf[:, :, :w.context], np.full(B, w.context, dtype=np.int32), Hq,
                                 16, pages_cap=(w.context + total_steps + 8 + 15) // 16, v_layout=rk.V_TOKEN_MAJOR)
            del Kf, Vf
            ix = rk.alloc_index(full, ps, N + total_steps + 8)
            if snapf_ws is None:
                snapf_ws = rk.alloc_workspace(rk.OP_SNAPKV, full, W, N)
            rk.snapkv_filter(Ld["qobs"], full, W, w.pool_kernel, N, ix, snapf_ws)
            km3, kn3 = rk.alloc_index_summaries(full, ix)
            rk.mt_build_page_summaries(full, ix, km3, kn3)
            ml.append(dict(cache=full, index=ix, kmax=km3, kmin=kn3, q=Ld["q"], out=Ld["out"],
                           ws=rk.mt_alloc_workspace(full, ix, T)))
        torch.cuda.synchronize()

        def mt_all():
            for L in ml:
                rk.mt_hsa_decode_append(L["cache"], L["index"], L["q"], layers[0]["new_k"], layers[0]["new_v"],
                                        L["kmax"], L["kmin"], k1, T, 0, L["out"], None, None, None, L["ws"], stream)

        mt_us = timed_graph(mt_all, max(2, args.kernel_reps // 2)) * 1e3 / len(ml)
        mt_pt = {"workload": f"RocketKV-MT, same budgets: cache of {w.context} tokens kept whole (token-major V, pages "
                             f"of 16), index of {N} tokens (+ appended), logical pages of {ps}, {len(ml)} layers",
                 "us_per_layer_step": round(mt_us, 3), "bytes_per_layer_step": hsa_bytes_at(P_now, ps, k1, T),
                 "speedup_vs_dense_full_kv": round(dense_us / mt_us, 2)}
        mt_pt["achieved_GBs"] = round(mt_pt["bytes_per_layer_step"] / (mt_us * 1e-6) / 1e9, 1)
        del ml

    # ------------------------------------------------------------------ one layer, batch 1, uncompressed context
    # BASELINE configs[1]: a single sequence of 32768 tokens, no SnapKV stage, budgets 256 / 1024 / 4096.
    # Eight (sequence, KV head) units only: a latency measurement more than a bandwidth one.
    single = None
    if not args.no_decomposed:
        w1 = wl.CONFIGS["llama8b_layer_32k"]
        sl = []
        for layer in range(32):
            d1 = wl.generate_device(w1, layer, dev)
            c1 = rk.pack_cache(d1["K"], d1["V"], d1["seq_lens"].cpu().numpy(), w1.n_q_heads, 16,
                               pages_cap=w1.context // 16 + 8)
            km1, kn1 = rk.alloc_summaries(c1)
            rk.build_page_summaries(c1, km1, kn1)
            sl.append(dict(cache=c1, kmax=km1, kmin=kn1, q=d1["q"].contiguous(),
                           out=torch.empty((1, w1.n_q_heads, D), dtype=torch.bfloat16, device=dev),
                           wsd=rk.alloc_workspace(rk.OP_DENSE_DECODE, c1)))
            del d1
        nk1 = layers[0]["new_k"][:1].contiguous()
        nv1 = layers[0]["new_v"][:1].contiguous()
        single = {"workload": "llama8b_layer_32k: one layer, batch 1, 32q/8kv heads, context 32768, page 16, k1 32",
                  "us_per_layer_step": {}}
        for Tb in (256, 1024, 4096):
            for L in sl:
                L["ws"] = rk.alloc_workspace(rk.OP_HSA_DECODE, L["cache"], Tb)

            def one_all():
                for L in sl:
                    rk.hsa_decode_append(L["cache"], L["q"], nk1, nv1, L["kmax"], L["kmin"], w1.channel_budget, Tb, 0,
                                         L["out"], None, None, None, L["ws"], stream)

            single["us_per_layer_step"][str(Tb)] = round(timed_graph(one_all, 6) * 1e3 / len(sl), 2)

        def dense_one():
            for L in sl:
                rk.dense_decode(L["cache"], L["q"], L["out"], None, L["wsd"], stream)

        single["dense_full_kv_us"] = round(timed_graph(dense_one, 6) * 1e3 / len(sl), 2)
        del sl

    # ------------------------------------------------------------------ the same step at larger batches
    # Same model shape and budgets at batch 64 and 128 (512 / 1024 units): the fixed latencies of a
    # launch are shared by more K/V bytes, so this shows how far the same kernel gets towards the
    # roofline at production batch sizes.  Eight layers each (8 / 16 GiB of compressed cache).
    big = None
    if not args.no_decomposed and not args.batch and not args.layers:
        big = []
        w70 = wl.CONFIGS["llama70b_step_b16"]  # 64 query / 8 KV heads (G = 8), same cache per layer
        wmha = wl.scaled(w, n_kv_heads=w.n_q_heads)  # LongChat-7B-like: 32 heads, no grouping
        for Bb, wbase, label in ((4 * B, w, "same shape and budgets"), (8 * B, w, "same shape and budgets"),
                                 (w70.batch, w70, "llama70b_step_b16 shape (G = 8), same budgets"),
                                 (B, wmha, "multi-head shape (32 KV heads, G = 1), same budgets")):
            nlb = 8
            wb = wl.scaled(wbase, batch=Bb, n_layers=nlb)
            Hq_b, G_b, Hkv_b = wb.n_q_heads, wb.group, wb.n_kv_heads
            bl = []
            snapb_ws = None
            for layer in range(nlb):
                d = wl.generate_device(wb, layer, dev, with_obs=True)
                srcb = rk.pack_cache(d["K"], d["V"], d["seq_lens"].cpu().numpy(), Hq_b, ps)
                dstb = rk.alloc_cache(Bb, Hq_b, Hkv_b, D, ps, pages_cap, dev, zero=True)
                if snapb_ws is None:
                    snapb_ws = rk.alloc_workspace(rk.OP_SNAPKV, srcb, W, N)
                rk.snapkv_compress(d["qobs"], srcb, W, w.pool_kernel, N, dstb, None, snapb_ws)
                kmb, knb = rk.alloc_summaries(dstb)
                rk.build_page_summaries(dstb, kmb, knb)
                torch.cuda.synchronize()
                gen = torch.Generator(device=dev)
                gen.manual_seed(88_000 + layer)
                bl.append(dict(cache=dstb, kmax=kmb, kmin=knb, q=d["q"].contiguous(),
                               new_k=torch.randn((Bb, Hkv_b, D), generator=gen, device=dev).bfloat16(),
                               new_v=torch.randn((Bb, Hkv_b, D), generator=gen, device=dev).bfloat16(),
                               out=torch.empty((Bb, Hq_b, D), dtype=torch.bfloat16, device=dev),
                               ws=rk.alloc_workspace(rk.OP_HSA_DECODE, dstb, T)))
                del d, srcb
            del snapb_ws

            def big_all():
                for L in bl:
                    rk.hsa_decode_append(L["cache"], L["q"], L["new_k"], L["new_v"], L["kmax"], L["kmin"], k1, T,
                                         0, L["out"], None, None, None, L["ws"], stream)

            big_us = timed_graph(big_all, max(2, args.kernel_reps // 2)) * 1e3 / nlb
            rowb = rk.pages_row_len(bl[0]["cache"], T)
            big_lists = []
            for L in bl:
                pgb = torch.empty((Bb, Hkv_b, rowb), dtype=torch.int32, device=dev)
                rk.hsa_select(L["cache"], L["q"], L["kmax"], L["kmin"], k1, T, 0, pgb, None, None, stream)
                big_lists.append(pgb)
            big_sink = rk.stream_gather(bl[0]["cache"], big_lists[0])

            def big_gather():
                for L, pgb in zip(bl, big_lists):
                    rk.stream_gather(L["cache"], pgb, big_sink, stream)

            big_gather_us = timed_graph(big_gather, max(2, args.kernel_reps // 2)) * 1e3 / nlb
            del big_lists
            nb_now = int(bl[0]["cache"].seq_lens[0].item())
            Pb = (nb_now + ps - 1) // ps
            kpb = min(Pb, max(1, T // ps))
            big_bytes = Bb * Hkv_b * ((kpb * ps * D * 2 * 2 + 2 * G_b * D * 2)
                                    + (k1 * ((Pb + 7) // 8 * 8) * 2 + G_b * D * 2 + kpb * 4)
                                    + (2 * D * 2 + 2 * D * 2 * 2))
            big_gbs = big_bytes / (big_us * 1e-6) / 1e9
            big.append({"workload": f"{label}, batch {Bb}, {nlb} layers",
                        "us_per_layer_step": round(big_us, 3), "gather_probe_us": round(big_gather_us, 3),
                        "bytes_per_layer_step": big_bytes,
                        "achieved_GBs": round(big_gbs, 1), "frac_of_hbm_peak": round(big_gbs / HBM_PEAK_GBS, 4),
                        "decode_tokens_per_s_attention_only_all_layers":
                            round(Bb / (big_us * 1e-6 * wbase.n_layers), 1)})
            del bl
            torch.cuda.empty_cache()

    # ------------------------------------------------------------------ one long prompt, batch 1
    # BASELINE configs[3]: a single 131072-token prompt (32 query / 8 KV heads), SnapKV to 8192 tokens,
    # then decode steps with append at token budget 2048, against full-KV dense attention over the
    # 131072 tokens.  Eight layers (4.3 GB of uncompressed cache), eight units per launch.
    long_pt = None
    if not args.no_decomposed and not args.batch and not args.layers:
        wm = wl.CONFIGS["mistral_snap_128k"]
        nlm = 8
        ll, snapm_ws, snapm_ms = [], None, []
        for layer in range(nlm):
            d = wl.generate_device(wm, layer, dev, with_obs=True)
            srcm = rk.pack_cache(d["K"], d["V"], d["seq_lens"].cpu().numpy(), wm.n_q_heads, 16)
            dstm = rk.alloc_cache(1, wm.n_q_heads, wm.n_kv_heads, D, 16, (wm.snap_keep + 512) // 16, dev, zero=True)
            if snapm_ws is None:
                snapm_ws = rk.alloc_workspace(rk.OP_SNAPKV, srcm, wm.window, wm.snap_keep)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(stream):
                e0.record(stream)
                rk.snapkv_compress(d["qobs"], srcm, wm.window, wm.pool_kernel, wm.snap_keep, dstm, None, snapm_ws, stream)
                e1.record(stream)
                stream.synchronize()
            snapm_ms.append(e0.elapsed_time(e1))
            kmm, knm = rk.alloc_summaries(dstm)
            rk.build_page_summaries(dstm, kmm, knm)
            torch.cuda.synchronize()
            ll.append(dict(src=srcm, cache=dstm, kmax=kmm, kmin=knm, q=d["q"].contiguous(),
                           out=torch.empty((1, wm.n_q_heads, D), dtype=torch.bfloat16, device=dev),
                           ws=rk.alloc_workspace(rk.OP_HSA_DECODE, dstm, wm.token_budget),
                           wsd=rk.alloc_workspace(rk.OP_DENSE_DECODE, srcm)))
            del d
        nkm = layers[0]["new_k"][:1].contiguous()
        nvm = layers[0]["new_v"][:1].contiguous()

        def long_all():
            for L in ll:
                rk.hsa_decode_append(L["cache"], L["q"], nkm, nvm, L["kmax"], L["kmin"], wm.channel_budget,
                                     wm.token_budget, 0, L["out"], None, None, None, L["ws"], stream)

        def long_dense():
            for L in ll:
                rk.dense_decode(L["src"], L["q"], L["out"], None, L["wsd"], stream)

        long_us = timed_graph(long_all, 6) * 1e3 / nlm
        long_dense_us = timed_graph(long_dense, 6) * 1e3 / nlm
        long_pt = {"workload": f"mistral_snap_128k: batch 1, 32q/8kv heads, prompt {wm.context} -> SnapKV {wm.snap_keep}, "
                               f"budget {wm.token_budget}, page 16, k1 {wm.channel_budget}, {nlm} layers",
                   "us_per_layer_step": round(long_us, 2), "dense_full_kv_us": round(long_dense_us, 2),
                   "speedup_vs_dense_full_kv": round(long_dense_us / long_us, 2),
                   "snapkv_ms_per_layer": round(float(np.median(snapm_ms)), 3)}
        del ll, snapm_ws
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ bytes
    kp = min(P_now, T // ps)
    attend_bytes = units * (kp * ps * D * 2 * 2 + 2 * G * D * 2)
    select_bytes = units * (k1 * ((P_now + 7) // 8 * 8) * 2 + G * D * 2 + kp * 4)
    append_bytes = units * (2 * D * 2 + 2 * D * 2 * 2)
    hsa_bytes = attend_bytes + select_bytes + append_bytes
    dense_bytes = units * (w.context * D * 2 * 2 + 2 * G * D * 2)
    att_gbs = attend_bytes / (attend_us * 1e-6) / 1e9
    hsa_gbs = hsa_bytes / (us_layer * 1e-6) / 1e9
    dense_gbs = dense_bytes / (dense_us * 1e-6) / 1e9

    # ------------------------------------------------------------------ CPU oracle baseline
    cpu = None
    if not args.no_cpu:
        import oracle
        oracle.build()
        L0 = layers[0]
        nb = min(2, B)
        Kc, Vc = rk.unpack_cache(L0["cache"])
        Kh = wl.to_bits(Kc[:nb, :, :n_now])
        Vh = wl.to_bits(Vc[:nb, :, :n_now])
        qh = wl.to_bits(L0["q"][:nb])
        lens = np.full(nb, n_now, dtype=np.int32)
        oracle.hsa_decode(qh, Kh, Vh, lens, ps, k1, T)  # warm
        reps, t_cpu0 = 0, time.perf_counter()
        while True:
            oracle.hsa_decode(qh, Kh, Vh, lens, ps, k1, T)
            reps += 1
            el = time.perf_counter() - t_cpu0
            if el >= args.cpu_seconds:
                break
        per_call = el / reps
        cpu_us_layer = per_call * (B / nb) * 1e6
        cpu = {"value": round(cpu_us_layer, 1), "unit": "us/layer-step", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"{reps} calls of the fp64 oracle's whole Algorithm 1 (summaries rebuilt, select, "
                         f"attention) on {nb} of {B} sequences x {Hkv} KV heads of layer 0 at n={n_now}, "
                         f"scaled by {B}/{nb}; {el:.1f} s of CPU time"}

    # Stage 1 on the CPU: one oracle call on two sequences of the uncompressed prompt (16 units),
    # scaled to the batch: an extrapolated figure for one layer's SnapKV stage.
    cpu_snap = None
    if not args.no_cpu and n_dense > 0:
        Ld = dense_layers[0]
        nb = min(2, B)
        Kc, _ = rk.unpack_cache(Ld["cache"])
        Kh = wl.to_bits(Kc[:nb, :, :w.context])
        del Kc
        qo = wl.to_bits(Ld["qobs"][:nb])
        lens = np.full(nb, w.context, dtype=np.int32)
        t_s0 = time.perf_counter()
        oracle.snapkv(qo, Kh, lens, ks=w.pool_kernel, N=N)
        el_s = time.perf_counter() - t_s0
        cpu_snap = {"value": round(el_s * (B / nb) * 1e3, 1), "unit": "ms/layer (SnapKV stage)", "cores": oracle.num_threads(),
                    "kind": "oracle", "extrapolated": True,
                    "sample": f"one call of the fp64 oracle's Stage 1 (window scores, votes, pooling, top-k) on {nb} of {B} "
                              f"sequences x {Hkv} KV heads of layer 0, prompt {w.context}, window {W}, pooling {w.pool_kernel}, "
                              f"keep {N}, scaled by {B}/{nb}; {el_s:.1f} s of CPU time; the GPU stage takes "
                              f"{float(np.median(snap_ms)):.3f} ms"}

    # the paper's own budget t counts Step 2 and Step 3 traffic together (Section 3.6): tokens of exact
    # attention plus the summary rows read, in key/value-pair equivalents of 2 D values
    t_eq = T + P_now * k1 / (2.0 * D)
    kernel_name, traffic = measured_traffic(B)

    out = {
        "metric": "hsa_decode_us_per_layer_step",
        "value": round(us_layer, 3),
        "unit": "us/layer-step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(float(np.median(per_step_ms)), 4),
        "ms_per_step_min": round(float(per_step_ms.min()), 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"llama8b_step_b16: {w.n_layers} layers x (32q/8kv heads, d128), batch {B}, "
                               f"ctx {w.context} -> SnapKV {N} (+{n_now - N} appended), HSA budget {T}, "
                               f"page {ps}, k1 {k1}",
                   "graph": graph is not None, "query_sets_cycled": n_var,
                   "paper_equivalent_budget": round(t_eq, 1)},
        "decode_tokens_per_s_attention_only": round(B / (ms_per_step * 1e-3), 1),
        "hsa_achieved_GBs": round(hsa_gbs, 1),
        "hsa_frac_of_hbm_peak": round(hsa_gbs / HBM_PEAK_GBS, 4),
        "hsa_bytes_per_layer_step": hsa_bytes,
        "dense_full_kv_us_per_layer_step": round(dense_us, 2),
        "dense_achieved_GBs": round(dense_gbs, 1),
        "speedup_vs_dense_full_kv": round(dense_us / us_layer, 2),
        "snapkv_ms_per_layer": round(float(np.median(snap_ms)), 3),
        "host_wall_ms_per_step": round(wall_ms / args.steps, 4),
        "setup_s": round(t_setup, 1),
        "stage_us_per_layer": {"attend_only": round(attend_us, 3), "gather_probe": round(gather_us, 3),
                               "gather_probe_GBs": round(units * kp * ps * D * 2 * 2 / (gather_us * 1e-6) / 1e9, 1),
                               "select_only": round(select_us, 3),
                               "decode_no_append": round(decode_us, 3), "append_only": round(append_us, 3),
                               "attend_only_GBs": round(att_gbs, 1)},
        # the step is one launch of the fused kernel per layer, so its average launch time is the
        # timed region divided by the number of launches
        "roofline": {"bound": "hbm", "kernel": kernel_name or "hsa_decode_kernel", "achieved": round(hsa_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(hsa_gbs / HBM_PEAK_GBS, 4),
                     # from the committed counter summary when it covers this batch size, else null
                     "traffic": traffic, "us_per_launch": round(us_layer, 3),
                     "bytes_per_launch": hsa_bytes,
                     # what a plain streaming read reaches on this GPU, and the fraction of that
                     "measured_read_GBs": None if read_gbs is None else round(read_gbs, 1),
                     "frac_of_measured_read": None if read_gbs is None else round(hsa_gbs / read_gbs, 4)},
        "decomposed_operating_point": dec_pt,
        "long_prompt_batch1": long_pt,
        "multi_turn_variant": mt_pt,
        "single_layer_batch1": single,
        "other_shapes_and_batches": big,
        "cpu_baseline": cpu,
        "cpu_baseline_snapkv": cpu_snap,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
