#!/usr/bin/env python3
"""Benchmark of the E-Forest ADC hot path on one MI355X.

One step = one pass of the whole hot path over the workload's query batch: lookup tables ->
tree levels and leaf buckets of every tree -> forest reduction with the per-query bound ->
top-k selection.  Inputs (queries, index image, codebooks) are resident in HBM before the timed
region.  Prints one JSON line (the last line of stdout); progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
# HBM bytes per launch of the dominant kernel, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised
# under profiles/ (counters scaled by what a 1 GiB copy in the same run reads).  Keyed by (workload, kernel class,
# traversal); reported only for the exact configuration that was profiled.
MEASURED_TRAFFIC_BYTES = {("cfg2", "reduce", "register-context"): 9.362e9, ("cfg2", "lds", "lds-resident"): 0.545e9}
# LDS read bandwidth of the chip: 256 compute units x 256 bytes per clock x 2.4 GHz (a conflict-free 16-byte-per-lane
# wave read, 1 KiB, occupies the LDS pipe for 4 clocks: SQ_LDS_IDX_ACTIVE minus SQ_LDS_BANK_CONFLICT per read)
LDS_PEAK_GBS = 256 * 256 * 2.4
# vector float32 operations that are neither packed nor fused: a quarter of the published 157.3 TFLOP/s (which counts
# two-wide packed fused multiply-adds); a wave instruction takes 4 clocks on its 16-lane SIMD
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
TRAVERSAL_NAMES = {0: "register-context", 1: "level-synchronous", 2: "lds-resident"}
PAPER_CONTEXT = {              # the paper's own numbers: one Core i7 at 3.6 GHz, one query at a time, SIFT1M, M=8, K=256
    "hardware": "Intel Core i7 3.6 GHz (paper, section Experiments)",
    "ms_per_query": {"flat_adc": 2.678, "e_tree": 1.760, "e_forest_2": 1.265},
    "distances_per_s": {"flat_adc": 1e6 / 2.678e-3, "e_tree": 1e6 / 1.760e-3, "e_forest_2": 1e6 / 1.265e-3},
}


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def make_inputs(cfg, etf, torch, scale_n=None, scale_q=None):
    """Synthetic workload: library-trained codebooks, database encoded by the library's device encoder, queries.
    Returns the encode timing as well (set-up work, outside the benchmark's timed region)."""
    from workload import GaussianMixture, SEED_TRAIN, SEED_DATABASE, SEED_QUERIES
    gm = GaussianMixture.from_config(cfg)
    N = scale_n or cfg.N
    Q = scale_q or cfg.Q
    enc = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    t0 = time.time()
    enc.pq_train(gm.sample(cfg.n_train, SEED_TRAIN), cfg.M, cfg.K, cfg.kmeans_iters, seed=SEED_TRAIN)
    log("k-means (%d x %d, %d iters): %.1f s" % (cfg.n_train, cfg.d, cfg.kmeans_iters, time.time() - t0))
    enc.profile_enable(True)
    t0 = time.time()
    codes = np.empty((N, cfg.M), dtype=np.uint8)
    ws = torch.empty(enc.encode_workspace_bytes() + 256, dtype=torch.uint8, device="cuda")
    # the first launch of a kernel also loads its code: keep that out of the encoder's kernel time
    enc.pq_encode_device(torch.zeros((64, cfg.d), dtype=torch.float32, device="cuda"), ws=ws)
    enc.profile_read()
    done = 0
    for chunk in gm.chunks(N, SEED_DATABASE):
        got = enc.pq_encode_device(torch.from_numpy(chunk).cuda(), ws=ws)
        codes[done:done + len(chunk)] = got.cpu().numpy()
        done += len(chunk)
        if (done >> 17) % 64 == 0:
            log("  generated + encoded %d of %d vectors, %.0f s" % (done, N, time.time() - t0))
    ms, cnt = enc.profile_read()["encode"]
    flops = 3.0 * N * cfg.d * cfg.K          # subtract, multiply, add per (vector, codeword, dimension)
    encode = {"vectors": N, "kernel_ms": ms, "launches": cnt, "vectors_per_s": N / (ms / 1e3) if ms > 0 else None,
              "TFLOPs": flops / (ms / 1e3) / 1e12 if ms > 0 else None,
              "note": "device encoder kernel time only; generation on the host and the copies are not included"}
    log("generate + encode %d vectors: %.1f s (device encoder kernels %.1f ms, %.1f TFLOP/s)"
        % (N, time.time() - t0, ms, encode["TFLOPs"] or 0.0))
    queries = gm.sample(Q, SEED_QUERIES)
    return enc.pq_get_codebooks(), codes, queries, encode


def algorithmic_bytes(stats, mode, S, tiles):
    """Bytes each kernel class has to move for `tiles` tiles of 64 queries, from the index statistics:
    every partial-sum / result row is 256 bytes per tile and is counted once where consecutive
    nodes share it (children of one parent, encodings of one tree-0 leaf)."""
    M, K, T, N, Nd = stats["M"], stats["K"], stats["T"], stats["N"], stats["n_distinct"]
    row = 256
    out = {"lut": tiles * M * K * row}
    if mode == "flat":
        G = 1
        while M * K * (64 // G) * 4 > 128 * 1024:
            G *= 2
        out["flat"] = tiles * (G * N * M + M * K * row)
        out["sample"] = tiles * (S * (4 + M * G) + S * row + M * K * row)
        return out
    if mode == "forest_lds":
        # every table slice in LDS: per query and distinct encoding, one 4-byte LDS read per chunk below the
        # S-chunk prefix kept in the context, plus the S upper ones for the first encoding of every prefix
        tr0 = stats["trees"][0]
        D0 = tr0["D"]
        Sl = 2 if D0 >= 3 else D0 - 1
        prefixes = (tr0["nI"][Sl - 1] + sum(tr0["nL"][:Sl])) if Sl > 0 else 0
        out["lds"] = tiles * 64 * 4 * (Nd * (M - Sl) + Sl * prefixes)
        out["sample"] = tiles * 64 * 4 * S * M
        G = 2
        while M * K * (64 // G) * 4 > 128 * 1024:
            G *= 2
        out["lds_hbm"] = tiles * (M * K * row + G * Nd * M)   # what the same kernel has to read from HBM
        return out
    if mode == "forest_ctx":
        # register-context traversal: trees 1..T-1 each write one result row per leaf (reading a 4..16 byte
        # record per leaf and their table slices); the fused kernel reads, per distinct encoding, one row
        # of each of those tables, their leaf numbers and its tree-0 record, plus tree 0's table slices
        rec = lambda D: max(4, 1 << max(D - 1, 0).bit_length())
        trees = stats["trees"]
        out["leaf"] = tiles * sum(tr["L2"] * (row + rec(tr["D"])) + tr["D"] * K * row for tr in trees[1:])
        per_enc = (T - 1) * (row + 4) + rec(trees[0]["D"])
        out["reduce"] = tiles * (Nd * per_enc + trees[0]["D"] * K * row)
        out["sample"] = tiles * (S * (per_enc + 4) + trees[0]["D"] * K * row)
        return out
    level = leaf = 0
    for tr in stats["trees"]:
        D = tr["D"]
        for l in range(D):
            nI, nL = tr["nI"][l], tr["nL"][l]
            prev = tr["nI"][l - 1] if l > 0 else 0
            if nI:
                level += nI * 5 + nI * row + min(nI, prev) * row + K * row
            if nL:
                stride = (D - l + 3) // 4 * 4
                leaf += nL * (stride + 8) + nL * row + min(nL, prev) * row + (D - l) * K * row
    out["level"] = tiles * level
    out["leaf"] = tiles * leaf
    U0 = stats["trees"][0]["L2"]
    gather = (U0 + (T - 1) * Nd) * row if T > 1 else Nd * row
    out["reduce"] = tiles * (gather + (Nd * 4 * T if T > 1 else 0))
    out["sample"] = tiles * (S * 4 * (1 + (T if T > 1 else 0)) + S * T * row + S * row)
    return out


def time_search(ctx, qd, k, mode, warmup, steps, torch, ws, out_ids, out_dist, batch=0):
    """One step = the whole query set; `batch` > 0 sends it in consecutive calls of that many queries (a
    workload defined with batched queries), all inside the timed region."""
    Q = qd.shape[0]
    cuts = [(0, Q)] if not batch or batch >= Q else [(a, min(Q, a + batch)) for a in range(0, Q, batch)]

    def step():
        for a, b in cuts:
            ctx.search(qd[a:b], k, mode, out_ids[a:b], out_dist[a:b], ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_read()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt, ctx.profile_read()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--scale-n", type=int, default=0, help="override N (debugging only; invalidates the metric)")
    ap.add_argument("--scale-q", type=int, default=0, help="override Q (debugging only; invalidates the metric)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline and the parity spot check")
    ap.add_argument("--no-others", action="store_true", help="skip the flat and single-tree legs")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--levels", action="store_true",
                    help="same as --traversal 1: the level-synchronous traversal (partial sums of internal nodes in HBM)")
    ap.add_argument("--traversal", type=int, default=2, choices=[0, 1, 2],
                    help="2 every table slice in LDS (default), 0 distance context in registers + result tables, 1 level-synchronous")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=VALUE", help="library option for every context (tuning)")
    ap.add_argument("--no-copy", action="store_true", help="skip the 1 GiB device copy (bandwidth ceiling / counter calibration)")
    args = ap.parse_args()
    if args.levels:
        args.traversal = 1
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus %d is not supported); "
              "the path would shard by query tile (index replicated) or by ranges of the sorted encodings" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1509_05186_amd as etf
    from workload import get_config
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    etf.load_library()          # raises if the HIP library is missing: there is no fallback

    cfg = get_config(args.config)
    k = cfg.topk or 100
    cb, codes, queries, encode_info = make_inputs(cfg, etf, torch, args.scale_n or None, args.scale_q or None)
    N, Q = codes.shape[0], queries.shape[0]
    stream = torch.cuda.current_stream().cuda_stream
    qd = torch.from_numpy(queries).cuda()
    out_ids = torch.empty((Q, k), dtype=torch.int32, device="cuda")
    out_dist = torch.empty((Q, k), dtype=torch.float32, device="cuda")

    def make_ctx(T, traversal=None):
        c = etf.Context(device=0, stream=stream)
        c.set_option("traversal", args.traversal if traversal is None else traversal)
        for nv in args.opt:
            name, val = nv.split("=")
            c.set_option(name, int(val))
        c.pq_set_codebooks(cb)
        t0 = time.time()
        c.index_build(codes, T=T)
        c.index_upload()
        log("index T=%d: build + upload %.1f s, %.1f MB on device" % (T, time.time() - t0, c.index_device_bytes() / 1e6))
        c.profile_enable(not args.no_profile)
        return c

    T = max(cfg.trees, 1)
    tiles = (Q + 63) // 64
    mode = etf.ETF_MODE_FOREST

    def measure_forest(traversal, steps, warmup):
        """Times the E-Forest search with one traversal; returns the numbers of the JSON line."""
        forest = make_ctx(T, traversal)
        stats = forest.index_stats()
        ws = forest.alloc_workspace(Q, k, mode)
        log("traversal %s: workspace %.2f GB" % (TRAVERSAL_NAMES[traversal], ws.numel() / 1e9))
        dt, prof = time_search(forest, qd, k, mode, warmup, steps, torch, ws, out_ids, out_dist, cfg.query_batch)
        ms_step = dt / steps * 1e3
        value = N * Q * steps / dt
        fallbacks = forest.last_fallback_count()
        log("E-Forest(T=%d) top-%d, %s: %.2f ms/step, %.3e distances/s, %d queries via the exact kernel"
            % (T, k, TRAVERSAL_NAMES[traversal], ms_step, value, fallbacks))
        S = forest.index_layout().n_sample_enc
        lds_path = "lds" in prof and prof["lds"][1] > 0
        ctx_path = traversal != 1 and T <= 4
        alg = algorithmic_bytes(stats, "forest_lds" if lds_path else "forest_ctx" if ctx_path else "forest", S, tiles)
        kernels = {}
        for name, (ms, cnt) in prof.items():
            if cnt:
                kernels[name] = {"ms_per_step": ms / steps, "launches_per_step": cnt / steps,
                                 "alg_GB_per_step": alg.get(name, 0) / 1e9,
                                 "alg_GBps": (alg.get(name, 0) / 1e9) / (ms / steps / 1e3) if ms > 0 and name in alg else None}
        roofline = None
        if kernels:
            dom = max(kernels, key=lambda n: kernels[n]["ms_per_step"])
            kd = kernels[dom]
            lps = kd["launches_per_step"]
            achieved = kd["alg_GBps"] or 0.0
            traffic = None if (args.scale_n or args.scale_q) else MEASURED_TRAFFIC_BYTES.get((cfg.name, dom, TRAVERSAL_NAMES[traversal]))
            if dom == "lds":
                # bound by the LDS pipe: algorithmic bytes are the 4-byte table entries the method reads per query
                roofline = {"bound": "alu", "resource": "LDS read bandwidth", "kernel": dom, "achieved": achieved,
                            "peak": LDS_PEAK_GBS, "unit": "GB/s", "frac": achieved / LDS_PEAK_GBS, "traffic": traffic,
                            # the same figure on the vector unit: one float32 add per 4-byte entry, against
                            # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz of unpacked, unfused float32 operations
                            "alu": {"achieved": achieved / 4e3, "peak": VALU_PEAK_TOPS, "unit": "TFLOP/s",
                                    "frac": achieved / 4e3 / VALU_PEAK_TOPS}}
            else:
                roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic}
            roofline.update({"alg_bytes_per_launch": alg.get(dom, 0) / lps if lps else None,
                             "avg_launch_ms": kd["ms_per_step"] / lps if lps else None, "launches_per_step": lps})
            if dom != "lds":
                # the traversal as a whole (levels + leaves + reduction): the bandwidth figure of the table-based paths
                trav = [n for n in ("level", "leaf", "reduce", "sample") if n in kernels]
                tms = sum(kernels[n]["ms_per_step"] for n in trav)
                tgb = sum(kernels[n]["alg_GB_per_step"] for n in trav)
                roofline["traversal"] = {"kernels": trav, "ms_per_step": tms, "alg_GB_per_step": tgb,
                                         "alg_GBps": tgb / (tms / 1e3) if tms > 0 else None,
                                         "frac": (tgb / (tms / 1e3)) / HBM_PEAK_GBS if tms > 0 else None}
        res = {"ms_per_step": ms_step, "value": value, "fallbacks": fallbacks, "kernels": kernels, "roofline": roofline,
               "stats": stats, "S": int(S), "traversal": TRAVERSAL_NAMES[traversal]}
        del ws
        return res

    main_res = measure_forest(args.traversal, args.steps, args.warmup)
    got_ids, got_dist = out_ids.cpu().numpy(), out_dist.cpu().numpy()
    ms_step, value, fallbacks = main_res["ms_per_step"], main_res["value"], main_res["fallbacks"]
    kernels, roofline, stats, S = main_res["kernels"], main_res["roofline"], main_res["stats"], main_res["S"]

    # ---- a plain device copy of known size: achievable-bandwidth ceiling, and the reference dispatch
    #      against which the HBM byte counters are scaled
    copy = None
    if not args.no_copy:
        nbytes = 1 << 30
        src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        copy = {"bytes_read": nbytes, "bytes_written": nbytes, "ms": ms, "GBps": 2 * nbytes / 1e9 / (ms / 1e3)}
        log("device copy of 1 GiB: %.3f ms, %.0f GB/s (read + write)" % (ms, copy["GBps"]))
        del src, dst

    # ---- the same workload through the flat kernel and a single E-Tree, same run
    others = {}
    if not args.no_others:
        osteps = max(2, min(args.steps, 10))   # the other legs: up to ten steps after two warm-ups
        owarm = 2
        if args.traversal == 2:
            # the same E-Forest search through the table-based traversal (per-tree result tables in HBM)
            r0 = measure_forest(0, osteps, owarm)
            others["e_forest_register_context"] = {k2: r0[k2] for k2 in ("value", "ms_per_step", "kernels", "roofline")}
        tree = make_ctx(1)
        for name, ctx, m in (("flat_gpu", tree, etf.ETF_MODE_FLAT), ("e_tree_gpu", tree, etf.ETF_MODE_TREE)):
            w2 = ctx.alloc_workspace(Q, k, m)
            # The flat scan lists every copy of an encoding; where one encoding has more copies than a candidate
            # list holds, every query ends in the whole-database selection kernel: one untimed-warm-up-free step
            heavy = m == etf.ETF_MODE_FLAT and ctx.index_stats()["max_dup"] > 32768
            fw, fs = (0, 1) if heavy else (owarm, osteps)
            d2, p2 = time_search(ctx, qd, k, m, fw, fs, torch, w2, out_ids, out_dist, cfg.query_batch)
            others[name] = {"value": N * Q * fs / d2, "ms_per_step": d2 / fs * 1e3, "steps": fs,
                            "fallback_queries": ctx.last_fallback_count(),
                            "kernels_ms_per_step": {n: v[0] / fs for n, v in p2.items() if v[1]}}
            log("%s: %.2f ms/step, %.3e distances/s" % (name, others[name]["ms_per_step"], others[name]["value"]))
            del w2
        others["e_tree_stats"] = tree.index_stats()["trees"]
        del tree
        # the paper's study of the number of trees: forests of 4 and of M trees beside the tree and the forest above
        by_trees = {"1": others["e_tree_gpu"]["ms_per_step"], str(T): ms_step}
        for tt in (4, cfg.M):
            if str(tt) in by_trees or cfg.M % tt:
                continue
            fc = make_ctx(tt)
            wf = fc.alloc_workspace(Q, k, mode)
            df, _ = time_search(fc, qd, k, mode, owarm, osteps, torch, wf, out_ids, out_dist, cfg.query_batch)
            by_trees[str(tt)] = df / osteps * 1e3
            del fc, wf
        others["forest_ms_per_step_by_trees"] = by_trees
        log("E-Forest by number of trees (ms/step): %s" % ", ".join("T=%s %.2f" % kv for kv in sorted(by_trees.items(), key=lambda kv: int(kv[0]))))
        # control without structure: independent uniform codes (every encoding distinct, prefixes shared at the first
        # two levels only by chance): the worst case for the tree, on the same queries and codebooks
        rc = np.random.default_rng(1509).integers(0, cfg.K, size=(N, cfg.M), dtype=np.uint8)
        uc = etf.Context(device=0, stream=stream)
        uc.set_option("traversal", args.traversal)
        uc.pq_set_codebooks(cb)
        uc.index_build(rc, T=T)
        uc.index_upload()
        ust = uc.index_stats()
        wu = uc.alloc_workspace(Q, k, mode)
        du, _ = time_search(uc, qd, k, mode, owarm, osteps, torch, wu, out_ids, out_dist, cfg.query_batch)
        others["unstructured_control"] = {"ms_per_step": du / osteps * 1e3, "value": N * Q * osteps / du, "n_distinct": ust["n_distinct"],
                                          "lookups_per_encoding": sum(t["lookups"] for t in ust["trees"]) / N,
                                          "fallback_queries": uc.last_fallback_count()}
        log("control, uniform random codes: %.2f ms/step, %.3e distances/s (%d distinct, %.2f tree lookups per encoding)"
            % (du / osteps * 1e3, N * Q * osteps / du, ust["n_distinct"], others["unstructured_control"]["lookups_per_encoding"]))
        del uc, wu, rc
        # the other payload on the same forest: the k largest scalar products (option metric = 1)
        ipc = make_ctx(T)
        ipc.set_option("metric", 1)
        w4 = ipc.alloc_workspace(Q, k, mode)
        d4, p4 = time_search(ipc, qd, k, mode, owarm, osteps, torch, w4, out_ids, out_dist, cfg.query_batch)
        others["scalar_product_search"] = {"value": N * Q * osteps / d4, "ms_per_step": d4 / osteps * 1e3,
                                           "kernels_ms_per_step": {n: v[0] / osteps for n, v in p4.items() if v[1]},
                                           "fallback_queries": ipc.last_fallback_count()}
        log("largest scalar products, E-Forest(T=%d) top-%d: %.2f ms/step, %.3e products/s"
            % (T, k, others["scalar_product_search"]["ms_per_step"], others["scalar_product_search"]["value"]))
        del ipc, w4
        # chunk order: the greedy suggestion for this database, its lookup count and the search on an index in that order
        oc = etf.Context(device=0, stream=stream)
        oc.set_option("traversal", args.traversal)
        oc.pq_set_codebooks(cb)
        t0 = time.time()
        order, lk_given, lk_order = oc.suggest_chunk_order(codes, T=T)
        t_suggest = time.time() - t0
        oc.index_set_chunk_order(order)
        oc.index_build(codes, T=T)
        oc.index_upload()
        oc.profile_enable(not args.no_profile)
        w5 = oc.alloc_workspace(Q, k, mode)
        d5, p5 = time_search(oc, qd, k, mode, owarm, osteps, torch, w5, out_ids, out_dist, cfg.query_batch)
        others["chunk_order"] = {"order": [int(v) for v in order], "lookups_given_order": lk_given, "lookups_suggested_order": lk_order,
                                 "lookups_on": "at most 2^18 evenly spaced vectors", "suggest_s": t_suggest,
                                 "ms_per_step": d5 / osteps * 1e3, "n_distinct": oc.index_stats()["n_distinct"],
                                 "kernels_ms_per_step": {n: v[0] / osteps for n, v in p5.items() if v[1]}}
        log("chunk order %s: lookups %d -> %d (sample), search %.2f ms/step" % (others["chunk_order"]["order"], lk_given, lk_order, d5 / osteps * 1e3))
        del oc, w5
        if args.traversal == 2:
            # the same index built on the device from device-resident codes, and the same search on it
            db = etf.Context(device=0, stream=stream)
            db.pq_set_codebooks(cb)
            codes_d = torch.from_numpy(codes).cuda()
            nimg, nws = db.index_build_device_bytes(N, T)
            img = torch.empty(nimg + 256, dtype=torch.uint8, device="cuda")
            wsb = torch.empty(nws + 256, dtype=torch.uint8, device="cuda")
            times = []
            for _ in range(4):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                db.index_build_device(codes_d, T=T, image=img, ws=wsb)   # synchronises before it returns
                times.append((time.perf_counter() - t0) * 1e3)
            del wsb
            w3 = db.alloc_workspace(Q, k, mode)
            d3, _ = time_search(db, qd, k, mode, owarm, osteps, torch, w3, out_ids, out_dist, cfg.query_batch)
            others["index_build_device"] = {"ms": min(times[1:]), "vectors_per_s": N / (min(times[1:]) / 1e3),
                                            "image_bytes": db.index_device_bytes(), "image_bytes_bound": nimg, "workspace_bytes": nws,
                                            "search_ms_per_step": d3 / osteps * 1e3,
                                            "note": "sort, merge of repeats, level arrays of every tree, samples: wall clock of the call; "
                                                    "the search on the device-built index is the same kernels"}
            log("index build on the device: %.2f ms (%.3e vectors/s); search on it %.2f ms/step"
                % (min(times[1:]), N / (min(times[1:]) / 1e3), d3 / osteps * 1e3))
            del db, img, w3, codes_d
        if cfg.name == "cfg2" and not (args.scale_n or args.scale_q):
            # all-pairs output at a size where the output stream decides: this database, the first 2048 queries
            ta = make_ctx(T)
            nqa = min(Q, 2048)
            dista = torch.empty((nqa, N), dtype=torch.float32, device="cuda")
            wa = ta.alloc_workspace(nqa, 0, mode)
            for _ in range(2):
                ta.adc(qd[:nqa], mode, dista, wa)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                ta.adc(qd[:nqa], mode, dista, wa)
            torch.cuda.synchronize()
            msa = (time.perf_counter() - t0) / 5 * 1e3
            gbs = nqa * N * 4 / 1e9 / (msa / 1e3)
            others["all_pairs_forest"] = {"ms_per_step": msa, "value": nqa * N / (msa / 1e3), "output_GBps": gbs,
                                          "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                                       "frac": gbs / HBM_PEAK_GBS},
                                          "workload": "cfg2's database, first %d queries, E-Forest T=%d, every distance written in input order" % (nqa, T)}
            log("all pairs (cfg2 database, %d queries): %.2f ms/step, %.3e distances/s, %.0f GB/s of output" % (nqa, msa, nqa * N / (msa / 1e3), gbs))
            del ta, dista, wa
            # the all-pairs output row of the path: configuration 1 (single E-Tree, every distance written in
            # input order), its own inputs
            c1 = get_config("cfg1")
            cb1, codes1, q1, _ = make_inputs(c1, etf, torch)
            t1 = etf.Context(device=0, stream=stream)
            t1.pq_set_codebooks(cb1)
            t1.index_build(codes1, T=1)
            t1.index_upload()
            q1d = torch.from_numpy(q1).cuda()
            dist1 = torch.empty((q1.shape[0], codes1.shape[0]), dtype=torch.float32, device="cuda")
            w1 = t1.alloc_workspace(q1.shape[0], 0, etf.ETF_MODE_TREE)
            for _ in range(3):
                t1.adc(q1d, etf.ETF_MODE_TREE, dist1, w1)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                t1.adc(q1d, etf.ETF_MODE_TREE, dist1, w1)
            torch.cuda.synchronize()
            ms1 = (time.perf_counter() - t0) / 20 * 1e3
            nd1 = codes1.shape[0] * q1.shape[0]
            others["all_pairs_cfg1"] = {"ms_per_step": ms1, "value": nd1 / (ms1 / 1e3), "output_GBps": nd1 * 4 / 1e9 / (ms1 / 1e3),
                                        "workload": "cfg1: N=%d Q=%d, single E-Tree, all pairs in input order" % (codes1.shape[0], q1.shape[0])}
            log("all pairs (cfg1): %.3f ms/step, %.3e distances/s, %.0f GB/s of output" % (ms1, others["all_pairs_cfg1"]["value"], others["all_pairs_cfg1"]["output_GBps"]))
            del t1, dist1, w1

    # ---- CPU oracle on a bounded sample of the same workload, and parity of the timed output on it
    cpu = None
    if not args.no_cpu:
        import oracle
        from parity import assert_topk_matches
        nq = min(Q, 16)
        t0 = time.perf_counter()
        oracle.search(queries[:nq], cb, codes, k)
        t1 = time.perf_counter() - t0
        nq2 = int(min(Q, max(nq, min(4096, nq * 12.0 / max(t1, 1e-3)))))   # about 12 s of wall clock on the host cores
        t0 = time.perf_counter()
        oracle.search(queries[:nq2], cb, codes, k)
        t2 = time.perf_counter() - t0
        cpu = {"value": N * nq2 / t2, "unit": "encoding-distances/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "first %d of %d queries against all %d encodings (float64 flat ADC + full-sort top-%d), %.1f s"
                         % (nq2, Q, N, k, t2)}
        log("CPU oracle: %.3e distances/s on %d threads (%s)" % (cpu["value"], cpu["cores"], cpu["sample"]))
        npar = min(Q, 24)
        ref = oracle.adc_all(queries[:npar], cb, codes)
        for j in range(npar):
            assert_topk_matches(got_ids[j], got_dist[j], ref[j], np.arange(N), k, "bench q%d" % j)
        # plus a spread of queries from the rest of the batch (other tiles, the ragged last tile)
        rest = np.unique(np.linspace(npar, Q - 1, 8).astype(int)) if Q > npar else []
        for j in rest:
            r = oracle.adc_all(queries[j:j + 1], cb, codes)[0]
            assert_topk_matches(got_ids[j], got_dist[j], r, np.arange(N), k, "bench q%d" % j)
        log("parity of the timed output against the oracle: ok on %d queries" % (npar + len(rest)))

    line = {
        "metric": "encoding-distances/sec (batched queries), E-Forest ADC + top-k, 1 GPU",
        "value": value, "unit": "encoding-distances/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: d=%d N=%d Q=%d PQ M=%d K=%d, E-Forest T=%d, top-%d, seeded %d-component Gaussian mixture"
                               % (cfg.name, cfg.d, N, Q, cfg.M, cfg.K, T, k, cfg.components),
                   "traversal": TRAVERSAL_NAMES[args.traversal], "query_batch": cfg.query_batch or Q,
                   "valid": not (args.scale_n or args.scale_q)},
        "roofline": roofline,
        # the table-based E-Forest traversal of the same run (per-tree result tables in HBM): the HBM-bandwidth figure
        "roofline_hbm_traversal": (others.get("e_forest_register_context") or {}).get("roofline"),
        "cpu_baseline": cpu,
        "kernels": kernels, "others": others, "encode_gpu": encode_info, "fallback_queries": fallbacks, "device_copy": copy,
        "index": {"n_distinct": stats["n_distinct"], "max_dup": stats["max_dup"], "device_MB": stats["device_bytes"] / 1e6,
                  "trees": stats["trees"], "sample": int(S)},
        "paper_context": PAPER_CONTEXT,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
