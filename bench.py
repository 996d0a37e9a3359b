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
# Each figure carries the hash of the kernel sources it was measured on (kernel_source_hash below); a run on other
# sources prints traffic: null.
MEASURED_TRAFFIC_BYTES = {
    ("cfg2", "lds16", "lds-resident"): (482.4e6, "4195ef506fb42311"),       # profiles/cfg2_forest_lds_resident.md
    ("cfg2", "reduce", "register-context"): (9.343e9, "4195ef506fb42311"),  # profiles/cfg2_forest_register_context.md
    ("cfg4", "lds16", "lds-resident"): (3.054e9, "4195ef506fb42311"),       # profiles/cfg4_forest_lds_resident.md
}
# LDS read bandwidth of the chip: 256 compute units x 256 bytes per clock x 2.4 GHz (a conflict-free 16-byte-per-lane
# wave read, 1 KiB, occupies the LDS pipe for 4 clocks: SQ_LDS_IDX_ACTIVE minus SQ_LDS_BANK_CONFLICT per read)
LDS_PEAK_GBS = 256 * 256 * 2.4
# Vector instructions: a float32 add, multiply or fused multiply-add issues for 128 lanes per clock and compute unit
# (the probe ETF_PROBE_VALU_F32 measures 2 wave instructions per CU-clock; the published 157.3 TFLOP/s is that rate
# with packed two-wide fused multiply-adds, four flops per lane); v_add3_u32 and the packed 16-bit operations issue
# for 64 lanes per clock (1 wave instruction per CU-clock; probes ETF_PROBE_VALU_ADD3, _PK16).
VALU_F32_PEAK_TOPS = 256 * 128 * 2.4e9 / 1e12     # single float32 operations per second, nominal clock
VALU_HALF_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12     # v_add3_u32 / v_pk_* lane instructions per second, nominal clock
VALU_PEAK_NOTE = "256 CUs x 128 lanes x 2.4 GHz of single float32 vector operations (not packed, not fused)"
CEILINGS = {}   # this run's probe results (measure_ceilings), filled in before the first timed search
TRAVERSAL_NAMES = {0: "register-context", 1: "level-synchronous", 2: "lds-resident"}
PATH_NOTES = {
    0: "E-Forest: depth-first leaf order with the distance context in registers, per-tree result tables in HBM summed per encoding",
    1: "E-Forest: level-synchronous kernels over the level arrays, per-tree result tables in HBM summed per encoding",
    2: "sorted distinct encodings scanned with every table slice in LDS and a distance context of two levels; the trees' "
       "sums are formed per encoding in registers (no per-tree result array); see roofline.lookups_per_query.  With "
       "kernel lds16 in `kernels` the scan that picks candidates runs on 16-bit fixed-point copies of the tables "
       "(entries rounded down, bound rounded up: nothing at or below the bound is lost) and every returned distance is "
       "recomputed as the float32 sum of the float32 table entries",
}
PAPER_CONTEXT = {              # the paper's own numbers: one Core i7 at 3.6 GHz, one query at a time, SIFT1M, M=8, K=256
    "hardware": "Intel Core i7 3.6 GHz (paper, section Experiments)",
    "ms_per_query": {"flat_adc": 2.678, "e_tree": 1.760, "e_forest_2": 1.265},
    "distances_per_s": {"flat_adc": 1e6 / 2.678e-3, "e_tree": 1e6 / 1.760e-3, "e_forest_2": 1e6 / 1.265e-3},
}


def lds_alu(tadds, eb):
    """The adds of a scan kernel (one per table entry, `tadds` T entries/s) against the vector units' rate for the
    instruction that does them: v_add_f32 for 4-byte entries (one entry per lane instruction), v_add3_u32 for 2-byte
    entries (two additions of two packed entries each per lane instruction)."""
    if eb == 4:
        peak, key, what = VALU_F32_PEAK_TOPS, "valu_v_add_f32_Tlane_instr_per_s", "one v_add_f32 per entry; " + VALU_PEAK_NOTE
        per = 1
    else:
        peak, key, per = VALU_HALF_PEAK_TOPS * 4, "valu_v_add3_u32_Tlane_instr_per_s", 4
        what = "four entry additions per v_add3_u32 lane instruction; 256 CUs x 64 lanes x 2.4 GHz of those"
    meas = CEILINGS.get(key)
    return {"achieved": tadds, "peak": peak, "unit": "Tadd/s", "frac": tadds / peak, "note": what,
            "measured_peak": meas * per if meas else None, "frac_of_measured_peak": tadds / (meas * per) if meas else None}


def kernel_source_hash():
    """Identifies the kernel sources a profile was taken on: sha256 over the library's source files, 16 hex digits."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1509_05186_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):     # what the kernels are compiled from; host-only .cpp files do not move a profile
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel, traversal):
    """(bytes per launch, note) from the rocprofv3 counter runs, or (None, why not)."""
    ent = MEASURED_TRAFFIC_BYTES.get((workload, kernel, traversal))
    if ent is None:
        return None, "no counter run recorded for this workload and kernel"
    nbytes, src = ent
    if src != kernel_source_hash():
        return None, "the recorded counter run (%.3e bytes) was taken on kernel sources %s, this run uses %s" % (nbytes, src, kernel_source_hash())
    return nbytes, "rocprofv3 FETCH_SIZE + WRITE_SIZE on kernel sources %s, see profiles/" % src


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


EXTRA_OPTS = []   # --opt NAME=VALUE pairs, applied to the encoding context as well


def make_inputs(cfg, etf, torch, scale_n=None, scale_q=None):
    """Synthetic workload: library-trained codebooks, database encoded by the library's device encoder, queries.
    Returns the encode timing as well (set-up work, outside the benchmark's timed region)."""
    from workload import GaussianMixture, SEED_TRAIN, SEED_DATABASE, SEED_QUERIES
    gm = GaussianMixture.from_config(cfg)
    N = scale_n or cfg.N
    Q = scale_q or cfg.Q
    enc = etf.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    plain = False
    for nv in EXTRA_OPTS:
        name, val = nv.split("=")
        enc.set_option(name, int(val))
        plain = plain or (name == "encode_kernel" and int(val) == 1)
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
    held, held_n = [], 0   # generated chunks already on the device, encoded a million vectors per call
    def flush():
        nonlocal done, held, held_n
        if not held:
            return
        got = enc.pq_encode_device(held[0] if len(held) == 1 else torch.cat(held), ws=ws)
        codes[done:done + held_n] = got.cpu().numpy()
        done += held_n
        held, held_n = [], 0
        if (done >> 20) % 8 == 0:
            log("  generated + encoded %d of %d vectors, %.0f s" % (done, N, time.time() - t0))
    for chunk in gm.chunks_threaded(N, SEED_DATABASE, 12):
        held.append(torch.from_numpy(chunk).cuda())
        held_n += len(chunk)
        if held_n >= (1 << 20):
            flush()
    flush()
    ms, cnt = enc.profile_read()["encode"]
    # plain kernel: subtract, multiply, add per (vector, codeword, dimension), three unfused vector instructions;
    # matrix-core kernel: the contraction x.c, two operations per (vector, codeword, dimension)
    flops = (3.0 if plain else 2.0) * N * cfg.d * cfg.K
    encode = {"vectors": N, "kernel_ms": ms, "launches": cnt, "vectors_per_s": N / (ms / 1e3) if ms > 0 else None,
              "kernel": "float32 rule for every codeword (vector unit)" if plain else "distances on the matrix cores, near-ties by the float32 rule",
              "TFLOPs": flops / (ms / 1e3) / 1e12 if ms > 0 else None,
              "ops_counted": "3 N d K unfused vector operations" if plain else "2 N d K of the float32 contraction",
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
        out["lds16"] = out["lds"] // 2      # the same entries as 16-bit ones (k_lds16)
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


class Workload:
    """One configuration's inputs, resident on the device: codebooks, codes, queries, output buffers."""

    def __init__(self, cfg, etf, torch, args, scale_n=None, scale_q=None):
        self.cfg, self.etf, self.torch, self.args = cfg, etf, torch, args
        self.k = cfg.topk or 100
        self.cb, self.codes, self.queries, self.encode_info = make_inputs(cfg, etf, torch, scale_n, scale_q)
        self.N, self.Q = self.codes.shape[0], self.queries.shape[0]
        self.stream = torch.cuda.current_stream().cuda_stream
        self.qd = torch.from_numpy(self.queries).cuda()
        self.out_ids = torch.empty((self.Q, self.k), dtype=torch.int32, device="cuda")
        self.out_dist = torch.empty((self.Q, self.k), dtype=torch.float32, device="cuda")
        self.T = max(cfg.trees, 1)
        self.tiles = (self.Q + 63) // 64
        self.codes_d = None
        self.valid = not (scale_n or scale_q)
        self._tree_lookups = None

    def make_ctx(self, T, traversal=None, profile=True, opts=()):
        """A context with an index of T trees over this database: built on the device for the large databases
        (the host builder takes seconds there), on the host otherwise."""
        etf, torch, args = self.etf, self.torch, self.args
        c = etf.Context(device=0, stream=self.stream)
        c.set_option("traversal", args.traversal if traversal is None else traversal)
        for nv in list(args.opt) + list(opts):
            name, val = nv.split("=")
            c.set_option(name, int(val))
        c.pq_set_codebooks(self.cb)
        t0 = time.time()
        if self.N >= 5_000_000:
            if self.codes_d is None:
                self.codes_d = torch.from_numpy(self.codes).cuda()
            c.index_build_device(self.codes_d, T=T)
            how = "built on the device"
        else:
            c.index_build(self.codes, T=T)
            c.index_upload()
            how = "build + upload"
        log("%s index T=%d: %s %.1f s, %.1f MB on device" % (self.cfg.name, T, how, time.time() - t0, c.index_device_bytes() / 1e6))
        c.profile_enable(profile and not args.no_profile)
        return c

    def tree_lookups(self):
        """Table lookups of one traversal of the single E-Tree over this database, L1 + L2 + sum of the postfix
        lengths: the paper's measure of the method's work, whatever the kernels do."""
        if self._tree_lookups is None:
            c = self.make_ctx(1, profile=False)
            self._tree_lookups = int(c.index_stats()["trees"][0]["lookups"])
            del c
        return self._tree_lookups

    def measure_search(self, T, traversal, steps, warmup, mode=None):
        """Times the search with one traversal; returns the numbers of a JSON leg."""
        etf, torch, cfg = self.etf, self.torch, self.cfg
        mode = etf.ETF_MODE_FOREST if mode is None else mode
        ctx = self.make_ctx(T, traversal)
        stats = ctx.index_stats()
        Qc = cfg.query_batch or self.Q
        ws = ctx.alloc_workspace(min(Qc, self.Q), self.k, mode)
        log("%s traversal %s: workspace %.2f GB" % (cfg.name, TRAVERSAL_NAMES[traversal], ws.numel() / 1e9))
        dt, prof = time_search(ctx, self.qd, self.k, mode, warmup, steps, torch, ws, self.out_ids, self.out_dist, cfg.query_batch)
        ms_step = dt / steps * 1e3
        value = self.N * self.Q * steps / dt
        fallbacks = ctx.last_fallback_count()
        log("%s T=%d top-%d, %s: %.2f ms/step, %.3e distances/s, %d queries of the last call via the exact kernel"
            % (cfg.name, T, self.k, TRAVERSAL_NAMES[traversal], ms_step, value, fallbacks))
        S = ctx.index_layout().n_sample_enc
        lds_path = any(n in prof and prof[n][1] > 0 for n in ("lds", "lds16"))
        ctx_path = traversal != 1 and T <= 4
        alg = algorithmic_bytes(stats, "forest_lds" if lds_path else "forest_ctx" if ctx_path else "forest", S, self.tiles)
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
            traffic, traffic_note = (None, "scaled run") if not self.valid else measured_traffic(cfg.name, dom, TRAVERSAL_NAMES[traversal])
            if dom in ("lds", "lds16"):
                # bound by the LDS pipe and the vector adds behind it: algorithmic bytes are the table entries this kernel
                # reads from LDS per query, 4 bytes each in k_lds, 2 bytes each in k_lds16
                eb = 4 if dom == "lds" else 2
                kernel_lookups = alg[dom] / (self.tiles * 64 * eb)
                tree_lookups = self.tree_lookups()
                forest_lookups = sum(t["lookups"] for t in stats["trees"])
                frac = achieved / LDS_PEAK_GBS
                ceil = CEILINGS.get("lds_read_b128_scattered_rows_GBps")
                roofline = {"bound": "alu", "resource": "LDS read bandwidth (on-chip): the kernel is a sequence of 16-byte table reads, "
                                                        "one add per %d-byte entry" % eb, "kernel": dom, "entry_bytes": eb,
                            "achieved": achieved, "peak": LDS_PEAK_GBS, "unit": "GB/s", "frac": frac,
                            "frac_of_measured_ceiling": achieved / ceil if ceil else None,
                            "measured_ceiling": {"GBps": ceil, "what": "ds_read_b128 of scattered 64-byte rows, this run's probe"} if ceil else None,
                            "traffic": traffic, "traffic_note": traffic_note,
                            "lookups_per_s": achieved * 1e9 / eb,
                            # the same time priced on the lookups the paper's single E-Tree needs for this database
                            # (L1 + L2 + postfix lengths): prefixes this kernel recomputes are not useful work
                            "method_frac": frac * tree_lookups / kernel_lookups,
                            "lookups_per_query": {"this_kernel": kernel_lookups, "e_tree": tree_lookups,
                                                  "e_forest_trees": forest_lookups, "flat_distinct": stats["n_distinct"] * stats["M"],
                                                  "flat": stats["N"] * stats["M"]},
                            "alu": lds_alu(achieved / eb / 1e3, eb)}
            else:
                roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_note": traffic_note}
            roofline.update({"alg_bytes_per_launch": alg.get(dom, 0) / lps if lps else None,
                             "avg_launch_ms": kd["ms_per_step"] / lps if lps else None, "launches_per_step": lps})
            if dom not in ("lds", "lds16"):
                # the traversal as a whole (levels + leaves + reduction): the bandwidth figure of the table-based paths
                trav = [n for n in ("level", "leaf", "reduce", "sample") if n in kernels]
                tms = sum(kernels[n]["ms_per_step"] for n in trav)
                tgb = sum(kernels[n]["alg_GB_per_step"] for n in trav)
                roofline["traversal"] = {"kernels": trav, "ms_per_step": tms, "alg_GB_per_step": tgb,
                                         "alg_GBps": tgb / (tms / 1e3) if tms > 0 else None,
                                         "frac": (tgb / (tms / 1e3)) / HBM_PEAK_GBS if tms > 0 else None}
        res = {"ms_per_step": ms_step, "value": value, "fallbacks": fallbacks, "kernels": kernels, "roofline": roofline,
               "stats": stats, "S": int(S), "traversal": TRAVERSAL_NAMES[traversal], "steps": steps}
        del ws, ctx
        return res

    def parity(self, picks, what):
        """The timed output (self.out_ids / out_dist) of the queries `picks` against the oracle's distances to every
        encoding, one query at a time."""
        import oracle
        from parity import assert_topk_matches_identity
        ids, dist = self.out_ids.cpu().numpy(), self.out_dist.cpu().numpy()
        if self.valid and not getattr(self, "codes_checked", False):
            # the codes are the device encoder's: a stretch of them against the oracle's float32 rule, once
            from workload import GaussianMixture, SEED_DATABASE
            x0 = next(iter(GaussianMixture.from_config(self.cfg).chunks(self.N, SEED_DATABASE)))[:5000]
            assert np.array_equal(oracle.encode_f32(x0, self.cb), self.codes[:len(x0)]), "device-encoded codes differ from the oracle's"
            self.codes_checked = True
        for j in picks:
            ref = oracle.adc_all(self.queries[j:j + 1], self.cb, self.codes)[0]
            assert_topk_matches_identity(ids[j], dist[j], ref, self.k, "%s q%d" % (what, j))
        log("%s: parity of the timed output against the oracle ok on queries %s" % (what, list(map(int, picks))))
        return [int(j) for j in picks]


def workload_string(wl, T):
    cfg = wl.cfg
    return ("%s: d=%d N=%d Q=%d PQ M=%d K=%d, E-Forest T=%d, top-%d, seeded %d-component Gaussian mixture"
            % (cfg.name, cfg.d, wl.N, wl.Q, cfg.M, cfg.K, T, wl.k, cfg.components))


def config_leg(name, etf, torch, args, steps, warmup):
    """Another configuration of the workload list, end to end in the same run: inputs, index, the default search
    timed over `steps` steps (queries in calls of the configuration's batch size), roofline of its dominant kernel,
    and a parity check of the timed output on a few spread-out queries."""
    from workload import get_config
    cfg = get_config(name)
    t0 = time.time()
    wl = Workload(cfg, etf, torch, args)
    res = wl.measure_search(wl.T, args.traversal, steps, warmup)
    leg = {"workload": workload_string(wl, wl.T), "query_batch": cfg.query_batch or wl.Q, "steps": steps, "warmup": warmup,
           "value": res["value"], "unit": "encoding-distances/s", "ms_per_step": res["ms_per_step"], "roofline": res["roofline"],
           "kernels": res["kernels"], "fallback_queries": res["fallbacks"], "encode_gpu": wl.encode_info,
           "index": {"n_distinct": res["stats"]["n_distinct"], "max_dup": res["stats"]["max_dup"],
                     "trees": [{kk: t[kk] for kk in ("D", "L1", "L2", "sumP", "lookups")} for t in res["stats"]["trees"]],
                     "sample": res["S"]}}
    if not args.no_cpu:
        Q = wl.Q
        picks = sorted(set([0, min(Q - 1, 255), min(Q - 1, 256), Q // 2, Q - 1]))
        leg["parity_checked_queries"] = wl.parity(picks, name + " E-Forest")
    if name == "cfg3":
        # this configuration times the single E-Tree as well
        rt = wl.measure_search(1, args.traversal, steps, warmup, etf.ETF_MODE_TREE)
        leg["e_tree"] = {"value": rt["value"], "ms_per_step": rt["ms_per_step"], "roofline": rt["roofline"], "kernels": rt["kernels"]}
        if not args.no_cpu:
            wl.parity([0, wl.Q // 2, wl.Q - 1], name + " E-Tree")
    leg["wall_s"] = time.time() - t0
    del wl
    torch.cuda.empty_cache()
    return leg


def ivf_leg(etf, torch, args, steps, warmup):
    """IVFADC on cfg2's vectors with the configuration the paper's application experiment quotes (K' = 8192 cells,
    w = 64 probed lists, residual PQ M = 8, K = 256), top-100 for all queries: coarse distances and probe selection,
    scalar-product tables, scan of the probed lists (merged, sorted entries), selection.  The coarse quantiser is
    8192 vectors drawn from the mixture (no k-means at that size on the host); codebooks are trained on residuals."""
    from workload import GaussianMixture, get_config, SEED_TRAIN, SEED_DATABASE, SEED_QUERIES
    cfg = get_config("cfg2")
    cells_n, w, k = 8192, 64, 100
    gm = GaussianMixture.from_config(cfg)
    stream = torch.cuda.current_stream().cuda_stream
    t0 = time.time()
    cent = gm.sample(cells_n, 77)
    xt = gm.sample(cfg.n_train, SEED_TRAIN)
    shape = etf.Context(device=0, stream=stream)           # codebooks of the right shape give the context d, M, K
    shape.pq_set_codebooks(np.zeros((cfg.M, cfg.K, cfg.d // cfg.M), dtype=np.float32))
    shape.ivf_set_coarse(cent)
    tc = shape.ivf_assign_device(torch.from_numpy(xt).cuda())[0].cpu().numpy()
    trainer = etf.Context(device=None)
    trainer.pq_train(xt - cent[tc], cfg.M, cfg.K, cfg.kmeans_iters, seed=SEED_TRAIN)
    cb = trainer.pq_get_codebooks()
    c = etf.Context(device=0, stream=stream)
    for nv in args.opt:
        name, val = nv.split("=")
        c.set_option(name, int(val))
    c.pq_set_codebooks(cb)
    c.ivf_set_coarse(cent)
    cells = np.empty(cfg.N, dtype=np.int32)
    codes = np.empty((cfg.N, cfg.M), dtype=np.uint8)
    done = 0
    c.profile_enable(True)
    c.profile_read()
    for chunk in gm.chunks_threaded(cfg.N, SEED_DATABASE, 12):
        ce, co = c.ivf_assign_device(torch.from_numpy(chunk).cuda())
        cells[done:done + len(chunk)] = ce.cpu().numpy()
        codes[done:done + len(chunk)] = co.cpu().numpy()
        done += len(chunk)
    assign_ms = c.profile_read()["encode"][0]
    c.ivf_build(cells, codes)
    c.ivf_upload()
    st = c.ivf_stats()
    queries = gm.sample(cfg.Q, SEED_QUERIES)
    qd = torch.from_numpy(queries).cuda()
    out_ids = torch.empty((cfg.Q, k), dtype=torch.int32, device="cuda")
    out_dist = torch.empty((cfg.Q, k), dtype=torch.float32, device="cuda")
    ws = torch.empty(c.ivf_workspace_bytes(cfg.Q, k, w) + 256, dtype=torch.uint8, device="cuda")
    log("IVFADC set-up %.1f s: %d cells, %d entries for %d vectors, largest list %d, workspace %.2f GB"
        % (time.time() - t0, st["cells"], st["entries"], st["N"], st["max_list"], ws.numel() / 1e9))
    for _ in range(warmup):
        c.ivf_search(qd, k, w, out_ids, out_dist, ws)
    torch.cuda.synchronize()
    c.profile_read()
    t0 = time.perf_counter()
    for _ in range(steps):
        c.ivf_search(qd, k, w, out_ids, out_dist, ws)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = c.profile_read()
    kernels = {n: {"ms_per_step": v[0] / steps, "launches_per_step": v[1] / steps} for n, v in prof.items() if v[1]}
    ms = dt / steps * 1e3
    # what one step evaluates: every entry of every probed list of every query
    pr_cells = None
    scanned = None
    leg = {"workload": "cfg2's vectors (d=%d N=%d Q=%d), IVFADC: %d cells, w=%d, residual PQ M=%d K=%d, top-%d"
                       % (cfg.d, cfg.N, cfg.Q, cells_n, w, cfg.M, cfg.K, k),
           "ms_per_step": ms, "queries_per_s": cfg.Q / (ms / 1e3), "steps": steps, "kernels": kernels,
           "fallback_queries": c.last_fallback_count(), "index": st, "assign_gpu_kernel_ms": assign_ms,
           "coarse_quantiser": "8192 vectors drawn from the mixture, not trained"}
    # rooflines of the two large kernel classes.  Coarse: the query-centroid products are a dense float32 contraction
    # on the matrix cores (2 Q K' d operations); the class also holds the probe selection, which re-evaluates the cells
    # near the w-th by the sequential float32 rule.  Scan: 4-byte table entries gathered from LDS, M per entry.
    if "ivf_coarse" in kernels:
        ach = 2.0 * cfg.Q * cells_n * cfg.d / (kernels["ivf_coarse"]["ms_per_step"] / 1e3) / 1e12
        meas = CEILINGS.get("mfma_f32_32x32x2_TFLOPs")
        leg["roofline_coarse"] = {"bound": "mfma", "kernel": "ivf_coarse (k_ivf_coarse_tc and k_ivf_probe_mfma together)",
                                  "dtype": "f32", "achieved": ach, "peak": 157.3, "unit": "TFLOP/s", "frac": ach / 157.3, "traffic": None,
                                  "frac_of_measured_peak": ach / meas if meas else None}
    if not args.no_cpu:
        from oracle import ivfadc
        from parity import assert_topk_matches
        picks = [0, 63, 64, cfg.Q // 2, cfg.Q - 1]
        ids_h, dist_h = out_ids.cpu().numpy(), out_dist.cpu().numpy()
        # the database side came from the device assignment: a stretch of it against the oracle's
        x0 = next(iter(gm.chunks(cfg.N, SEED_DATABASE)))[:300]
        oc, oe = ivfadc.build(x0, cent, cb)
        assert np.array_equal(oc, cells[:len(x0)]) and np.array_equal(oe, codes[:len(x0)]), "device assignment differs from the oracle's"
        leg["assignment_checked"] = "first %d vectors: cells and residual codes == oracle" % len(x0)
        xhat = ivfadc.reconstruct(cent, cb, cells, codes)
        pr = ivfadc.probes(queries[picks], cent, w)
        scanned = 0
        for jj, j in enumerate(picks):
            inside = np.flatnonzero(np.isin(cells, pr[jj]))
            scanned += len(inside)
            diff = xhat[inside] - queries[j].astype(np.float64)
            ref = np.einsum("ij,ij->i", diff, diff)
            assert_topk_matches(ids_h[j], dist_h[j], ref, inside, k, "bench ivf q%d" % j)
        leg["parity_checked_queries"] = picks
        leg["vectors_in_probed_lists_per_query"] = scanned / len(picks)
        if "ivf_scan" in kernels:
            gbs = scanned / len(picks) * cfg.Q * cfg.M * 4.0 / (kernels["ivf_scan"]["ms_per_step"] / 1e3) / 1e9
            leg["roofline_scan"] = {"bound": "alu", "resource": "LDS reads (on-chip): one gathered 4-byte table entry per chunk of every entry of the probed lists, counted once",
                                    "kernel": "ivf_scan", "achieved": gbs, "peak": LDS_PEAK_GBS, "unit": "GB/s", "frac": gbs / LDS_PEAK_GBS, "traffic": None,
                                    "note": "entries per query from the %d checked queries; the kernel evaluates the nearest lists a second time for its bound" % len(picks)}
        log("IVFADC: parity of the timed output against the oracle ok on queries %s" % picks)
    log("IVFADC (8192 cells, w=64) top-100: %.2f ms/step, %.3e queries/s; kernels %s"
        % (ms, leg["queries_per_s"], {n: round(v["ms_per_step"], 3) for n, v in kernels.items()}))
    return leg


def measure_ceilings(etf, torch, stream):
    """What this card's memory delivers to plain streaming kernels (the library's probe kernels): sequential reads,
    writes, a copy, and scattered 256-byte rows, over a 4 GiB window (HBM) and a 64 MiB window (inside the memory-side
    cache)."""
    c = etf.Context(device=0, stream=stream)
    out = {}
    for label, nbytes in (("4GiB", 4 << 30), ("64MiB", 64 << 20)):
        a = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        b = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        a.view(torch.float32).normal_()
        reps = 5 if nbytes > (1 << 30) else 50
        for kind, kname, moved in ((etf.ETF_PROBE_READ, "read", nbytes), (etf.ETF_PROBE_WRITE, "write", nbytes),
                                   (etf.ETF_PROBE_COPY, "copy", 2 * nbytes), (etf.ETF_PROBE_ROWS, "rows_256B_scattered", nbytes)):
            tgt = b if kind == etf.ETF_PROBE_WRITE else a
            for _ in range(2):
                c.probe_bandwidth(kind, tgt, b if kind != etf.ETF_PROBE_WRITE else a, nbytes)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                c.probe_bandwidth(kind, tgt, b if kind != etf.ETF_PROBE_WRITE else a, nbytes)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            out["%s_%s_GBps" % (kname, label)] = moved / 1e9 / (ms / 1e3)
        del a, b
    # LDS read rate of the chip (no device memory involved): conflict-free 16-byte reads, and the table lookups'
    # pattern of 64-byte rows at scattered positions
    b = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    total = 64 << 30
    for kind, kname in ((etf.ETF_PROBE_LDS, "lds_read_b128"), (etf.ETF_PROBE_LDS_SCATTER, "lds_read_b128_scattered_rows")):
        c.probe_bandwidth(kind, b, b, total)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            c.probe_bandwidth(kind, b, b, total)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 3
        out["%s_GBps" % kname] = total / 1e9 / (ms / 1e3)
    # issue rate of the vector units for the instructions the scan kernels are made of, in lane instructions per second
    # (a wave instruction is 64 of them): one float32 add, the three-operand integer add, the packed 16-bit add
    nops = 2048 * 256 * 64 * 4096
    for kind, kname in ((etf.ETF_PROBE_VALU_F32, "valu_v_add_f32"), (etf.ETF_PROBE_VALU_ADD3, "valu_v_add3_u32"),
                        (etf.ETF_PROBE_VALU_PK16, "valu_v_pk_add_u16")):
        c.probe_bandwidth(kind, b, b, nops)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            c.probe_bandwidth(kind, b, b, nops)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 3
        out["%s_Tlane_instr_per_s" % kname] = nops / 1e12 / (ms / 1e3)
    # the float32 matrix instruction of the table, encoder and coarse-quantiser kernels, nothing but that instruction
    nflop = 2048 * 4 * 32 * 4096 * 2048
    c.probe_bandwidth(etf.ETF_PROBE_MFMA_F32, b, b, nflop)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        c.probe_bandwidth(etf.ETF_PROBE_MFMA_F32, b, b, nflop)
    e1.record()
    torch.cuda.synchronize()
    out["mfma_f32_32x32x2_TFLOPs"] = nflop / 1e12 / (e0.elapsed_time(e1) / 3 / 1e3)
    log("ceilings (GB/s; T lane instructions/s): " + ", ".join("%s %.4g" % kv for kv in out.items()))
    return out


def encode_leg(etf, torch, cfg_name):
    """The device encoder alone on one configuration's database (for counter runs)."""
    from workload import get_config
    cfg = get_config(cfg_name)
    _, _, _, info = make_inputs(cfg, etf, torch)
    return info


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--scale-n", type=int, default=0, help="override N (debugging only; invalidates the metric)")
    ap.add_argument("--scale-q", type=int, default=0, help="override Q (debugging only; invalidates the metric)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline and every parity check")
    ap.add_argument("--no-others", action="store_true", help="skip the legs beside the headline search")
    ap.add_argument("--no-configs", action="store_true", help="skip the legs of the other configurations (cfg3, cfg4, cfg5)")
    ap.add_argument("--configs", default="cfg3,cfg4,cfg5", help="the other configurations timed beside the headline")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--levels", action="store_true",
                    help="same as --traversal 1: the level-synchronous traversal (partial sums of internal nodes in HBM)")
    ap.add_argument("--traversal", type=int, default=2, choices=[0, 1, 2],
                    help="2 every table slice in LDS (default), 0 distance context in registers + result tables, 1 level-synchronous")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=VALUE", help="library option for every context (tuning)")
    ap.add_argument("--no-copy", action="store_true", help="skip the device copy and the memory ceilings")
    ap.add_argument("--encode-only", action="store_true", help="run the device encoder on the configuration's database and stop (counter runs)")
    args = ap.parse_args()
    EXTRA_OPTS[:] = list(args.opt)
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
    if args.encode_only:
        print(json.dumps({"encode_gpu": encode_leg(etf, torch, args.config)}), flush=True)
        return

    cfg = get_config(args.config)
    wl = Workload(cfg, etf, torch, args, args.scale_n or None, args.scale_q or None)
    cb, codes, queries, encode_info = wl.cb, wl.codes, wl.queries, wl.encode_info
    N, Q, k, T = wl.N, wl.Q, wl.k, wl.T
    stream, qd, out_ids, out_dist = wl.stream, wl.qd, wl.out_ids, wl.out_dist
    mode = etf.ETF_MODE_FOREST
    make_ctx = wl.make_ctx

    # ---- a plain device copy of known size (the reference dispatch against which the HBM byte counters are
    #      scaled) and the memory ceilings of this card from the library's probe kernels
    copy = ceilings = None
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
        ceilings = measure_ceilings(etf, torch, stream)
    CEILINGS.clear()
    CEILINGS.update(ceilings or {})

    main_res = wl.measure_search(T, args.traversal, args.steps, args.warmup)
    got_ids, got_dist = out_ids.cpu().numpy(), out_dist.cpu().numpy()
    ms_step, value, fallbacks = main_res["ms_per_step"], main_res["value"], main_res["fallbacks"]
    kernels, roofline, stats, S = main_res["kernels"], main_res["roofline"], main_res["stats"], main_res["S"]

    # ---- the same workload through the other paths, same run
    others = {}
    if not args.no_others:
        osteps = max(2, min(args.steps, 10))   # the other legs: up to ten steps after two warm-ups
        owarm = 2
        if args.traversal == 2:
            # the same E-Forest search through the table-based traversal (per-tree result tables in HBM)
            r0 = wl.measure_search(T, 0, osteps, owarm)
            others["e_forest_register_context"] = {k2: r0[k2] for k2 in ("value", "ms_per_step", "kernels", "roofline")}
        tree = make_ctx(1)
        for name, ctx, m in (("flat_gpu", tree, etf.ETF_MODE_FLAT), ("e_tree_gpu", tree, etf.ETF_MODE_TREE)):
            w2 = ctx.alloc_workspace(min(Q, cfg.query_batch or Q), k, m)
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
            wf = fc.alloc_workspace(min(Q, cfg.query_batch or Q), k, mode)
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
        wu = uc.alloc_workspace(min(Q, cfg.query_batch or Q), k, mode)
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
        w4 = ipc.alloc_workspace(min(Q, cfg.query_batch or Q), k, mode)
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
        w5 = oc.alloc_workspace(min(Q, cfg.query_batch or Q), k, mode)
        d5, p5 = time_search(oc, qd, k, mode, owarm, osteps, torch, w5, out_ids, out_dist, cfg.query_batch)
        others["chunk_order"] = {"order": [int(v) for v in order], "lookups_given_order": lk_given, "lookups_suggested_order": lk_order,
                                 "lookups_on": "at most 2^18 evenly spaced vectors", "suggest_s": t_suggest,
                                 "ms_per_step": d5 / osteps * 1e3, "n_distinct": oc.index_stats()["n_distinct"],
                                 "kernels_ms_per_step": {n: v[0] / osteps for n, v in p5.items() if v[1]}}
        log("chunk order %s: lookups %d -> %d (sample), search %.2f ms/step" % (others["chunk_order"]["order"], lk_given, lk_order, d5 / osteps * 1e3))
        del oc, w5
        # which chunks form a tree: the cut (and order) with the fewest lookups for T trees, and the search on that index
        # (the register-context traversal, where a tree's leaves are what is evaluated, shows what the cut is worth)
        pc = etf.Context(device=0, stream=stream)
        pc.set_option("traversal", args.traversal)
        pc.pq_set_codebooks(cb)
        t0 = time.time()
        pcb, porder, lk_equal, lk_best = pc.suggest_partition(codes, T=T)
        t_part = time.time() - t0
        pc.index_set_chunk_order(porder)
        pc.index_build(codes, T=T, chunk_begin=pcb)
        pc.index_upload()
        w6 = pc.alloc_workspace(min(Q, cfg.query_batch or Q), k, mode)
        d6, _ = time_search(pc, qd, k, mode, owarm, osteps, torch, w6, out_ids, out_dist, cfg.query_batch)
        others["tree_partition"] = {"chunk_begin": [int(v) for v in pcb], "order": [int(v) for v in porder],
                                    "lookups_equal_cut": lk_equal, "lookups_suggested_cut": lk_best,
                                    "lookups_on": "at most 2^16 evenly spaced vectors", "suggest_s": t_part,
                                    "ms_per_step": d6 / osteps * 1e3, "fallback_queries": pc.last_fallback_count()}
        log("tree partition %s, order %s: lookups %d -> %d (sample), search %.2f ms/step"
            % (others["tree_partition"]["chunk_begin"], others["tree_partition"]["order"], lk_equal, lk_best, d6 / osteps * 1e3))
        del pc, w6
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
            w3 = db.alloc_workspace(min(Q, cfg.query_batch or Q), k, mode)
            d3, _ = time_search(db, qd, k, mode, owarm, osteps, torch, w3, out_ids, out_dist, cfg.query_batch)
            others["index_build_device"] = {"ms": min(times[1:]), "vectors_per_s": N / (min(times[1:]) / 1e3),
                                            "image_bytes": db.index_device_bytes(), "image_bytes_bound": nimg, "workspace_bytes": nws,
                                            "search_ms_per_step": d3 / osteps * 1e3,
                                            "note": "sort, merge of repeats, level arrays of every tree, samples: wall clock of the call; "
                                                    "the search on the device-built index is the same kernels"}
            log("index build on the device: %.2f ms (%.3e vectors/s); search on it %.2f ms/step"
                % (min(times[1:]), N / (min(times[1:]) / 1e3), d3 / osteps * 1e3))
            del db, img, w3, codes_d
        if cfg.name == "cfg2" and wl.valid:
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
            # a step is two launches of a few microseconds: timed over 200 steps without event pairs around the
            # kernels (they cost about as much as the kernels), then 20 steps with them for the split
            for _ in range(3):
                t1.adc(q1d, etf.ETF_MODE_TREE, dist1, w1)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(200):
                t1.adc(q1d, etf.ETF_MODE_TREE, dist1, w1)
            torch.cuda.synchronize()
            ms1 = (time.perf_counter() - t0) / 200 * 1e3
            t1.profile_enable(not args.no_profile)
            for _ in range(20):
                t1.adc(q1d, etf.ETF_MODE_TREE, dist1, w1)
            torch.cuda.synchronize()
            p1 = t1.profile_read()
            nd1 = codes1.shape[0] * q1.shape[0]
            gb1 = nd1 * 4 / 1e9 / (ms1 / 1e3)
            others["all_pairs_cfg1"] = {"ms_per_step": ms1, "value": nd1 / (ms1 / 1e3), "output_GBps": gb1,
                                        "roofline": {"bound": "hbm", "achieved": gb1, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gb1 / HBM_PEAK_GBS},
                                        "kernels_ms_per_step": {n: v[0] / 20 for n, v in p1.items() if v[1]},
                                        "workload": "cfg1: N=%d Q=%d, single E-Tree, all pairs in input order" % (codes1.shape[0], q1.shape[0])}
            if not args.no_cpu:
                import oracle
                from parity import assert_distances_close
                assert_distances_close(dist1.cpu().numpy(), oracle.adc_all(q1, cb1, codes1), "bench cfg1 all pairs")
                others["all_pairs_cfg1"]["parity"] = "every distance against the oracle: ok"
            log("all pairs (cfg1): %.3f ms/step, %.3e distances/s, %.0f GB/s of output" % (ms1, others["all_pairs_cfg1"]["value"], gb1))
            del t1, dist1, w1

        if cfg.name == "cfg2" and wl.valid:
            others["ivfadc"] = ivf_leg(etf, torch, args, osteps, owarm)

    # ---- CPU oracle on a bounded sample of the same workload, and parity of the timed output on it
    cpu = None
    if not args.no_cpu:
        import oracle
        from parity import assert_topk_matches_identity
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
        picks = sorted(set(list(range(npar)) + [int(v) for v in np.linspace(npar, Q - 1, 8)])) if Q > npar else list(range(npar))
        for j in picks:      # the first tile, other tiles, the ragged last tile
            r = oracle.adc_all(queries[j:j + 1], cb, codes)[0]
            assert_topk_matches_identity(got_ids[j], got_dist[j], r, k, "bench q%d" % j)
        log("parity of the timed output against the oracle: ok on %d queries" % len(picks))
        # the codes the search ran on are the device encoder's: a stretch of them against the oracle's float32 rule
        from workload import GaussianMixture, SEED_DATABASE
        x0 = next(iter(GaussianMixture.from_config(cfg).chunks(N, SEED_DATABASE)))[:20000]
        assert np.array_equal(oracle.encode_f32(x0, cb), codes[:len(x0)]), "device-encoded codes differ from the oracle's"
        cpu["codes_checked"] = "first %d database vectors: device encoder == oracle.encode_f32" % len(x0)
        log("codes of the first %d database vectors equal the oracle's" % len(x0))

    # ---- the other configurations of the workload list, each end to end with its own roofline and parity check
    if not args.no_configs and cfg.name == "cfg2" and wl.valid:
        del wl, qd, out_ids, out_dist
        torch.cuda.empty_cache()
        for name in [c for c in args.configs.split(",") if c]:
            others[name] = config_leg(name, etf, torch, args, 5, 2)

    line = {
        "metric": "encoding-distances/sec (batched queries), E-Forest ADC + top-k, 1 GPU",
        "value": value, "unit": "encoding-distances/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "dtype_note": "returned distances and their order: float32 sums of float32 table entries; the candidate filter "
                      "(kernel lds16, if listed in `kernels`) adds 16-bit fixed-point entries",
        "config": {"workload": "%s: d=%d N=%d Q=%d PQ M=%d K=%d, E-Forest T=%d, top-%d, seeded %d-component Gaussian mixture"
                               % (cfg.name, cfg.d, N, Q, cfg.M, cfg.K, T, k, cfg.components),
                   "traversal": TRAVERSAL_NAMES[args.traversal], "path": PATH_NOTES[args.traversal],
                   "query_batch": cfg.query_batch or Q, "valid": not (args.scale_n or args.scale_q),
                   "kernel_sources": kernel_source_hash()},
        "roofline": roofline,
        # the table-based E-Forest traversal of the same run (per-tree result tables in HBM): the HBM-bandwidth figure
        "roofline_hbm_traversal": (others.get("e_forest_register_context") or {}).get("roofline"),
        "cpu_baseline": cpu,
        "kernels": kernels, "others": others, "encode_gpu": encode_info, "fallback_queries": fallbacks, "device_copy": copy,
        "memory_ceilings": ceilings,
        "index": {"n_distinct": stats["n_distinct"], "max_dup": stats["max_dup"], "device_MB": stats["device_bytes"] / 1e6,
                  "trees": stats["trees"], "sample": int(S)},
        "paper_context": PAPER_CONTEXT,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
