#!/usr/bin/env python3
"""Benchmark of the micrograph hot path on one MI355X.

A *step* is one pass of the whole hot path over one batch (or one group of batches that share a
pre-gather): hopgnn_sample -> hopgnn_pregather -> hopgnn_gather -> L x hopgnn_sage_fwd for fresh
seeds, inputs resident in HBM, no host synchronisation inside the timed region, issued as ONE
library call (hopgnn_batch_fwd) on ONE stream.  `value` is that single-stream rate; the rate with
consecutive steps alternating over a few streams is reported beside it.

The default run times the Products-shaped workload (2.4 M vertices x 100 fp32 features, 1024 seeds,
fanout [15,10,5], hidden 256) as the top-level line and carries the other workload shapes -
the 2^20-vertex R-MAT shape, the 16 M-vertex bf16 shape and the 100 M-vertex fp16 shape at groups
of 8, 16, 32 and 64 batches - in `per_config`.  Timed loops of `--steps` steps are repeated until
`--min-seconds` of wall time have passed and the median repeat is reported.

Kernel durations for the roofline come from HIP event pairs recorded by the library around one
kernel per step inside timed repeats of their own (so that the markers do not slow the repeats
`value` is taken from); the cost of a pair with nothing between is measured the same way and
subtracted.  The CPU oracle is timed on the host cores on a bounded sample of the same workload.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
# HBM bytes of the gather kernel per algorithmic byte, by row size in bytes, from rocprofv3 --pmc
# FETCH_SIZE and WRITE_SIZE runs scaled by a plain copy kernel (profiles/gather_traffic_pmc.txt,
# profiles/batch_traffic_pmc.txt).  Row sizes without a counter run report no traffic figure.
# HBM bytes by the profiler's counters (FETCH_SIZE x 2 + WRITE_SIZE, scaled by a plain copy of known
# size) over algorithmic bytes, per row size, measured on this command's own inputs
# (profiles/batch_traffic_pmc.txt: workloads 5, 3 and 4)
GATHER_TRAFFIC_OVER_ALGORITHMIC = {256: 1.008, 400: 1.127, 512: 1.012}
# the same for the first projection of the fused path: counter bytes per launch over "left operand once +
# output" (the self half of the operand is read from the gathered rows, which partly stay in cache)
PROJECT_L1_TRAFFIC_OVER_IO = {3: (116153.2 + 32768.0) * 1024 / (169984 * 200 * 4 + 2 * 16384 * 256 * 4),
                              4: (68137.1 + 4096.0) * 1024 / (106496 * 512 * 2 + 2 * 4096 * 256 * 2)}
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0}
DTYPE_NAME = {"torch.float32": "f32", "torch.bfloat16": "bf16", "torch.float16": "f16"}
HEADLINE_CONFIG = 3
PER_CONFIG = [(2, 1), (4, 1), (5, 8), (5, 16), (5, 32), (5, 64)]      # (workload shape, batches per pre-gather)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=0,
                    help="workload shape 1..5 (default: shape 3 as the headline with the other shapes in per_config)")
    ap.add_argument("--group", type=int, default=0, help="batches per pre-gather (0: the shape's default)")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams (each with its own buffers) of the multi-stream figure; with --backward, "
                         "--model, --dedup, --layerwise: of the timed loop itself")
    ap.add_argument("--min-seconds", type=float, default=0.3,
                    help="repeat the timed loop of --steps steps until this much wall time has passed")
    ap.add_argument("--per-config", action="store_true", help="with --config: also run the other shapes")
    ap.add_argument("--no-per-config", action="store_true", help="only the headline workload")
    ap.add_argument("--backward", action="store_true",
                    help="training steps: the layers' backward pass with in-place gradient accumulation and one "
                         "SGD update per step")
    ap.add_argument("--model", choices=["sage", "gcn", "gat"], default="sage",
                    help="layer type: GraphSAGE-mean (the headline workload), GCN-style mean, graph attention")
    ap.add_argument("--no-merge", action="store_true",
                    help="with a group > 1: run every batch's layers separately instead of one launch per layer "
                         "over the group's merged micrographs")
    ap.add_argument("--no-fuse", action="store_true",
                    help="two kernels per layer (segmented mean, projection) for every layer, instead of letting each "
                         "projection also form the next layer's neighbour means from the slot tree's shape")
    ap.add_argument("--dedup", action="store_true",
                    help="sample per-micrograph deduplicated frontiers (hopgnn_sample_dedup): the same rows for the "
                         "seeds over fewer rows below them (with --backward: GraphSAGE-mean training steps)")
    ap.add_argument("--layerwise", action="store_true",
                    help="layer-wise sampled micrographs (the shape's fanouts are the budgets of draws per level)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    return ap.parse_args()


def cpu_baseline(cfg, g, X, W, group, budget_s, all_cores_s=6.0, row_cap=None):
    """Time the CPU oracle as it stands on the same workload.

    Shapes the oracle finishes in seconds run whole batches (row_cap None).  For the larger shapes a
    group's sampling, pre-gather and gather run in full, and the layers run for the group's first
    batch only, each on its first `row_cap` destination rows over a source table compacted to the
    rows those read; a layer's seconds are scaled by rows / rows run (a layer is a loop over
    independent rows) and by the group's batch count (its batches have the same shape), and the
    figure says so."""
    import numpy as np

    import oracle
    from oracle.checks import ORC_DT, to_bits, weights_bits
    from paper_2409_00657_amd import synth

    off = g.offsets.cpu().numpy()
    idx = g.indices.cpu().numpy()
    big = X.shape[0] > 4_000_000
    Xh = None if big else to_bits(X)
    wb = weights_bits(W)
    odt = ORC_DT[X.dtype]
    L = len(cfg.fanouts)
    lv = oracle.level_sizes(cfg.batch, cfg.fanouts)

    def compact(table, self_idx, nbr):
        """The rows of `table` that the index lists read, and the lists renumbered to them (untimed)."""
        used = np.unique(np.concatenate([self_idx[self_idx >= 0], nbr[nbr >= 0]]))
        pos = np.full(table.shape[0], -1, np.int32)
        pos[used] = np.arange(len(used), dtype=np.int32)
        ren = lambda a: np.where(a >= 0, pos[np.maximum(a, 0)], -1).astype(np.int32)
        return np.ascontiguousarray(table[used]), ren(self_idx), ren(nbr)

    def layers_seconds(Xu, ids, indptr, remap):
        """Seconds of the L layers of one batch: whole, or scaled from the first row_cap rows."""
        if row_cap is None:
            t0 = time.perf_counter()
            oracle.forward(Xu, odt, ids, indptr, remap, cfg.batch, cfg.fanouts, wb)
            return time.perf_counter() - t0
        B, total = cfg.batch, 0.0
        for k in range(1, L + 1):
            n_dst = sum(lv[:L - k + 1])
            rows = min(n_dst, row_cap)
            ip = np.asarray(indptr[:rows + 1], np.int32)
            nnz = int(ip[rows])
            Ws, Wn, b = wb[k - 1]
            if k == 1:
                H, self_idx, nbr = compact(Xu, remap[:rows], remap[B:B + nnz])
            else:       # the rows a capped earlier layer did not produce do not exist: only the time is
                # wanted, so this layer's sources are stand-in rows of the right shape and type
                e = np.arange(nnz, dtype=np.int32)
                self_idx = np.arange(rows, dtype=np.int32)
                nbr = np.where(ids[B:B + nnz] >= 0, rows + e, -1).astype(np.int32)
                H = np.resize(Xu.reshape(-1), (rows + nnz) * Ws.shape[0]).reshape(rows + nnz, Ws.shape[0])
            t0 = time.perf_counter()
            o64 = oracle.sage_fwd(H, odt, self_idx, ip, nbr, Ws, Wn, b, relu=(k < L))
            oracle.round_store(o64, odt)
            total += (time.perf_counter() - t0) * (n_dst / rows)
        return total

    def one_group(it):
        """One group of batches; returns the (scaled) seconds of its timed part."""
        seeds = [synth.seeds(cfg.n_vertices, cfg.batch, 10_000 + it * group + b).numpy() for b in range(group)]
        rows = None
        if big:   # the oracle cannot hold the table: hand it the rows it will ask for (untimed)
            ids0 = np.concatenate([oracle.sample(off, idx, s, cfg.fanouts, key=it * group + b)[0]
                                   for b, s in enumerate(seeds)])
            u0, _ = oracle.pregather(ids0)
            import torch
            rows = to_bits(X[torch.from_numpy(u0).long().to(X.device)])
        t0 = time.perf_counter()
        ids, indptr = [], None
        for b, s in enumerate(seeds):
            i, indptr = oracle.sample(off, idx, s, cfg.fanouts, key=it * group + b)
            ids.append(i)
        allids = np.concatenate(ids)
        uniq, remap = oracle.pregather(allids)
        Xu = oracle.gather(rows, np.arange(len(uniq), dtype=np.int32)) if big else oracle.gather(Xh, uniq)
        t = time.perf_counter() - t0
        T = len(ids[0])
        if row_cap is None:
            for b in range(group):
                t += layers_seconds(Xu, ids[b], indptr, remap[b * T:(b + 1) * T])
        else:
            t += group * layers_seconds(Xu, ids[0], indptr, remap[:T])
        return t

    what = ("whole batches" if row_cap is None else
            "batches (sampling, pre-gather, gather in full; layers of the group's first batch on their first "
            "%d rows, scaled by rows/rows run and by the group's batch count)" % row_cap)
    done, t_total, it = 0, 0.0, 0
    wall0 = time.perf_counter()
    while True:
        t_total += one_group(it)
        done += group
        it += 1
        if time.perf_counter() - wall0 >= budget_s or it >= 64:
            break
    out = {"value": done / t_total, "unit": "batches/s", "cores": 1, "kind": "oracle",
           "sample": "%d %s of %s (sample+pregather+gather+%d layers, fp64 C oracle, 1 thread)"
                     % (done, what, cfg.name, L),
           "seconds": round(time.perf_counter() - wall0, 2)}
    # the same oracle on every core of this process's share: micrographs (here: whole groups) are
    # independent, so each thread runs its own groups (the C library holds no state and the calls
    # release the interpreter lock); the oracle itself is unchanged
    n_threads = min(16, len(os.sched_getaffinity(0)))
    if n_threads > 1 and all_cores_s > 0:
        from concurrent.futures import ThreadPoolExecutor
        t_start = time.perf_counter()

        def worker(w):
            n, t = 0, 0.0
            while n == 0 or time.perf_counter() - t_start < all_cores_s:
                t += one_group(1000 + w * 4096 + n)
                n += 1
            return n, t
        with ThreadPoolExecutor(max_workers=n_threads) as pool:
            res = list(pool.map(worker, range(n_threads)))
        elapsed = time.perf_counter() - t_start
        n_groups = sum(n for n, _ in res)
        # whole batches: groups finished / wall time.  Scaled samples: every thread's rate from its own
        # scaled seconds, summed (the threads run side by side)
        rate = (n_groups * group / elapsed) if row_cap is None else sum(n * group / t for n, t in res if t > 0)
        out["all_cores"] = {"value": rate, "unit": "batches/s", "cores": n_threads,
                            "sample": "%d %s on %d threads, one group per thread at a time"
                                      % (n_groups * group, what, n_threads),
                            "seconds": round(elapsed, 2)}
    return out


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2] if xs else float("nan")


def run_workload(cfg_id, group, args, cache, cpu_budget, stats_steps=6):
    """Time one workload shape: single stream (the definition of a batch), several streams, kernel
    durations from event pairs in timed repeats of their own, ratios of the pre-gather, and the
    CPU oracle.  Returns the workload's record."""
    import torch

    from paper_2409_00657_amd import binding as hb
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import BatchShape, HotPath

    dev = "cuda:0"
    cfg = synth.CONFIGS[cfg_id]
    if cache.get("cfg_id") != cfg_id:         # graph, features and weights are shared by a shape's group sizes
        cache.clear()
        torch.cuda.empty_cache()
        cache.update(cfg_id=cfg_id, g=cfg.make_graph(device=dev), X=cfg.make_features(device=dev),
                     W=cfg.make_weights(device=dev))
    g, X, W = cache["g"], cache["X"], cache["W"]
    merge = group > 1 and not args.no_merge
    n_multi = max(1, args.streams)
    hps = [HotPath(g.offsets, g.indices, X, W, cfg.batch, cfg.fanouts, group=group, merge=merge,
                   fuse_tree=not args.no_fuse) for _ in range(n_multi)]
    streams = [torch.cuda.Stream() for _ in range(n_multi)]      # default priority
    raw_streams = [s.cuda_stream for s in streams]
    hp, sh = hps[0], hps[0].shape               # sh: the layout the layers run on (merged: the whole group)
    shb = BatchShape(cfg.batch, list(cfg.fanouts))
    L, K, Wm = sh.n_layers, args.steps, args.warmup
    hidden = hp.H[-1].shape[1]
    outs = [torch.empty((group * cfg.batch, hidden), dtype=X.dtype, device=dev) for _ in range(n_multi)]
    es, dname = X.element_size(), DTYPE_NAME[str(X.dtype)]

    # fresh seeds and keys for every step of every repeat (a pool that the repeats walk through)
    pool = 64 * max(K, 1) + Wm
    seeds_all = synth.seeds(cfg.n_vertices, cfg.batch * group * pool, 0, device=dev).view(pool, group * cfg.batch)
    seed_views = [seeds_all[i] for i in range(pool)]
    keys_all = [[i * group + b for b in range(group)] for i in range(pool)]
    torch.cuda.synchronize()

    def step(i, j=0, marks=None):
        hps[j].forward(seed_views[i % pool], keys_all[i % pool], outs[j], raw_streams[j], marks)

    for i in range(Wm):
        step(i)
    torch.cuda.synchronize()

    # stages whose kernels are bracketed by an event pair, one per step in the marked repeats
    stages = [("gather", hb.MARK_GATHER), ("empty_pair", hb.MARK_EMPTY), ("sample", hb.MARK_SAMPLE),
              ("pregather", hb.MARK_PREGATHER)]
    for k in range(1, L + 1):
        stages.append(("project_l%d" % k, hb.MARK_PROJECT + k))
        if k == 1 or not hp.fused:      # fused slot-tree layers: the previous projection made this layer's means
            stages.append(("aggregate_l%d" % k, hb.MARK_AGGREGATE + k))
    ev = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(2)) for _ in range(K)]
    for a, b in ev:                       # record once so that the handles exist
        a.record(streams[0])
        b.record(streams[0])
    torch.cuda.synchronize()
    raw_ev = [(a.cuda_event, b.cuda_event) for a, b in ev]
    stage_ms = {name: [] for name, _ in stages}

    # timed repeats of exactly K steps each, alternating: plain (-> value), marked (-> kernel durations)
    plain, marked, cursor, n_rep = [], [], Wm, 0
    t_begin = time.perf_counter()
    while True:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            step(cursor + i)
        torch.cuda.synchronize()
        plain.append(time.perf_counter() - t0)
        cursor += K
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            step(cursor + i, 0, raw_ev[i] + (stages[(n_rep * K + i) % len(stages)][1],))
        torch.cuda.synchronize()
        marked.append(time.perf_counter() - t0)
        for i in range(K):
            stage_ms[stages[(n_rep * K + i) % len(stages)][0]].append(ev[i][0].elapsed_time(ev[i][1]))
        cursor += K
        n_rep += 1
        enough = all(len(v) >= 3 for v in stage_ms.values())
        if (sum(plain) >= args.min_seconds and n_rep >= 3 and enough) or n_rep >= 400:
            break
    t_single = _median(plain)

    # the same steps alternating over several streams, each with its own buffers
    multi = []
    if n_multi > 1:
        for i in range(Wm):
            step(cursor + i, i % n_multi)
        cursor += Wm
        while sum(multi) < args.min_seconds / 2 or len(multi) < 3:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(K):
                step(cursor + i, i % n_multi)
            torch.cuda.synchronize()
            multi.append(time.perf_counter() - t0)
            cursor += K
            if len(multi) >= 400:
                break
    wall_timed = time.perf_counter() - t_begin

    # untimed replay of a few steps: U, valid slots per level, what per-batch pre-gathering would fetch
    U_sum = valid_sum = U_per_batch_sum = 0
    valid_level = [0] * (L + 1)
    level_off = [sum(sh.levels[:h]) for h in range(L + 2)]
    n_stats = min(stats_steps, K) if group <= 16 else 2
    for i in range(n_stats):
        step(Wm + i)
        torch.cuda.synchronize()
        U_sum += int(hp.n_uniq.item())
        ok = (hp.ids >= 0).view(hp.layer_batches, -1)      # one row per separately laid out batch
        for h in range(L + 1):
            valid_level[h] += int(ok[:, level_off[h]:level_off[h + 1]].sum().item())
        if group > 1:
            for b in range(group):
                if merge:   # batch b's slots of every level of the merged level-major array
                    ib = torch.cat([hp.ids[level_off[h] + b * shb.levels[h]:level_off[h] + (b + 1) * shb.levels[h]]
                                    for h in range(L + 1)])
                else:
                    ib = hp.ids[b * shb.n_slots:(b + 1) * shb.n_slots]
                U_per_batch_sum += int(torch.unique(ib[ib >= 0]).numel())
    valid_sum = sum(valid_level)
    U_avg = U_sum / n_stats
    valid_level = [v / n_stats for v in valid_level]

    # algorithmic work of every bracketed kernel, per launch (a merged group's layer is one launch)
    row_bytes = X.shape[1] * es
    empty = sum(stage_ms["empty_pair"]) / len(stage_ms["empty_pair"])
    kernels = {}

    def add(name, bound, work, peak, unit, extra=None):
        raw = sum(stage_ms[name]) / len(stage_ms[name])
        net = max(raw - empty, 1e-6)
        scale = 1e-9 if unit == "GB/s" else 1e-12
        ach = work / (net * 1e-3) * scale
        rec = {"bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
               "work_per_launch": work, "avg_launch_ms": net, "avg_event_pair_ms": raw,
               "median_event_pair_ms": _median(stage_ms[name]), "samples": len(stage_ms[name])}
        if extra:
            rec.update(extra)
        kernels[name] = rec

    gather_bytes = U_avg * (2 * row_bytes + 4)
    add("gather", "hbm", gather_bytes, HBM_PEAK_GBPS, "GB/s",
        {"kernel": "gather_rows",
         "traffic": (gather_bytes * GATHER_TRAFFIC_OVER_ALGORITHMIC[row_bytes]
                     if row_bytes in GATHER_TRAFFIC_OVER_ALGORITHMIC else None)})
    slots = group * shb.n_slots
    add("pregather", "hbm", 8.0 * slots + 4 * U_avg, HBM_PEAK_GBPS, "GB/s", {"kernel": "bitmap pre-gather (3 launches)"})
    w_off = 8 if g.offsets.dtype == torch.int64 else 4
    parents = sum(valid_level[:L])
    add("sample", "hbm", parents * (2 * w_off + 4) + 8.0 * (slots - group * cfg.batch), HBM_PEAK_GBPS, "GB/s",
        {"kernel": "sample_micrographs"})
    din = X.shape[1]
    runs = 1 if merge else group          # a stage marker brackets the first run's kernel only
    for k in range(1, L + 1):
        n_dst, nnz = sh.n_dst(k), sh.nnz(k)
        nnz_valid = sum(valid_level[1:L - k + 2]) / runs
        flops = 2.0 * n_dst * 2 * din * hidden
        # left operand once + output (fused slot-tree layers store the next layer's destination rows and
        # as many rows of neighbour means instead of every row)
        out_rows = 2 * sh.n_dst(k + 1) if (hp.fused and k < L) else n_dst
        io = n_dst * 2 * din * es + out_rows * hidden * es
        add("project_l%d" % k, "mfma", flops, MFMA_PEAK_TFLOPS[dname] * 1.0, "TFLOP/s",
            {"kernel": "sage_project", "M": n_dst, "K": 2 * din, "N": hidden,
             "hbm_bytes_operand_once_plus_output": io})
        kernels["project_l%d" % k]["hbm_GBps"] = io / (kernels["project_l%d" % k]["avg_launch_ms"] * 1e-3) * 1e-9
        kernels["project_l%d" % k]["hbm_frac"] = kernels["project_l%d" % k]["hbm_GBps"] / HBM_PEAK_GBPS
        if k == 1 and hp.fused and group == 1 and cfg_id in PROJECT_L1_TRAFFIC_OVER_IO:
            kernels["project_l1"]["traffic"] = io * PROJECT_L1_TRAFFIC_OVER_IO[cfg_id]
        if "aggregate_l%d" % k not in stage_ms:
            din = hidden
            continue
        agg_bytes = nnz_valid * din * es + n_dst * din * es + 4.0 * (nnz + n_dst)
        src_bytes = (U_avg if k == 1 else sh.n_dst(k - 1)) * din * es
        cached = src_bytes < 256e6 and agg_bytes > 1.5 * src_bytes
        add("aggregate_l%d" % k, "cache (peak shown is HBM's, for scale)" if cached else "hbm", agg_bytes, HBM_PEAK_GBPS, "GB/s",
            {"kernel": "sage_mean", "rows": n_dst, "valid_entries": nnz_valid, "source_table_bytes": src_bytes,
             "note": ("rows are re-read several times each from a table that fits the 256 MB Infinity Cache: "
                      "the rate is cache bandwidth, not HBM" if cached else "")})
        din = hidden
    # the kernel that takes the largest share of a step
    share = {n: r["avg_launch_ms"] * (runs if n.startswith(("project", "aggregate")) else 1)
             for n, r in kernels.items()}
    dominant = max(share, key=share.get)
    step_ms = t_single / K * 1e3
    rec = {
        "workload": cfg.name, "dtype": dname, "group": group, "merged_layers": merge, "fused_tree_layers": hp.fused,
        "n_vertices": cfg.n_vertices, "n_edges": g.n_edges, "feature_dim": cfg.d, "batch": cfg.batch,
        "fanouts": cfg.fanouts, "hidden": cfg.hidden, "slots_per_batch": shb.n_slots,
        "batches_per_s": K * group / t_single, "ms_per_step": step_ms, "repeats": len(plain),
        "ms_per_step_min_max": [min(plain) / K * 1e3, max(plain) / K * 1e3],
        "ms_per_step_p10_p90": [sorted(plain)[len(plain) // 10] / K * 1e3, sorted(plain)[(len(plain) * 9) // 10] / K * 1e3],
        "timed_steps": K * len(plain),
        "ms_per_step_with_markers": _median(marked) / K * 1e3,
        "multi_stream": ({"streams": n_multi, "batches_per_s": K * group / _median(multi),
                          "ms_per_step": _median(multi) / K * 1e3, "repeats": len(multi)} if multi else None),
        "timed_wall_s": round(wall_timed, 3),
        "unique_rows_per_step": U_avg,
        "unique_over_valid_slots": U_sum / max(valid_sum, 1),
        "unique_group_over_sum_of_per_batch_unique": (U_sum / U_per_batch_sum) if group > 1 else 1.0,
        "valid_slot_fraction": valid_sum / (n_stats * slots),
        "kernels": kernels, "dominant_kernel": dominant,
        "kernel_share_of_step": {n: round(v / step_ms, 4) for n, v in share.items() if n != "empty_pair"},
        "empty_event_pair_ms": empty,
    }
    if cpu_budget > 0:
        # whole batches where the oracle finishes one in about a second; a stated, scaled sample beyond
        rec["cpu_baseline"] = cpu_baseline(cfg, g, X, W, group, cpu_budget * 0.6, all_cores_s=cpu_budget * 0.4,
                                           row_cap={1: None, 2: None, 3: 8192}.get(cfg_id, 1024))
    del hps, outs, seeds_all
    torch.cuda.empty_cache()
    return rec


def roofline_block(rec, name):
    k = rec["kernels"][name]
    out = {"kernel": k.get("kernel", name), "stage": name, "bound": k["bound"], "achieved": k["achieved"],
           "peak": k["peak"], "unit": k["unit"], "frac": k["frac"], "traffic": k.get("traffic"),
           "work_per_launch": k["work_per_launch"], "avg_launch_ms": k["avg_launch_ms"],
           "avg_event_pair_ms": k["avg_event_pair_ms"], "empty_event_pair_ms": rec["empty_event_pair_ms"],
           "samples": k["samples"]}
    for extra in ("M", "K", "N", "hbm_bytes_operand_once_plus_output", "hbm_GBps", "hbm_frac", "source_table_bytes",
                  "note"):
        if extra in k:
            out[extra] = k[extra]
    return out


def main_headline(args):
    """The GraphSAGE-mean forward path over slot trees: the headline workload and, unless told
    otherwise, the other shapes."""
    import torch

    from paper_2409_00657_amd import binding as hb
    from paper_2409_00657_amd import synth

    hb.load_library()                      # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    head_cfg = args.config or HEADLINE_CONFIG
    head_group = args.group or synth.CONFIGS[head_cfg].groups[0]
    cache = {}
    cpu = 0.0 if args.no_cpu_baseline else args.cpu_seconds
    t0 = time.perf_counter()
    head = run_workload(head_cfg, head_group, args, cache, cpu)
    others = []
    if not args.no_per_config and (args.config == 0 or args.per_config):
        for cid, grp in PER_CONFIG:
            if (cid, grp) == (head_cfg, head_group):
                continue
            # the oracle leg of the other shapes is short; the largest groups have none (one group's
            # sampling and sort alone take longer than the budget)
            others.append(run_workload(cid, grp, args, cache, 0.0 if (args.no_cpu_baseline or grp > 8) else 6.0,
                                       stats_steps=3))
    cache.clear()
    dom = head["dominant_kernel"]
    out = {
        "metric": "micrograph batches/s", "value": head["batches_per_s"], "unit": "batches/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"],
        "data": "synthetic",
        "config": {"workload": head["workload"], "n_vertices": head["n_vertices"], "n_edges": head["n_edges"],
                   "feature_dim": head["feature_dim"], "batch": head["batch"], "fanouts": head["fanouts"],
                   "hidden": head["hidden"], "group": head["group"], "merged_layers": head["merged_layers"],
                   "fused_tree_layers": head["fused_tree_layers"], "slots_per_batch": head["slots_per_batch"], "streams": 1, "backward": False, "layer": "sage",
                   "repeats_of_steps": head["repeats"], "min_seconds": args.min_seconds},
        "gather_GBps": head["kernels"]["gather"]["achieved"],
        "gather_frac_of_hbm_peak": head["kernels"]["gather"]["frac"],
        "multi_stream": head["multi_stream"],
        "unique_rows_per_step": head["unique_rows_per_step"],
        "unique_over_valid_slots": head["unique_over_valid_slots"],
        "valid_slot_fraction": head["valid_slot_fraction"],
        "roofline": roofline_block(head, dom),
        "roofline_gather": roofline_block(head, "gather"),
        "kernels": head["kernels"], "kernel_share_of_step": head["kernel_share_of_step"],
        "ms_per_step_min_max": head["ms_per_step_min_max"],
        "ms_per_step_with_markers": head["ms_per_step_with_markers"],
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    if others:
        keep = ("workload", "dtype", "group", "merged_layers", "fused_tree_layers", "batch", "fanouts", "hidden", "batches_per_s",
                "ms_per_step", "repeats", "multi_stream", "unique_rows_per_step", "unique_over_valid_slots",
                "unique_group_over_sum_of_per_batch_unique", "valid_slot_fraction", "dominant_kernel",
                "kernel_share_of_step", "cpu_baseline")
        out["per_config"] = []
        for r in others:
            e = {k: r[k] for k in keep if k in r}
            e["roofline"] = roofline_block(r, r["dominant_kernel"])
            e["roofline_gather"] = roofline_block(r, "gather")
            e["kernel_frac"] = {n: round(k["frac"], 4) for n, k in r["kernels"].items() if n != "empty_pair"}
            e["kernel_avg_launch_ms"] = {n: round(k["avg_launch_ms"], 5) for n, k in r["kernels"].items()}
            out["per_config"].append(e)
    out["bench_wall_s"] = round(time.perf_counter() - t0, 1)
    print(json.dumps(out))


def main_dedup(args):
    """The forward step over deduplicated frontiers: same JSON line, call-by-call sequence."""
    import torch

    from paper_2409_00657_amd import binding as hb
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import DedupPath

    hb.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config or HEADLINE_CONFIG]
    g = cfg.make_graph(device=dev)
    X = cfg.make_features(device=dev)
    W = cfg.make_weights(device=dev)
    n_streams = max(1, args.streams)
    group = args.group or cfg.groups[0]
    sampler = "layer" if args.layerwise else "node"
    # training steps update the weights: every stream is then a worker with its own replica
    Ws = [W] + [[tuple(None if t is None else t.clone() for t in layer) for layer in W]
                for _ in range(n_streams - 1)] if args.backward else [W] * n_streams
    dps = [DedupPath(g.offsets, g.indices, X, Ws[j], cfg.batch, cfg.fanouts, group=group, sampler=sampler,
                     model=args.model) for j in range(n_streams)]
    if args.backward:
        for d in dps:
            d.enable_backward()
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    n_total = args.warmup + args.steps
    seeds = [torch.cat([synth.seeds(cfg.n_vertices, cfg.batch, i * group + b, device=dev) for b in range(group)])
             for i in range(n_total)]
    keys = [[i * group + b for b in range(group)] for i in range(n_total)]
    torch.cuda.synchronize()

    outs = [torch.empty((group * cfg.batch, cfg.hidden), dtype=X.dtype, device=dev) for _ in range(n_streams)]
    raw_streams = [s.cuda_stream for s in streams]

    def step_fwd(i, marks=None):
        j = i % n_streams
        dps[j].forward(seeds[i], keys[i], outs[j], raw_streams[j], marks)

    def step_train(i, marks=None):
        """Forward call by call, backward with in-place accumulation, update: one iteration."""
        j = i % n_streams
        with torch.cuda.stream(streams[j]):         # the gather's event pair records on the current stream
            dps[j].train_step(seeds[i], keys[i], 1e-4, raw_streams[j], marks)

    step = step_train if args.backward else step_fwd

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(2)) for _ in range(args.steps)]
    for i, e in enumerate(ev):      # record once so that the handles exist
        e[0].record(streams[i % n_streams])
        e[1].record(streams[i % n_streams])
    torch.cuda.synchronize()
    raw_marks = ev if args.backward else [(a.cuda_event, b.cuda_event) for a, b in ev]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, raw_marks[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    gather_ms = sorted(a.elapsed_time(b) for a, b in ev)
    # instrumented replay on one stream: stage times, U, node counts
    dp, L = dps[0], len(cfg.fanouts)
    E = lambda: torch.cuda.Event(enable_timing=True)
    stage = {"sample": 0.0, "pregather": 0.0, "gather": 0.0, "compose": 0.0}
    for k in range(1, L + 1):
        stage["sage_l%d" % k] = 0.0
    n_replay, U_sum, nodes_sum, valid_sum = min(args.steps, 50), 0, 0, 0
    for i in range(n_replay):
        j = args.warmup + i
        fns = [("sample", lambda: dp.sample(seeds[j], keys[j])), ("pregather", dp.pregather), ("gather", dp.gather),
               ("compose", dp.compose)] + [("sage_l%d" % k, (lambda k=k: dp.layer(k))) for k in range(1, L + 1)]
        for name, fn in fns:
            a, b = E(), E()
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            stage[name] += a.elapsed_time(b)
        U_sum += int(dp.n_uniq.item())
        nodes_sum += int(dp.level_start[L + 1].item())
    stage = {k: v / n_replay for k, v in stage.items()}
    U_avg = U_sum / n_replay
    row_bytes = X.shape[1] * X.element_size()
    gather_bytes = U_avg * (2 * row_bytes + 4)
    g_avg = sum(gather_ms) / len(gather_ms)
    gbps = gather_bytes / (g_avg * 1e-3) / 1e9
    out = {
        "metric": "micrograph batches/s", "value": args.steps * group / elapsed, "unit": "batches/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": DTYPE_NAME[str(X.dtype)],
        "data": "synthetic",
        "config": {"workload": cfg.name, "n_vertices": cfg.n_vertices, "n_edges": g.n_edges, "feature_dim": cfg.d,
                   "batch": cfg.batch, "fanouts": cfg.fanouts, "hidden": cfg.hidden, "group": group, "streams": n_streams,
                   "deduplicated_frontiers": True, "sampler": sampler + "-wise", "backward": bool(args.backward), "layer": args.model, "slots_per_batch": dp.capacity // group},
        "unique_rows_per_step": U_avg, "nodes_per_step": nodes_sum / n_replay,
        "nodes_over_slots": nodes_sum / n_replay / dp.capacity,
        "stage_ms": {k: round(v, 5) for k, v in stage.items()},
        "roofline": {"kernel": "gather_rows", "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS,
                     "traffic": (gather_bytes * GATHER_TRAFFIC_OVER_ALGORITHMIC[row_bytes]
                                 if row_bytes in GATHER_TRAFFIC_OVER_ALGORITHMIC else None),
                     "algorithmic_bytes_per_launch": gather_bytes, "avg_launch_ms": g_avg,
                     "launch_ms_percentiles": {"p10": gather_ms[len(gather_ms) // 10], "p50": gather_ms[len(gather_ms) // 2],
                                               "p90": gather_ms[(len(gather_ms) * 9) // 10]}},
    }
    print(json.dumps(out))




def main_variant(args):
    """Training steps (--backward) and the other layer types (--model gcn|gat) on one workload: one JSON
    line with the gather kernel's roofline (event pairs inside the timed region)."""
    import torch

    from paper_2409_00657_amd import binding as hb
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath

    hb.load_library()                      # fail loudly if the HIP library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config or HEADLINE_CONFIG]
    group = args.group or cfg.groups[0]
    g = cfg.make_graph(device=dev)
    X = cfg.make_features(device=dev)
    W = cfg.make_weights(device=dev)
    n_streams = max(1, args.streams)
    merge = group > 1 and not args.no_merge and not args.backward
    # training steps update the weights: every stream is then a worker with its own replica
    Ws = [W] + [[tuple(None if t is None else t.clone() for t in layer) for layer in W]
                for _ in range(n_streams - 1)] if args.backward else [W] * n_streams
    hps = [HotPath(g.offsets, g.indices, X, Ws[j], cfg.batch, cfg.fanouts, group=group, model=args.model, merge=merge)
           for j in range(n_streams)]
    streams = [torch.cuda.Stream() for _ in range(n_streams)]      # default priority
    if args.backward:
        for h in hps:
            h.enable_backward()
    hp = hps[0]
    sh = hp.shape                                   # the layout the layers run on (merged: the whole group)
    from paper_2409_00657_amd.pipeline import BatchShape
    shb = BatchShape(cfg.batch, list(cfg.fanouts))  # one batch
    n_total = args.warmup + args.steps
    seeds = [[synth.seeds(cfg.n_vertices, cfg.batch, i * group + b, device=dev) for b in range(group)]
             for i in range(n_total)]
    keys = [[i * group + b for b in range(group)] for i in range(n_total)]
    torch.cuda.synchronize()

    seeds_cat = [torch.cat(s) for s in seeds]
    hidden = hp.H[-1].shape[1]
    outs = [torch.empty((group * cfg.batch, hidden), dtype=X.dtype, device=dev) for _ in range(n_streams)]
    raw_streams = [s.cuda_stream for s in streams]

    def step_fwd(i, marks=None):
        """One whole forward step on stream i % n_streams: one call of hopgnn_batch_fwd."""
        j = i % n_streams
        hps[j].forward(seeds_cat[i], keys[i], outs[j], raw_streams[j], marks)

    def step_calls(i, ev=None):
        """The same step call by call (with the backward pass, if asked for)."""
        h, stream = hps[i % n_streams], streams[i % n_streams]
        st = stream.cuda_stream
        h.sample_group(seeds_cat[i], keys[i], st)
        h.pregather(st)
        if ev is not None:
            ev[0].record(stream)
        h.gather(st)
        if ev is not None:
            ev[1].record(stream)
        for b in range(h.layer_batches):
            h.layers(b, st)
            if args.backward:
                h.backward(b, st)
        if args.backward:       # end of the iteration: update from the accumulated gradients, clear them
            h.apply_sgd(1e-4, st)

    by_calls = args.backward
    step = step_calls if by_calls else step_fwd
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # one event pair per timed step around the gather launch; recorded once here so that the
    # handles exist, then re-recorded by the step itself
    gather_ev = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(2)) for _ in range(args.steps)]
    for i, e in enumerate(gather_ev):
        e[0].record(streams[i % n_streams])
        e[1].record(streams[i % n_streams])
    torch.cuda.synchronize()
    marks = gather_ev if by_calls else [(e[0].cuda_event, e[1].cuda_event) for e in gather_ev]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, marks[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    gather_ms = [e[0].elapsed_time(e[1]) for e in gather_ev]

    # untimed, instrumented replay of the same steps on one stream: U per step and a per-stage breakdown
    stage = {"sample": 0.0, "pregather": 0.0, "gather": 0.0}
    empty_ms = []
    for k in range(1, sh.n_layers + 1):
        stage["sage_l%d" % k] = 0.0
    U_sum, valid_sum, U_per_batch_sum = 0, 0, 0
    E = lambda: torch.cuda.Event(enable_timing=True)
    n_replay = min(args.steps, 50)
    st0 = torch.cuda.current_stream().cuda_stream
    for i in range(n_replay):
        j = args.warmup + i
        e = [E() for _ in range(6)]
        e[0].record()
        hp.sample_group(seeds_cat[j], keys[j], st0)
        e[1].record()
        hp.pregather(st0)
        e[2].record()
        hp.gather(st0)
        e[3].record()
        e[4].record()        # an empty pair: what two event markers cost with nothing between
        e[5].record()
        torch.cuda.synchronize()
        empty_ms.append(e[4].elapsed_time(e[5]))
        stage["sample"] += e[0].elapsed_time(e[1])
        stage["pregather"] += e[1].elapsed_time(e[2])
        stage["gather"] += e[2].elapsed_time(e[3])
        U_sum += int(hp.n_uniq.item())
        valid_sum += int((hp.ids >= 0).sum().item())
        if group > 1:       # reporting only: what per-batch pre-gathering would have fetched
            for b in range(group):
                if merge:   # batch b's slots of every level of the merged level-major array
                    ib = torch.cat([hp.ids[sum(sh.levels[:h]) + b * shb.levels[h]:
                                           sum(sh.levels[:h]) + (b + 1) * shb.levels[h]] for h in range(len(sh.levels))])
                else:
                    ib = hp.ids[b * shb.n_slots:(b + 1) * shb.n_slots]
                U_per_batch_sum += int(torch.unique(ib[ib >= 0]).numel())
        for b in range(hp.layer_batches):      # one event pair per layer, summed over the group's batches
            for k in range(1, sh.n_layers + 1):
                a, c = E(), E()
                a.record()
                hp.layer(b, k, st0)
                c.record()
                torch.cuda.synchronize()
                stage["sage_l%d" % k] += a.elapsed_time(c)
    stage = {k: v / n_replay for k, v in stage.items()}
    U_avg = U_sum / n_replay
    row_bytes = X.shape[1] * X.element_size()
    # algorithmic bytes of one gather launch: every unique row read once and written once,
    # plus its 4-byte index
    gather_bytes = U_avg * (2 * row_bytes + 4)
    # The duration used for the roofline is the event pair around the launch, which also holds
    # the two markers' own cost (a pair with nothing between reads ~5 us): an upper bound of the
    # kernel's duration, so the fraction is a lower bound.  rocprofv3's per-kernel average
    # (profiles/) is the direct figure; the pair minus the empty pair is given beside it.
    gather_ms_raw = sum(gather_ms) / len(gather_ms)
    gs = sorted(gather_ms)
    gather_pct = {"p10": gs[len(gs) // 10], "p50": gs[len(gs) // 2], "p90": gs[(len(gs) * 9) // 10]}
    empty_ms_avg = sum(empty_ms) / len(empty_ms)
    gather_ms_avg = gather_ms_raw
    gather_ms_net = max(gather_ms_raw - empty_ms_avg, 1e-6)
    gather_gbps = gather_bytes / (gather_ms_avg * 1e-3) / 1e9
    # per-stage algorithmic work (whole entry points, from the instrumented replay)
    es = X.element_size()
    valid_avg = valid_sum / n_replay
    stage_work = {"gather": {"bound": "hbm", "bytes": gather_bytes}}
    stage_work["pregather"] = {"bound": "hbm", "bytes": group * shb.n_slots * 8 + 4 * U_avg}
    din = X.shape[1]
    for k in range(1, sh.n_layers + 1):
        n_dst, nnz = shb.n_dst(k), shb.nnz(k)
        if args.model == "sage":
            flops = 2.0 * n_dst * 2 * din * cfg.hidden
            nbytes = (nnz + n_dst) * din * es + 4 * (nnz + 2 * n_dst) + n_dst * cfg.hidden * es
        elif args.model == "gcn":      # one weight matrix over the aggregate
            flops = 2.0 * n_dst * din * cfg.hidden
            nbytes = (nnz + n_dst) * din * es + 4 * (nnz + 2 * n_dst) + n_dst * cfg.hidden * es
        else:                          # projection once per source row, then fp32 rows through the softmax gather
            n_src = U_avg / group if k == 1 else shb.n_dst(k - 1)
            flops = 2.0 * n_src * din * cfg.hidden
            nbytes = n_src * din * es + (nnz + n_dst) * cfg.hidden * 4 + 4 * (nnz + 2 * n_dst) + n_dst * cfg.hidden * es
        stage_work["sage_l%d" % k] = {"bound": "hbm+mfma", "bytes": group * nbytes, "flops": group * flops}
        din = cfg.hidden
    for name, w in stage_work.items():
        t = stage[name] * 1e-3
        w["GBps"] = round(w["bytes"] / t / 1e9, 1)
        if "flops" in w:
            w["TFLOPs"] = round(w["flops"] / t / 1e12, 2)

    out = {
        "metric": "micrograph batches/s",
        "value": args.steps * group / elapsed,
        "unit": "batches/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAME[str(X.dtype)], "data": "synthetic",
        "config": {"workload": cfg.name, "n_vertices": cfg.n_vertices, "n_edges": g.n_edges,
                   "feature_dim": cfg.d, "batch": cfg.batch, "fanouts": cfg.fanouts,
                   "hidden": cfg.hidden, "group": group, "merged_layers": merge, "slots_per_batch": shb.n_slots,
                   "streams": n_streams, "backward": bool(args.backward), "layer": args.model},
        "gather_GBps": gather_gbps,
        "gather_frac_of_hbm_peak": gather_gbps / HBM_PEAK_GBPS,
        "unique_rows_per_step": U_avg,
        "unique_over_valid_slots": U_sum / max(valid_sum, 1),
        "unique_group_over_sum_of_per_batch_unique": (U_sum / U_per_batch_sum) if group > 1 else 1.0,
        "valid_slot_fraction": valid_sum / (n_replay * group * shb.n_slots),
        "stage_ms": {k: round(v, 5) for k, v in stage.items()},
        "stage_work": stage_work,
        "roofline": {"kernel": "gather_rows", "bound": "hbm", "achieved": gather_gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gather_gbps / HBM_PEAK_GBPS,
                     "traffic": (gather_bytes * GATHER_TRAFFIC_OVER_ALGORITHMIC[row_bytes]
                                 if row_bytes in GATHER_TRAFFIC_OVER_ALGORITHMIC else None),
                     "algorithmic_bytes_per_launch": gather_bytes,
                     "avg_launch_ms": gather_ms_avg, "launch_ms_percentiles": gather_pct,
                     "empty_event_pair_ms": empty_ms_avg,
                     "achieved_net_of_marker_cost": gather_bytes / (gather_ms_net * 1e-3) / 1e9},
    }
    if not args.no_cpu_baseline and args.model == "sage":   # the oracle's whole-batch chain is the GraphSAGE one
        out["cpu_baseline"] = cpu_baseline(cfg, g, X, W, group, args.cpu_seconds)
    print(json.dumps(out))



def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is the single-GPU hot path (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.model != "sage" and args.backward and (args.dedup or args.layerwise):
        print("bench.py: --backward over deduplicated frontiers is built for the GraphSAGE-mean layer "
              "(slot-tree batches train all three layer kinds)", file=sys.stderr)
        sys.exit(2)
    if args.dedup or args.layerwise:
        return main_dedup(args)
    if args.backward or args.model != "sage":
        return main_variant(args)
    return main_headline(args)


if __name__ == "__main__":
    main()
