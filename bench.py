#!/usr/bin/env python3
"""Benchmark of the micrograph hot path on one MI355X.

A *step* is one whole batch: hopgnn_sample -> hopgnn_pregather -> hopgnn_gather ->
L x hopgnn_sage_fwd for B fresh seeds, all on one stream, inputs resident in HBM,
no host synchronisation inside the timed region.  The forward-only step issues that
sequence through hopgnn_batch_fwd (one library call); consecutive steps alternate over
a few streams, each with its own buffers, so that the small kernels of one batch overlap
the next batch's.  The default workload is the
R-MAT 2^20-vertex shape (128 fp32 features, 1024 seeds, fanout [10,10], hidden 128).

Prints ONE JSON line: batches/s, the gather kernel's effective HBM GB/s against the
8 TB/s peak (timed with events inside the timed region), a per-stage breakdown, and
the CPU oracle timed on the host cores on a bounded sample of the same workload.
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
# FETCH_SIZE and WRITE_SIZE runs scaled by a plain copy kernel: 512-byte rows (workloads 2 and 4)
# profiles/gather_traffic_pmc.txt; 400-byte rows (workload 3; rows straddle cache lines)
# profiles/batch_traffic_pmc.txt.  Row sizes without a counter run report no traffic figure.
GATHER_TRAFFIC_OVER_ALGORITHMIC = {512: 1.012, 400: 1.077}
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0}
DTYPE_NAME = {"torch.float32": "f32", "torch.bfloat16": "bf16", "torch.float16": "f16"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload shape 1..5")
    ap.add_argument("--group", type=int, default=0, help="batches per pre-gather (0: the shape's default)")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams (each with its own buffers) that consecutive steps alternate over")
    ap.add_argument("--backward", action="store_true",
                    help="training steps: the layers' backward pass with in-place gradient accumulation and one "
                         "SGD update per step")
    ap.add_argument("--model", choices=["sage", "gcn", "gat"], default="sage",
                    help="layer type: GraphSAGE-mean (the headline workload), GCN-style mean, graph attention")
    ap.add_argument("--no-merge", action="store_true",
                    help="with a group > 1: run every batch's layers separately instead of one launch per layer "
                         "over the group's merged micrographs")
    ap.add_argument("--dedup", action="store_true",
                    help="sample per-micrograph deduplicated frontiers (hopgnn_sample_dedup): the same rows for the "
                         "seeds over fewer rows below them; one batch per pre-gather, forward only")
    ap.add_argument("--layerwise", action="store_true",
                    help="layer-wise sampled micrographs (the shape's fanouts are the budgets of draws per level)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    return ap.parse_args()


def cpu_baseline(cfg, g, X, W, group, budget_s):
    """Time the CPU oracle as it stands (single thread) on whole batches of the same workload."""
    import numpy as np

    import oracle
    from paper_2409_00657_amd import synth
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import ORC_DT, to_bits, weights_bits

    off = g.offsets.cpu().numpy()
    idx = g.indices.cpu().numpy()
    big = X.shape[0] > 4_000_000
    Xh = None if big else to_bits(X)
    wb = weights_bits(W)
    odt = ORC_DT[X.dtype]
    def one_group(it):
        """One group of whole batches; returns the seconds of its timed part."""
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
        T = len(ids[0])
        for b in range(group):
            oracle.forward(Xu, odt, ids[b], indptr, remap[b * T:(b + 1) * T], cfg.batch, cfg.fanouts, wb)
        return time.perf_counter() - t0

    done, t_total, it = 0, 0.0, 0
    while True:
        t_total += one_group(it)
        done += group
        it += 1
        if t_total >= budget_s or it >= 64:
            break
    out = {"value": done / t_total, "unit": "batches/s", "cores": 1, "kind": "oracle",
           "sample": "%d whole batches of %s (sample+pregather+gather+%d layers, fp64 C oracle, 1 thread)"
                     % (done, cfg.name, len(cfg.fanouts)),
           "seconds": round(t_total, 2)}
    # the same oracle on every core of this process's share: micrographs (here: whole groups) are
    # independent, so each thread runs its own groups (the C library holds no state and the calls
    # release the interpreter lock); the oracle itself is unchanged
    n_threads = min(16, len(os.sched_getaffinity(0)))
    if not big and n_threads > 1:
        from concurrent.futures import ThreadPoolExecutor
        wall = min(8.0, budget_s)
        t_start = time.perf_counter()

        def worker(w):
            n = 0
            while time.perf_counter() - t_start < wall:
                one_group(1000 + w * 4096 + n)
                n += 1
            return n
        with ThreadPoolExecutor(max_workers=n_threads) as pool:
            counts = list(pool.map(worker, range(n_threads)))
        elapsed = time.perf_counter() - t_start
        out["all_cores"] = {"value": sum(counts) * group / elapsed, "unit": "batches/s", "cores": n_threads,
                            "sample": "%d whole batches on %d threads, one group per thread at a time"
                                      % (sum(counts) * group, n_threads),
                            "seconds": round(elapsed, 2)}
    return out


def main_dedup(args):
    """The forward step over deduplicated frontiers: same JSON line, call-by-call sequence."""
    import torch

    from paper_2409_00657_amd import binding as hb
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import DedupPath

    hb.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
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


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is the single-GPU hot path (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.dedup or args.layerwise:
        if args.model != "sage" and args.backward:
            print("bench.py: --backward is built for the GraphSAGE-mean layer", file=sys.stderr)
            sys.exit(2)
        return main_dedup(args)

    import torch

    from paper_2409_00657_amd import binding as hb
    from paper_2409_00657_amd import synth
    from paper_2409_00657_amd.pipeline import HotPath

    hb.load_library()                      # fail loudly if the HIP library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    group = args.group or cfg.groups[0]
    g = cfg.make_graph(device=dev)
    X = cfg.make_features(device=dev)
    W = cfg.make_weights(device=dev)
    n_streams = max(1, args.streams)
    if args.model != "sage" and args.backward:
        print("bench.py: --backward is built for the GraphSAGE-mean layer", file=sys.stderr)
        sys.exit(2)
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


if __name__ == "__main__":
    main()
