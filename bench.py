#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

Default workload (the largest configuration that fits one GPU, the fifth of the five): one share of the
trillion-edge run - 2-layer GraphSAGE-mean 64 -> 128 -> 16 on an R-MAT scale-24 local subgraph with edge
factor 256 (2^24 nodes, 2^32 local edges, int32 indices / int64 offsets), features 64-dim bf16 ~N(0,1)
(fp32 arithmetic), 16 classes, stand-in global degrees for the 255 missing shares, full-graph mode.

One timed step = grp_train_step on the share + grp_aggregate (shrinkage factors) over 256 resident
partition gradients (this share's and 255 seeded stand-ins): one per-worker body plus the
scale-and-reduce of the paper's phase-parallel algorithm.  The share is generated as sorted rows and
adopted once (grp_partition_from_csr) before the timed region; all inputs are resident in HBM.
Metric: per-partition train-step edges/s = nnz_used / t_step.

Prints ONE JSON line with `roofline` (dominant kernel, timed with HIP events on the launch stream in a
second, separately profiled pass over the same steps) and `cpu_baseline` (the fp64 numpy oracle timed on
the host on the same model at R-MAT scale 14 with the same edge factor, with one BLAS thread and with all).
`--workload c2-step` is the second configuration (MFMA-bound), the other names are evidence runs.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X published HBM3E bandwidth
PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X published dense fp32 matrix rate

# HBM bytes per launch of a kernel in a workload come from rocprofv3 --pmc runs of this script (FETCH_SIZE,
# then WRITE_SIZE, scaled by what the same counter reads for a plain copy); their summaries under profiles/
# carry one line `traffic_bytes_per_launch <workload> <kernel> <fetch bytes> <write bytes>` per kernel.
def _traffic_from_profiles(workload):
    table = {}
    pdir = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not name.endswith((".md", ".txt")):
            continue
        for line in open(os.path.join(pdir, name), encoding="utf-8"):
            f = line.strip().strip("`").split()
            if len(f) == 5 and f[0] == "traffic_bytes_per_launch" and f[1] == workload:
                table[f[2]] = {"fetch": float(f[3]), "write": float(f[4]), "source": f"profiles/{name}"}
    return table


GRAPH_SEED = 2602018722
N_NODES, N_EDGES, RMAT_SCALE = 2_400_000, 62_000_000, 22
K_PARTS, PART_SEED, PART_ID = 8, 1, 0
DIMS = [100, 256, 256, 47]


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def _time_steps(torch, fn, warmup, steps):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def _kernel_table(g, torch, fn, steps, detail=False):
    g.grp_profile_enable(2 if detail else 1)
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    prof = g.grp_profile_report()
    g.grp_profile_enable(False)
    kernels = {}
    for name, r in prof.items():
        kernels[name] = dict(launches_per_step=r["launches"] / steps, avg_us=r["ms"] / r["launches"] * 1e3,
                             ms_per_step=r["ms"] / steps,
                             gflops=r["flops"] / r["ms"] / 1e6 if r["ms"] > 0 else 0.0,
                             gbs=r["bytes"] / r["ms"] / 1e6 if r["ms"] > 0 else 0.0)
    for name in sorted(kernels, key=lambda k: -kernels[k]["ms_per_step"]):
        k = kernels[name]
        log(f"  {name:28s} {k['launches_per_step']:5.1f} launches/step {k['ms_per_step']:9.4f} ms/step "
            f"{k['gflops'] / 1e3:8.2f} TFLOP/s {k['gbs']:9.1f} GB/s")
    return kernels


def _device_copy_gbs(torch, dev):
    """Measured read+write rate of a plain 1 GiB device-to-device copy (the practical HBM ceiling that
    the published 8 TB/s peak is quoted beside)."""
    src = torch.ones(1 << 28, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 10
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    del src, dst
    return 2.0 * (1 << 30) / dt / 1e9


def _roofline(kernels, traffic_table):
    """The dominant kernel against its roofline; `traffic` = counter-measured HBM bytes per launch if a
    committed rocprofv3 --pmc summary has them for this workload and kernel."""
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    k = kernels[dom]
    if dom.startswith("gemm") and "reduce" not in dom:
        r = dict(kernel=dom, bound="mfma", achieved=k["gflops"] / 1e3, peak=PEAK_FP32_MFMA_TFLOPS, unit="TFLOP/s",
                 frac=k["gflops"] / 1e3 / PEAK_FP32_MFMA_TFLOPS)
    else:
        r = dict(kernel=dom, bound="hbm", achieved=k["gbs"], peak=PEAK_HBM_GBS, unit="GB/s", frac=k["gbs"] / PEAK_HBM_GBS)
    t = traffic_table.get(dom.split("[")[0])
    r["traffic"] = t["fetch"] + t["write"] if t else None
    if t:
        r["traffic_source"] = t["source"]
        if r["bound"] == "hbm":     # counter-measured bytes over the live launch time
            r["achieved_traffic_GBs"] = r["traffic"] / (k["avg_us"] * 1e-6) / 1e9
            r["traffic_frac_of_peak"] = r["achieved_traffic_GBs"] / PEAK_HBM_GBS
    r["avg_launch_us"] = k["avg_us"]
    r["launches_per_step"] = k["launches_per_step"]
    r["algorithmic_bytes_per_launch"] = k["gbs"] * 1e9 * k["avg_us"] * 1e-6
    return r


def _spmm_table(kernels, traffic_table):
    """Per SpMM kernel: algorithmic GB/s, counter-measured GB/s and the ratio of the two byte counts (how much
    more than the compulsory bytes the launch moved), where counters exist."""
    out = {}
    for name, k in kernels.items():
        if not name.startswith("spmm_rows"):
            continue
        e = dict(launches_per_step=k["launches_per_step"], avg_us=k["avg_us"], algorithmic_GBs=k["gbs"],
                 algorithmic_frac_of_peak=k["gbs"] / PEAK_HBM_GBS)
        t = traffic_table.get(name.split("[")[0])
        if t:
            e["counter_GBs"] = (t["fetch"] + t["write"]) / (k["avg_us"] * 1e-6) / 1e9
            e["counter_frac_of_peak"] = e["counter_GBs"] / PEAK_HBM_GBS
            e["wasted_traffic_factor"] = (t["fetch"] + t["write"]) / (k["gbs"] * 1e9 * k["avg_us"] * 1e-6)
        out[name] = e
    return out


def _timed_steps(torch, fn, warmup, steps):
    """Exactly `steps` calls between two synchronisations: (wall seconds per step, median of the per-step HIP
    event intervals in seconds)."""
    for _ in range(warmup):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    return dt, per[len(per) // 2] * 1e-3


def _oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        return os.cpu_count() or 1


def run_evidence_workload(args, g, synth, torch, dev):
    """Evidence runs for the configurations other than the headline one: real shapes, synthetic data,
    one JSON line each.  Graphs are generated directly as local subgraphs (one partition's share)."""
    import numpy as np
    wl = args.workload
    if args.copy_calibration:
        cal_src = torch.ones(1 << 28, device=dev)      # 1 GiB read + 1 GiB written by one plain copy kernel
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()
        del cal_src, cal_dst
    out = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "data": "synthetic", "device_copy_GBs": _device_copy_gbs(torch, dev)}
    if wl == "aggregate-stress":
        K, P = 64, 1 << 26                                  # 17 GB of gradients: shows the kernel's bandwidth
        grads = torch.empty(K, P, device=dev).normal_()
        stats = g.new_stats(K, device=dev)
        upd = torch.empty(P, device=dev)
        fn = lambda: g.grp_aggregate(grads, P, stats, K, P, g.EST_NONE, upd)
        dt = _time_steps(torch, fn, args.warmup, args.steps)
        kernels = _kernel_table(g, torch, fn, args.steps, detail=args.shapes)
        out.update(metric="aggregated gradient bytes/s (K=64, P=2^26; non-config stress shape)", unit="GB/s",
                   value=4.0 * P * (K + 1) / dt / 1e9, ms_per_step=dt * 1e3, dtype="f32",
                   config={"workload": "aggregate-stress: K=64 partition gradients of P=2^26 floats"},
                   roofline=_roofline(kernels, _traffic_from_profiles(wl)), kernels=kernels)
        print(json.dumps(out), flush=True)
        return

    if wl == "c1-step":
        # configuration 1 (the correctness configuration): 10,000 nodes, 100,000 uniform edges, K = 4, GCN-2 hidden 64.
        # ~6 k edges per partition: launch-bound, so one iteration (4 steps + aggregate + optimizer step) is
        # also timed as a captured HIP graph.
        N, E, K, dims = 10_000, 100_000, 4, [64, 64, 8]
        src, dst = synth.uniform_graph(N, E, seed=GRAPH_SEED - 2 + 1, device=dev)
        parts = [g.grp_partition(src, dst, N, K, PART_SEED, p) for p in range(K)]
        model = g.model_desc(g.ARCH_GCN, dims)
        opts = g.step_opts(estimator=g.EST_SHRINKAGE, full_graph=True)
        xg = synth.normal_matrix(N, dims[0], GRAPH_SEED, device=dev)
        yg = synth.labels(N, dims[-1], GRAPH_SEED, device=dev)
        l2gs = [torch.from_numpy(p.array("l2g")).to(dev) for p in parts]
        xs = [xg[i].contiguous() for i in l2gs]
        ys = [yg[i].contiguous() for i in l2gs]
        theta = synth.model_weights("gcn", dims, GRAPH_SEED, device=dev)
        P = g.grp_param_count(model)
        ld = (P + 3) // 4 * 4
        grads = torch.zeros(K, ld, device=dev)
        stats = g.new_stats(K, device=dev)
        upd = torch.zeros(P, device=dev)
        wss = [torch.empty(g.grp_step_workspace_bytes(p, model, opts), dtype=torch.uint8, device=dev) for p in parts]
        opt = g.optimizer_desc(g.OPT_SGD, lr=1e-6)           # a tiny rate: every iteration does essentially the same work

        def fn():
            for p in range(K):
                g.grp_train_step(parts[p], model, opts, xs[p], ys[p], None, theta, wss[p], grads[p],
                                 stats[p * g.STATS_BYTES:(p + 1) * g.STATS_BYTES])
            g.grp_aggregate(grads, ld, stats, K, P, g.EST_SHRINKAGE, upd)
            g.grp_optimizer_step(opt, P, 1, theta, upd)
        lanes = [torch.cuda.Stream() for _ in range(K)]       # default priority

        def fn_lanes():            # the partitions of a phase are independent: one stream each, joined before the reduction
            main = torch.cuda.current_stream()
            ready = main.record_event()
            for p in range(K):
                lanes[p].wait_event(ready)
                g.grp_train_step(parts[p], model, opts, xs[p], ys[p], None, theta, wss[p], grads[p],
                                 stats[p * g.STATS_BYTES:(p + 1) * g.STATS_BYTES], stream=lanes[p])
            for p in range(K):
                main.wait_stream(lanes[p])
            g.grp_aggregate(grads, ld, stats, K, P, g.EST_SHRINKAGE, upd)
            g.grp_optimizer_step(opt, P, 1, theta, upd)

        def captured(f):
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                f()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                f()
            return graph
        dt = _time_steps(torch, fn, args.warmup, args.steps)
        dt_lanes = _time_steps(torch, fn_lanes, args.warmup, args.steps)
        graph, graph_lanes = captured(fn), captured(fn_lanes)
        dt_graph = _time_steps(torch, graph.replay, args.warmup, args.steps)
        dt_graph_lanes = _time_steps(torch, graph_lanes.replay, args.warmup, args.steps)
        kernels = _kernel_table(g, torch, fn, args.steps, detail=args.shapes)
        nnz = sum(p.nnz for p in parts)
        best = min(dt, dt_lanes, dt_graph, dt_graph_lanes)
        out.update(metric="train-step edges/s over the 4 partitions (fwd+bwd), one iteration = 4 steps + aggregate + optimizer",
                   unit="edges/s", value=nnz / best, ms_per_step=best * 1e3, dtype="f32",
                   config={"workload": f"c1-step: GCN-2 {dims}, {N} nodes / {E} uniform edges, K={K}, local edges {nnz}",
                           "ms_per_iteration_eager": dt * 1e3, "ms_per_iteration_hip_graph": dt_graph * 1e3,
                           "ms_per_iteration_eager_4_streams": dt_lanes * 1e3,
                           "ms_per_iteration_hip_graph_4_streams": dt_graph_lanes * 1e3, "params": P},
                   roofline=_roofline(kernels, {}), kernels=kernels)
        print(json.dumps(out), flush=True)
        return

    if wl == "c2-partition-build":
        # the partition builders on the headline graph (what a super-epoch switch costs): one partition of 8 by
        # hash from the whole edge list, the one-off split into 8 chunks, base + swept chunk from the chunks,
        # the 1-hop halo variant and the weighted variant.  One "step" = one grp_partition call.
        src, dst = synth.rmat_graph(RMAT_SCALE, N_EDGES, seed=GRAPH_SEED, n_nodes=N_NODES, device=dev)
        ew = synth.edge_weights(N_EDGES, GRAPH_SEED, device=dev)
        torch.cuda.synchronize()

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps

        def build(make):
            def fn():
                p = make()
                fn.nnz = p.nnz
                p.destroy()
            return fn
        reps = max(3, args.steps // 5)
        full = build(lambda: g.grp_partition(src, dst, N_NODES, K_PARTS, PART_SEED, PART_ID))
        dt_full = timed(full, reps)
        t0 = time.perf_counter()
        ck = g.grp_chunks_build(src, dst, N_NODES, K_PARTS, PART_SEED)
        torch.cuda.synchronize()
        dt_chunks = time.perf_counter() - t0
        alone = build(lambda: g.grp_partition_from_chunks(ck, 0, 0))
        pair = build(lambda: g.grp_partition_from_chunks(ck, 0, 3))
        halo = build(lambda: g.grp_partition_halo(src, dst, N_NODES, K_PARTS, PART_SEED, PART_ID, 1))
        wgt = build(lambda: g.grp_partition_weighted(src, dst, ew, N_NODES, K_PARTS, PART_SEED, PART_ID))
        times = {"grp_partition_ms": dt_full * 1e3, "grp_chunks_build_once_ms": dt_chunks * 1e3,
                 "from_chunks_base_alone_ms": timed(alone, reps) * 1e3, "from_chunks_base_plus_swept_ms": timed(pair, reps) * 1e3,
                 "grp_partition_halo_1hop_ms": timed(halo, 3) * 1e3, "grp_partition_weighted_ms": timed(wgt, 3) * 1e3,
                 "local_edges": {"hash": full.nnz, "base_alone": alone.nnz, "base_plus_swept": pair.nnz, "halo": halo.nnz}}
        ck.destroy()
        # the feature movement of a switch: this partition's rows of the global feature matrix
        part0 = g.grp_partition(src, dst, N_NODES, K_PARTS, PART_SEED, PART_ID)
        l2g0 = torch.from_numpy(part0.array("l2g")).to(dev)
        xg = synth.normal_matrix(N_NODES, DIMS[0], GRAPH_SEED, device=dev)
        dt_gather = timed(lambda: g.grp_gather_rows(xg, l2g0), reps)
        times["gather_feature_rows_ms"] = dt_gather * 1e3
        times["gather_feature_rows_GBs"] = (2.0 * part0.n * DIMS[0] * 4 + 8.0 * part0.n) / dt_gather / 1e9
        part0.destroy()
        del xg, l2g0
        kernels = _kernel_table(g, torch, full, reps)        # the pass over the edge list
        dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
        out.update(metric="edges/s scanned by grp_partition (one partition of 8 from the whole edge list)", unit="edges/s",
                   value=N_EDGES / dt_full, ms_per_step=dt_full * 1e3, dtype="int64", steps=reps,
                   config={"workload": "c2-partition-build: the partition builders on the R-MAT 2.4M-node / 62M-edge graph, K = c = 8",
                           **times},
                   roofline={"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["gbs"], "peak": PEAK_HBM_GBS,
                             "unit": "GB/s", "frac": kernels[dom]["gbs"] / PEAK_HBM_GBS, "traffic": None,
                             "avg_launch_us": kernels[dom]["avg_us"],
                             "whole_call_GBs": 16.0 * N_EDGES / dt_full / 1e9}, kernels=kernels)
        print(json.dumps(out), flush=True)
        return

    if wl == "c2-minibatch-epoch":
        # the loop as the paper's experiments run it, on the headline graph: 8 hash partitions trained in turn on
        # the one GPU (phase-parallel, M = 1 worker's worth of memory at a time is not needed: all 8 are resident),
        # mini-batches of 1024 seeds with fanouts (15, 10, 5) over every partition's training nodes (8 % of the
        # nodes, the share of the products-sized dataset), shrinkage factor per batch, Adam, dropout 0.5.
        src, dst = synth.rmat_graph(RMAT_SCALE, N_EDGES, seed=GRAPH_SEED, n_nodes=N_NODES, device=dev)
        parts = [g.grp_partition(src, dst, N_NODES, K_PARTS, PART_SEED, p) for p in range(K_PARTS)]
        del src, dst
        dims = [100, 256, 256, 47]
        model = g.model_desc(g.ARCH_SAGE_MEAN, dims)
        xg = synth.normal_matrix(N_NODES, dims[0], GRAPH_SEED, device=dev)
        yg = synth.labels(N_NODES, dims[-1], GRAPH_SEED, device=dev)
        tmg = synth.train_mask(N_NODES, 0.08, GRAPH_SEED, device=dev)
        l2gs = [torch.from_numpy(p.array("l2g")).to(dev) for p in parts]
        xs = [xg[i].contiguous() for i in l2gs]
        ys = [yg[i].contiguous() for i in l2gs]
        masks = [tmg[i].contiguous() for i in l2gs]
        del xg, yg, tmg
        theta = synth.model_weights("sage", dims, GRAPH_SEED, device=dev)
        epochs = max(1, args.steps // 10)

        def timed_epochs(lanes, graphs=False):
            tr = g.MiniBatchTrainer(parts, model, xs, ys, masks, theta, g.EST_SHRINKAGE, K_PARTS, 1024, (15, 10, 5), 7,
                                    g.optimizer_desc(g.OPT_ADAM, lr=0.003), dropout_rate=0.5, dropout_seed=1, lanes=lanes,
                                    graphs=graphs)
            for _ in range(max(1, args.warmup // 3)):
                tr.run_epoch()
            torch.cuda.synchronize()
            first = len(tr.history)
            t0 = time.perf_counter()
            for _ in range(epochs):
                tr.run_epoch()
            torch.cuda.synchronize()
            return tr, first, (time.perf_counter() - t0) / epochs
        tr, first, dt_one = timed_epochs(1)
        tr, first, dt_threads = timed_epochs(4)              # four host threads, each with its stream and workspace
        losses_eager = tr.losses()
        tr, first, dt = timed_epochs(8, graphs=True)         # one host thread replaying captured steps on eight streams
        assert tr.losses() == losses_eager, "the captured steps must reproduce the uncaptured ones bit for bit"
        used = sum(int(g.read_stats(h)["nnz_used"].sum()) for h in tr.history[first:]) / epochs
        out.update(metric="sampled edges/s over one mini-batch epoch of all 8 partitions (fwd+bwd, aggregate, Adam)",
                   unit="edges/s", value=used / dt, ms_per_step=dt * 1e3, dtype="f32", steps=epochs,
                   config={"workload": f"c2-minibatch-epoch: SAGE-mean-3 {dims}, fanouts (15,10,5), 1024 seeds per batch, "
                                       f"8 partitions of the R-MAT 2.4M-node / 62M-edge graph, {sum(tr.n_train)} training nodes",
                           "ms_per_epoch": dt * 1e3, "launch": "captured steps (HIP graphs) replayed on 8 streams by one host thread",
                           "ms_per_epoch_uncaptured_one_host_thread": dt_one * 1e3,
                           "ms_per_epoch_uncaptured_four_host_threads": dt_threads * 1e3,
                           "iterations_per_epoch": tr.iters,
                           "train_steps_per_epoch": tr.iters * K_PARTS, "sampled_edges_per_epoch": used,
                           "losses_first_last": [tr.losses()[0], tr.losses()[-1]]},
                   roofline=None)
        print(json.dumps(out), flush=True)
        return

    if wl in ("c2-gat-step", "c2-dropout-step", "c2-weighted-step"):
        # the headline workload's partition with the attention model in place of GraphSAGE, with
        # GraphSAGE and dropout 0.5 on the hidden layers, or with weighted edges (weighted-mean GraphSAGE)
        src, dst = synth.rmat_graph(RMAT_SCALE, N_EDGES, seed=GRAPH_SEED, n_nodes=N_NODES, device=dev)
        if wl == "c2-weighted-step":
            ew = synth.edge_weights(N_EDGES, GRAPH_SEED, device=dev)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            part = g.grp_partition_weighted(src, dst, ew, N_NODES, K_PARTS, PART_SEED, PART_ID)
            torch.cuda.synchronize()
            print(f"[bench] weighted partition built in {(time.perf_counter() - t0) * 1e3:.1f} ms", file=sys.stderr, flush=True)
            del ew
        else:
            part = g.grp_partition(src, dst, N_NODES, K_PARTS, PART_SEED, PART_ID)
        del src, dst
        l2g = torch.from_numpy(part.array("l2g")).to(dev)
        dims = [100, 256, 256, 47]
        gat = wl == "c2-gat-step"
        model = g.model_desc(g.ARCH_GAT if gat else g.ARCH_SAGE_MEAN, dims)
        opts = g.step_opts(estimator=g.EST_SHRINKAGE, full_graph=True, dropout_rate=0.5 if wl == "c2-dropout-step" else 0.0,
                           dropout_seed=1)
        x = synth.normal_matrix(N_NODES, dims[0], GRAPH_SEED, device=dev)[l2g].contiguous()
        y = synth.labels(N_NODES, dims[-1], GRAPH_SEED, device=dev)[l2g].contiguous()
        theta = synth.model_weights("gat" if gat else "sage", dims, GRAPH_SEED, device=dev)
        P = g.grp_param_count(model)
        grad = torch.zeros((P + 3) // 4 * 4, device=dev)
        stats = g.new_stats(1, device=dev)
        ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=dev)
        fn = lambda: g.grp_train_step(part, model, opts, x, y, None, theta, ws, grad, stats)
        dt = _time_steps(torch, fn, args.warmup, args.steps)
        kernels = _kernel_table(g, torch, fn, args.steps, detail=args.shapes)
        out.update(metric="per-partition train-step edges/s (fwd+bwd)", unit="edges/s", value=part.nnz / dt,
                   ms_per_step=dt * 1e3, dtype="f32",
                   config={"workload": (f"c2-gat-step: GAT-3 (one head) {dims}" if gat else
                                        f"c2-dropout-step: SAGE-mean-3 {dims} with dropout 0.5" if wl == "c2-dropout-step" else
                                        f"c2-weighted-step: SAGE-mean-3 {dims} on weighted edges (weighted mean)") +
                                       f", partition 0 of 8 of the R-MAT 2.4M-node / 62M-edge graph, n={part.n}, nnz={part.nnz}",
                           "params": P},
                   roofline=_roofline(kernels, {}), kernels=kernels)
        print(json.dumps(out), flush=True)
        return

    big_csr = None
    if wl in ("c4-spmm", "c4-step"):
        scale, n, E, seed, F0, bf16 = 22, 1 << 22, 100_000_000, GRAPH_SEED - 2 + 4, 128, False
    elif wl in ("c5-spmm", "c5-step"):
        # configuration 5 at its stated size: 2^24 nodes, edge factor 256 = 2^32 edges
        scale, n, E, seed, F0, bf16 = 24, 1 << 24, 1 << 32, GRAPH_SEED - 2 + 5, 64, True
        if args.small:
            scale, n, E = 20, 1 << 20, 1 << 28
    else:                                                    # c3-step
        scale, n, E, seed, F0, bf16 = 23, 7_000_000, 100_000_000, GRAPH_SEED - 2 + 3, 128, True
    t0 = time.time()
    missing = {"c3-step": 15, "c5-spmm": 255, "c5-step": 255}.get(wl, 0)    # the other partitions' shares of each node's in-degree
    if wl.startswith("c5"):
        # generated as sorted rows and adopted as they are: an edge list of 2^32 edges plus a sort of it would not fit
        rowptr, col = synth.rmat_local_csr(scale, E, seed=seed, n_nodes=n, device=dev, chunk=1 << 28, slice_edges=1 << 28,
                                           progress=lambda done, total: log(f"{wl}: generated {done} of {total} edges"))
        d_global = synth.stand_in_global_degree(rowptr[1:] - rowptr[:-1], torch.arange(n, device=dev), seed, missing)
        torch.cuda.synchronize()
        t1 = time.time()
        part = g.grp_partition_from_csr(rowptr, col, n, d_global_in=d_global)
        torch.cuda.synchronize()
        log(f"{wl}: grp_partition_from_csr took {time.time() - t1:.2f}s")
        big_csr = (rowptr, col)
    else:
        src, dst = synth.rmat_graph(scale, E, seed=seed, n_nodes=n, device=dev, chunk=1 << 28,
                                    progress=lambda done, total: log(f"{wl}: generated {done} of {total} edges"))
        torch.cuda.synchronize()
        d_global = None
        if missing:
            d_local = torch.bincount(dst, minlength=n)
            d_global = synth.stand_in_global_degree(d_local, torch.arange(n, device=dev), seed, missing)
        part = g.grp_partition_from_local_coo(src, dst, n, d_global_in=d_global)
        del src, dst
    nnz = part.nnz
    torch.cuda.empty_cache()
    log(f"{wl}: local graph n={n} nnz={nnz} generated and built in {time.time() - t0:.1f}s")
    traffic = _traffic_from_profiles(wl) if not args.small else {}

    if wl.endswith("-spmm"):
        F = 256 if wl == "c4-spmm" else 64
        x = synth.normal_matrix(n, F, seed, device=dev)
        if bf16:
            x = synth.to_bf16_rne(x)
        y = torch.empty(n, F, device=dev)
        dt_code = g.DTYPE_BF16 if bf16 else g.DTYPE_FP32

        def fn():
            g.grp_spmm(part, False, g.SCALE_MEAN, False, F, x, F, dt_code, y, F)      # forward (CSR)
            g.grp_spmm(part, True, g.SCALE_MEAN, False, F, x, F, dt_code, y, F)       # transposed (CSC)
        dt, dt_med = _timed_steps(torch, fn, args.warmup, args.steps)
        kernels = _kernel_table(g, torch, fn, args.steps, detail=args.shapes)
        el = 2 if bf16 else 4
        b_min = 4 * nnz + 8 * (n + 1) + el * F * n + 4 * F * n
        out.update(metric="SpMM edges/s (one forward + one transposed aggregation)", unit="edges/s",
                   value=2 * nnz / dt, ms_per_step=dt * 1e3, ms_per_step_median_hip_events=dt_med * 1e3,
                   dtype="bf16-stored, f32 accumulate" if bf16 else "f32",
                   config={"workload": f"{wl}: mean aggregation, F={F}, R-MAT scale {scale}, n={n}, nnz={nnz}",
                           "algorithmic_bytes_per_call": b_min, "no_reuse_bytes_per_call": nnz * (4 + el * F) + 4 * F * n},
                   roofline=_roofline(kernels, traffic), spmm=_spmm_table(kernels, traffic), kernels=kernels)
        print(json.dumps(out), flush=True)
        return

    # full train steps
    K_agg = 1
    if wl == "c4-step":
        dims = [128] + [256] * 7 + [64]
        model = g.model_desc(g.ARCH_GCN_RESIDUAL, dims)
        opts = g.step_opts(estimator=g.EST_NONE, full_graph=True)
        arch = "gcn"
        x = synth.normal_matrix(n, dims[0], seed, device=dev)
    elif wl == "c5-step":
        dims = [64, 128, 16]
        model = g.model_desc(g.ARCH_SAGE_MEAN, dims, feat_dtype=g.DTYPE_BF16)
        opts = g.step_opts(estimator=g.EST_SHRINKAGE, full_graph=True)
        arch = "sage"
        x = synth.to_bf16_rne(synth.normal_matrix(n, dims[0], seed, device=dev))
        K_agg = 256                                           # shrinkage aggregation of 256 partition gradients
    else:
        dims = [128, 256, 256, 172]
        model = g.model_desc(g.ARCH_SAGE_MEAN, dims, feat_dtype=g.DTYPE_BF16)
        train = torch.nonzero(synth.train_mask(n, 0.05, seed, device=dev)).flatten().to(torch.int32)
        seeds = train[:1024].contiguous()
        opts = g.step_opts(estimator=g.EST_BATCH_MIN_DIST, full_graph=False, seeds=seeds, fanouts=(15, 10, 5),
                           sampler_seed=7, batch_id=0)
        arch = "sage"
        x = synth.to_bf16_rne(synth.normal_matrix(n, dims[0], seed, device=dev))
    y = synth.labels(n, dims[-1], seed, device=dev)
    theta = synth.model_weights(arch, dims, seed, device=dev)
    P = g.grp_param_count(model)
    ld = (P + 3) // 4 * 4
    grads = torch.zeros(K_agg, ld, device=dev)
    stats = g.new_stats(K_agg, device=dev)
    update = torch.zeros(P, device=dev)
    ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=dev)
    log(f"{wl}: workspace {ws.numel() / 1e9:.2f} GB, P={P}")
    st0 = stats[:g.STATS_BYTES]

    def fn():
        g.grp_train_step(part, model, opts, x, y, None, theta, ws, grads[0], st0)
        if K_agg > 1:
            g.grp_aggregate(grads, ld, stats, K_agg, P, g.EST_SHRINKAGE, update)
    if K_agg > 1:
        # the other shares' gradients and statistics: seeded stand-ins around this share's (inputs of the reduction)
        g.grp_train_step(part, model, opts, x, y, None, theta, ws, grads[0], st0)
        torch.cuda.synchronize()
        noise = synth.normal_matrix(K_agg - 1, ld, seed, stream=41, std=0.05, device=dev)
        grads[1:] = grads[0][None, :] * (1.0 + noise)
        rec = g.read_stats(stats).copy()
        spread = synth.stream_bits(seed, 42, torch.arange(K_agg, dtype=torch.int64)).numpy() % 1000
        for p in range(1, K_agg):
            rec[p] = rec[0]
            rec[p]["R"] = float(int(rec[0]["R"] * (0.75 + 0.0005 * int(spread[p]))))
        stats.copy_(torch.from_numpy(rec.view(np.uint8).copy()).to(dev))
    dt, dt_med = _timed_steps(torch, fn, args.warmup, args.steps)
    dt_eager = dt
    if wl == "c3-step":
        # a chain of ~65 small launches: the host's launch cost bounds the uncaptured step, so the step is also
        # captured once in a HIP graph and the replays are timed (the same work: nothing in the graph depends on
        # the captured batch; a trainer rewrites the seed buffer and the device-resident batch id between replays)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        want = grads[0].clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):         # the stream of the warm-up: its helper stream exists
            fn()
        dt_graph, dt_graph_med = _timed_steps(torch, graph.replay, args.warmup, args.steps)
        assert torch.equal(grads[0], want), "the replayed step must reproduce the uncaptured one bit for bit"
        if dt_graph < dt:
            dt, dt_med = dt_graph, dt_graph_med
    kernels = _kernel_table(g, torch, fn, args.steps, detail=args.shapes)
    used = int(g.read_stats(stats)[0]["nnz_used"])
    k_layers = len(dims) - 1
    out.update(metric="per-partition train-step edges/s (fwd+bwd)", unit="edges/s", value=used / dt, ms_per_step=dt * 1e3,
               ms_per_step_median_hip_events=dt_med * 1e3,
               dtype="f32 (input features stored in bf16)" if wl in ("c3-step", "c5-step") else "f32",
               config={"workload": f"{wl}: dims {dims}, R-MAT scale {scale}, n={n}, nnz={nnz}, edges used per step {used}"
                                   + (f", + shrinkage aggregation of {K_agg} gradients" if K_agg > 1 else ""),
                       "params": P, "small": bool(args.small), "sliced_schedule": not args.no_slices,
                       **({"launch": "HIP graph replay" if dt < dt_eager else "uncaptured",
                           "ms_per_step_uncaptured": dt_eager * 1e3} if wl == "c3-step" else {})},
               edge_traversals_per_s=used / dt * (2 * k_layers - 1),
               roofline=_roofline(kernels, traffic), spmm=_spmm_table(kernels, traffic), kernels=kernels)
    if wl == "c5-step" and not args.no_cpu_baseline:
        out["cpu_baseline"] = _c5_cpu_baseline(synth, torch, seed, dims)
    print(json.dumps(out), flush=True)


def _c5_cpu_baseline(synth, torch, seed, dims, scale=14, edge_factor=256):
    """The oracle's train step + shrinkage aggregation on the same model and graph family at R-MAT scale 14 with
    the same edge factor (1/1024 of the configuration's nodes and edges: the oracle needs ~1.6 us per edge, about 13 s for the two timings), timed
    with one BLAS thread and with the default thread count.  A reported baseline, never tuned."""
    import numpy as np
    from oracle import coverage as ocov
    from oracle import step as ostep
    n, E = 1 << scale, (1 << scale) * edge_factor
    rowptr, col = synth.rmat_local_csr(scale, E, seed=seed, n_nodes=n)
    deg = rowptr[1:] - rowptr[:-1]
    dg = synth.stand_in_global_degree(deg, torch.arange(n), seed, 255)
    part = dict(n=n, nnz=E, l2g=np.arange(n), rowptr=rowptr.numpy(), col=col.numpy(),
                d_local_in=deg.numpy().astype(np.int32), d_global_in=dg.numpy())
    x = synth.to_bf16_rne(synth.normal_matrix(n, dims[0], seed)).to(torch.float32).double().numpy()
    y = synth.labels(n, dims[-1], seed).numpy()
    th = synth.model_weights("sage", dims, seed).double().numpy()

    def once():
        t0 = time.time()
        og, ost = ostep.train_step(part, "sage", dims, th, x, y, estimator=ocov.SHRINKAGE)
        ocov.aggregate([og] * 256, [ost] * 256, ocov.SHRINKAGE)
        return time.time() - t0
    threads = _oracle_threads()
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            t1 = once()
    except Exception:
        t1 = None
    tn = once()
    log(f"oracle at scale {scale}: {t1 if t1 is None else round(t1, 1)} s with 1 thread, {tn:.1f} s with {threads}")
    best = tn if t1 is None or tn < t1 else t1
    return {"value": E / best, "unit": "edges/s", "cores": threads if best == tn else 1, "kind": "oracle",
            "value_one_thread": None if t1 is None else E / t1, "value_all_threads": E / tn, "threads_all": threads,
            "sample": f"R-MAT scale {scale}, edge factor {edge_factor}: n={n}, nnz={E} (1/{(1 << 24) // n} of the configuration's "
                      f"2^24 nodes and 2^32 edges), same model {dims}, one oracle train_step + aggregation of 256 gradients; "
                      f"{tn:.1f} s with {threads} threads, {'n/a' if t1 is None else f'{t1:.1f}'} s with 1"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--small", action="store_true", help="scaled-down graph (debugging only; not a valid result)")
    ap.add_argument("--shapes", action="store_true", help="per-launch-shape kernel table on stderr (debugging)")
    ap.add_argument("--workload", default="c5-step",
                    choices=["c2-step", "c1-step", "c2-partition-build", "c2-minibatch-epoch", "c2-gat-step", "c2-dropout-step", "c2-weighted-step", "c3-step", "c4-step", "c4-spmm", "c5-spmm", "c5-step", "aggregate-stress"],
                    help="c5-step (default) is the headline workload, the largest configuration at its stated size; "
                         "c2-step is the second configuration, the others are evidence runs (each prints one JSON "
                         "line of the same form)")
    ap.add_argument("--no-slices", action="store_true",
                    help="build the partitions without the source-sliced schedule of their long rows (the aggregation then "
                         "walks them in 512-edge chunks, row by row): the reference point of the schedule's effect")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (partitions are processed in turn); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2602_01872_amd as g
    import synth

    g.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.no_slices:
        g.grp_set_slice_policy(1 << 62, 100)
    if args.workload != "c2-step":
        run_evidence_workload(args, g, synth, torch, dev)
        return
    n_nodes, n_edges, scale = N_NODES, N_EDGES, RMAT_SCALE
    if args.small:
        n_nodes, n_edges, scale = 240_000, 6_200_000, 18

    t0 = time.time()
    src, dst = synth.rmat_graph(scale, n_edges, seed=GRAPH_SEED, n_nodes=n_nodes, device=dev)
    torch.cuda.synchronize()
    log(f"graph generated on device in {time.time() - t0:.1f}s")

    model = g.model_desc(g.ARCH_SAGE_MEAN, DIMS)
    opts = g.step_opts(estimator=g.EST_SHRINKAGE, full_graph=True)
    P = g.grp_param_count(model)
    ld = (P + 3) // 4 * 4
    grads = torch.zeros(K_PARTS, ld, device=dev)
    stats = g.new_stats(K_PARTS, device=dev)
    theta = synth.model_weights("sage", DIMS, GRAPH_SEED, device=dev)
    update = torch.zeros(P, device=dev)

    # one-off: build the 8 partitions, run each once so that all 8 gradients are resident
    t0 = time.time()
    keep = None
    for p in range(K_PARTS):
        part = g.grp_partition(src, dst, n_nodes, K_PARTS, PART_SEED, p)
        n = part.n
        l2g = torch.from_numpy(part.array("l2g")).to(dev)
        # features / labels are functions of the global node id (same values for the oracle)
        x = synth.normal_matrix(n_nodes, DIMS[0], GRAPH_SEED, device=dev)[l2g].contiguous() if p == PART_ID else None
        if x is None:
            x = synth.normal_matrix(n, DIMS[0], GRAPH_SEED + p, device=dev)
        y = synth.labels(n_nodes, DIMS[-1], GRAPH_SEED, device=dev)[l2g].contiguous()
        ws = torch.empty(g.grp_step_workspace_bytes(part, model, opts), dtype=torch.uint8, device=dev)
        g.grp_train_step(part, model, opts, x, y, None, theta, ws, grads[p],
                         stats[p * g.STATS_BYTES:(p + 1) * g.STATS_BYTES])
        torch.cuda.synchronize()
        if p == PART_ID:
            keep = (part, x, y, ws)
        else:
            part.destroy()
            del ws, x, y
    log(f"8 partitions built and stepped once in {time.time() - t0:.1f}s")
    part, x, y, ws = keep
    nnz = part.nnz
    st_slice = stats[PART_ID * g.STATS_BYTES:(PART_ID + 1) * g.STATS_BYTES]

    def step():
        g.grp_train_step(part, model, opts, x, y, None, theta, ws, grads[PART_ID], st_slice)
        g.grp_aggregate(grads, ld, stats, K_PARTS, P, g.EST_SHRINKAGE, update)

    if args.copy_calibration:
        cal_src = torch.ones(1 << 28, device=dev)      # 1 GiB read + 1 GiB written by one elementwise kernel
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()
        del cal_src, cal_dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    edges_per_s = nnz / (dt / args.steps)
    log(f"{ms_per_step:.3f} ms/step, {edges_per_s:.3e} edges/s (n={part.n}, nnz={nnz})")

    # per-kernel pass: same steps with every launch bracketed by HIP events on the launch stream
    g.grp_profile_enable(2 if args.shapes else 1)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = g.grp_profile_report()
    g.grp_profile_enable(False)
    kernels = {}
    for name, r in prof.items():
        avg_ms = r["ms"] / r["launches"]
        kernels[name] = dict(launches_per_step=r["launches"] / args.steps, avg_us=avg_ms * 1e3,
                             ms_per_step=r["ms"] / args.steps,
                             gflops=r["flops"] / r["ms"] / 1e6 if r["ms"] > 0 else 0.0,
                             gbs=r["bytes"] / r["ms"] / 1e6 if r["ms"] > 0 else 0.0)
    roofline = _roofline(kernels, _traffic_from_profiles("c2-step") if not args.small else {})
    for name in sorted(kernels, key=lambda k: -kernels[k]["ms_per_step"]):
        k = kernels[name]
        log(f"  {name:18s} {k['launches_per_step']:5.1f} launches/step {k['ms_per_step']:8.4f} ms/step "
            f"{k['gflops'] / 1e3:8.2f} TFLOP/s {k['gbs']:9.1f} GB/s")

    out = {
        "metric": "per-partition train-step edges/s (fwd+bwd)", "value": edges_per_s, "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[1]: SAGE-mean-3 100-256-256-47, R-MAT 2.4M nodes / 62M edges, partition 0 of 8 "
                               "(hash), full-graph train step + shrinkage aggregation of 8 gradients",
                   "n_local": part.n, "nnz_local": nnz, "params": P, "small": bool(args.small)},
        "roofline": roofline,
        "kernels": kernels,
        # every layer aggregates forward and all but the first also over the transposed graph
        "edge_traversals_per_s": edges_per_s * (2 * 3 - 1),
        "device_copy_GBs": _device_copy_gbs(torch, dev),
    }

    if not args.no_cpu_baseline:
        from oracle import coverage as ocov
        from oracle import graph as ograph
        from oracle import step as ostep
        try:
            from threadpoolctl import threadpool_info
            threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count() or 1
        sh, dh = src.cpu().numpy(), dst.cpu().numpy()
        t0 = time.time()
        op = ograph.partition(sh, dh, n_nodes, K_PARTS, PART_SEED, PART_ID)
        t_part = time.time() - t0
        xh, yh, th = x.cpu().double().numpy(), y.cpu().numpy(), theta.cpu().double().numpy()
        t0 = time.time()
        og, ost = ostep.train_step(op, "sage", DIMS, th, xh, yh, estimator=ocov.SHRINKAGE)
        gh = grads.cpu().double().numpy()[:, :P]
        recs = g.read_stats(stats)
        ostats = [dict(S=int(r["S"]), sum_ratio=float(r["sum_ratio"]), R=float(r["R"])) for r in recs]
        ostats[PART_ID] = ost
        G, _ = ocov.aggregate([og if p == PART_ID else gh[p] for p in range(K_PARTS)], ostats, ocov.SHRINKAGE)
        t_cpu = time.time() - t0
        log(f"oracle: partition {t_part:.1f}s, train_step+aggregate {t_cpu:.1f}s on {threads} threads")
        out["cpu_baseline"] = {"value": op["nnz"] / t_cpu, "unit": "edges/s", "cores": threads, "kind": "oracle",
                               "sample": "the same partition 0 at full size, one oracle train_step + aggregate "
                                         f"({t_cpu:.1f} s); oracle partition build {t_part:.1f} s not included"}
        # full-size parity report (not asserted here; tests/ hold the assertions)
        bit_exact = all(np.array_equal(part.array(k), op[k]) for k in ("rowptr", "col", "colptr", "row", "l2g",
                                                                         "d_global_in"))
        gpu_g = gh[PART_ID]

        def tensor_errors(ref):
            off, errs = 0, {}
            for l in range(len(DIMS) - 1):
                for nm, cnt in ((f"W{l}", DIMS[l] * DIMS[l + 1]), (f"Wn{l}", DIMS[l] * DIMS[l + 1]), (f"b{l}", DIMS[l + 1])):
                    a, b = gpu_g[off:off + cnt], ref[off:off + cnt]
                    errs[nm] = float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))
                    off += cnt
            return errs

        # Hidden pre-activations within rounding distance of 0 can take either ReLU-derivative decision.
        # The oracle lists them; it is rerun with the decisions the library took at those elements (read
        # from its stored activations) and its own decisions everywhere else.
        _, ost_k = ostep.train_step(op, "sage", DIMS, th, xh, yh, estimator=ocov.SHRINKAGE, near_kink=4e-6)
        near = ost_k["near_kink"]
        decisions = {}
        for l in range(len(DIMS) - 2):
            el = [e for e in near if e[0] == l]
            if el:
                vals = g.read_activation(part, model, opts, ws, l, [e[1] for e in el], [e[2] for e in el])
                decisions.update({e: bool(v > 0) for e, v in zip(el, vals)})
        og_m, _ = ostep.train_step(op, "sage", DIMS, th, xh, yh, estimator=ocov.SHRINKAGE, relu_set=decisions)
        G_m, _ = ocov.aggregate([og_m if p == PART_ID else gh[p] for p in range(K_PARTS)], ostats, ocov.SHRINKAGE)
        upd = update.cpu().double().numpy()
        out["parity_full_size"] = {"partition_bit_exact": bool(bit_exact),
                                   "loss_rel_err": abs(float(recs[PART_ID]["loss"]) - ost["loss"]) / abs(ost["loss"]),
                                   "S_equal": int(recs[PART_ID]["S"]) == ost["S"],
                                   "R_equal": float(recs[PART_ID]["R"]) == ost["R"],
                                   "near_kink_elements": len(near),
                                   "grad_rel_err": tensor_errors(og_m),
                                   "update_rel_err": float(np.abs(upd - G_m).max() / max(np.abs(G_m).max(), 1e-30)),
                                   "grad_rel_err_oracle_decisions": tensor_errors(og),
                                   "note": "grad_rel_err / update_rel_err: the oracle takes the library's ReLU-derivative "
                                           "decision at the hidden pre-activations it finds within 4e-6 rms of zero and "
                                           "its own everywhere else; *_oracle_decisions: its own at those too"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
