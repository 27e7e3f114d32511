#!/usr/bin/env python3
"""Throughput of one full-batch training iteration (forward, reweighted loss, backward, update)
on one vertex-cut partition, on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--scale 1.0]

Prints ONE JSON line: partition edges per second per iteration (edges = directed adjacency
entries of the unmasked partition), the roofline of the kernel that takes the largest share of the
iteration (one template instance at one launch shape, timed live with HIP events on the launching
stream), the aggregation kernel's own line, and the CPU oracle timed on the same workload.  Inputs are
synthetic (seeded power-law graph shaped like the paper's dataset, N(0,1) features, uniform labels,
Glorot weights) and resident in HBM before the timed region.

With the default configuration (cfg1, the Reddit-shaped workload the metric is quoted on) the line also
carries an "also" object with the same measurement of cfg2 (bf16, DropEdge-K, short rows), cfg4 (all
eight partitions back to back, hidden 512) and cfg3 (the papers100M-shaped graph at full size, one partition
of 28M nodes), where the aggregation is bound by HBM rather than by the caches.  cfg3's graph is streamed
block by block into the library's piece-wise partition builder (the 1.6-billion-entry edge list is never held
whole; about 40 s of host work before its timed steps).
"""
from __future__ import annotations

import argparse
import gc
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F32_TFLOPS = 157.3
PEAK_MFMA_BF16_TFLOPS = 2500.0
HOST_WORKERS = 12     # threads for the host-side input generators (the GPU machine gives one GPU 16 cores)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_hash() -> str:
    """Hash of the kernel sources: a traffic profile is only quoted for the kernels it was taken on."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2308_03209_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        # the library's sources; gather_ceiling.hip is a stand-alone program and not part of any profiled kernel
        if name.endswith((".hip", ".cpp", ".h")) and name != "gather_ceiling.hip":
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def cpu_baseline(wl, sample_scale: float, cut: str = "random"):
    """Time the oracle (as it stands) on one iteration over partition 0 of the workload (scaled down in nodes
    and edges by sample_scale where the full size would take minutes; same average degree and model widths)."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import dropedge as o_dropedge
    from oracle import epoch as o_epoch
    from oracle import partition as o_partition
    from paper_2308_03209_amd import inputs

    ws = wl.scaled(sample_scale) if sample_scale != 1.0 else wl
    src, dst = inputs.workload_graph(ws)
    O = o_partition.build_partition(ws.n_nodes, src, dst, ws.n_parts, 0, inputs.SEED_CUT, method=cut)
    del src, dst
    ids = O["local2global"]
    dims = ws.layer_dims()
    X = inputs.node_features(ids, ws.d_feat, workers=HOST_WORKERS)
    if ws.dtype == "bf16":   # the oracle sees the features exactly as stored
        import torch
        X = torch.from_numpy(X).to(torch.bfloat16).float().numpy()
    X = X.astype(np.float64)
    multilabel = ws.loss == "sigmoid_bce"
    y = inputs.node_multilabels(ids, ws.n_classes) if multilabel else inputs.node_labels(ids, ws.n_classes)
    layers = inputs.model_params(ws.kind, dims)
    om = {"kind": ws.kind, "layers": [{k: v.astype(np.float64) for k, v in l.items()} for l in layers]}
    graph = o_dropedge.full_graph(O)
    if ws.dropedge_K:
        keep = o_dropedge.masks(O["n_edges"], ws.dropedge_K, ws.dropedge_p, inputs.SEED_MASKS)
        graph = o_dropedge.masked_graph(O, keep[o_dropedge.pick(inputs.SEED_MASKS, 0, ws.dropedge_K)])
    t0 = time.perf_counter()
    if multilabel:
        from oracle import loss as o_loss
        logits, saved = o_epoch.forward(om, graph, X, ws.dropout, inputs.SEED_DROPOUT, 0)
        _, dlogits = o_loss.weighted_sigmoid_bce(logits, y, O["dar_weight"], 1.0 / ws.n_nodes)
        o_epoch.backward(om, graph, saved, dlogits)
    else:
        o_epoch.partition_loss_and_grads(om, graph, X, y, O["dar_weight"], 1.0 / ws.n_nodes, ws.dropout,
                                         inputs.SEED_DROPOUT, 0)
    dt = time.perf_counter() - t0
    threads = max([int(i.get("num_threads", 1)) for i in threadpool_info()] + [1])
    what = "the workload itself" if sample_scale == 1.0 else f"the workload scaled x{sample_scale:g} in nodes and edges"
    return {"value": O["nnz"] / dt, "unit": "edges/s", "cores": threads, "kind": "oracle",
            "sample": f"one iteration on partition 0 of {what} "
                      f"({O['n_nodes']} nodes, {O['nnz']} directed edges, same widths), {dt:.1f} s; numpy fp64, "
                      f"BLAS threads for the dense products, one thread for the per-row aggregation loops"}


def build_partitions(wl, cut: str):
    """[(part_id, Partition, Masks or None)] for the workload's trained partitions."""
    from paper_2308_03209_amd import binding as B
    from paper_2308_03209_amd import inputs

    flags = B.CUT_DBH if cut == "dbh" else 0
    t0 = time.time()
    parts = []
    if wl.stream:
        # block by block into the piece-wise builder: one builder per trained partition, every block fed to each
        if cut != "random":
            raise SystemExit("bench.py: the streamed workload supports the random cut only (the degree-aware cut "
                             "needs every degree before the first edge is assigned)")
        stream = inputs.workload_stream(wl)
        builders = [B.PartitionBuilder(wl.n_nodes, wl.n_parts, i, inputs.SEED_CUT, 0) for i in wl.train_parts]
        seen = 0
        for k, (src, dst) in enumerate(stream.blocks(workers=HOST_WORKERS)):
            for bld in builders:
                bld.add_edges(src, dst)
            seen += len(src)
            if k % 4 == 3 or k == stream.n_blocks - 1:
                log(f"[bench] graph: block {k + 1} of {stream.n_blocks}, {seen} undirected edges so far "
                    f"({time.time() - t0:.0f} s)")
        log(f"[bench] graph: {wl.n_nodes} nodes, {seen} undirected edges streamed ({time.time() - t0:.1f} s)")
        built = [(i, bld.finish()) for i, bld in zip(wl.train_parts, builders)]
        log(f"[bench] partitions finished and uploaded ({time.time() - t0:.1f} s)")
    else:
        src, dst = inputs.workload_graph(wl, progress=lambda text: log(f"[bench] graph: {text} ({time.time() - t0:.0f} s)"))
        log(f"[bench] graph: {wl.n_nodes} nodes, {len(src)} undirected edges ({time.time() - t0:.1f} s)")
        built = []
        for i in wl.train_parts:
            t1 = time.time()
            built.append((i, B.build_partition(wl.n_nodes, src, dst, wl.n_parts, i, inputs.SEED_CUT, flags=flags)))
            log(f"[bench] partition {i}: built and uploaded in {time.time() - t1:.1f} s")
        del src, dst
    for part_id, P in built:
        masks = None
        if wl.dropedge_K:
            t1 = time.time()
            masks = B.dropedge_k(P, wl.dropedge_K, wl.dropedge_p, inputs.SEED_MASKS + part_id)   # synchronises
            log(f"[bench] partition {part_id}: {wl.dropedge_K} DropEdge masks drawn and compacted on the device in "
                f"{1e3 * (time.time() - t1):.1f} ms")
        parts.append((part_id, P, masks))
    return parts


def load_traffic(wl, scale: float):
    """bytes per launch by kernel instance from the committed rocprofv3 counter summary of this workload, if it
    was taken on the kernel sources of this tree; else (None, reason)."""
    path = os.path.join(ROOT, "profiles", f"cfg{wl.index}_traffic.json")
    if scale != 1.0:
        return None, "no counter profile for a scaled workload"
    if not os.path.exists(path):
        return None, f"no counter profile committed for this workload (profiles/cfg{wl.index}_traffic.json)"
    data = json.load(open(path))
    if data.get("kernel_source_hash") != kernel_source_hash():
        return None, (f"profiles/cfg{wl.index}_traffic.json was taken on other kernel sources "
                      f"({data.get('kernel_source_hash')}, tree {kernel_source_hash()}): not quoted")
    return data.get("bytes_per_launch", {}), None


def run_leg(wl, steps: int, warmup: int, cut: str, scale: float):
    """Builds the workload on the GPU, times `steps` iterations, returns the measurement as a dict."""
    import numpy as np
    import torch

    from paper_2308_03209_amd import binding as B
    from paper_2308_03209_amd import inputs
    from paper_2308_03209_amd import model as M
    from paper_2308_03209_amd import train as T

    log(f"[bench] workload {wl.name}: seeds graph={inputs.SEED_GRAPH + wl.index} perm={inputs.SEED_PERM + wl.index} "
        f"cut={inputs.SEED_CUT} masks={inputs.SEED_MASKS} features={inputs.SEED_FEATURES} labels={inputs.SEED_LABELS} "
        f"params={inputs.SEED_PARAMS}")
    dims = wl.layer_dims()
    model = M.Model(wl.kind, dims)
    model.load(inputs.model_params(wl.kind, dims))
    parts = build_partitions(wl, cut)
    # partitions are trained one after the other, so their activation buffers are shared
    pool = M.BufferPool(max(P.num_nodes for _, P, _ in parts)) if len(parts) > 1 else None
    tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    runs, nnz_total = [], 0
    for part_id, P, masks in parts:
        t0 = time.time()
        ids = P.host_array(B.ARR_LOCAL2GLOBAL)
        X = torch.from_numpy(inputs.node_features(ids, wl.d_feat, workers=HOST_WORKERS)).to(tdtype).cuda()
        if wl.loss == "sigmoid_bce":
            y = torch.from_numpy(inputs.node_multilabels(ids, wl.n_classes)).cuda()
        else:
            y = torch.from_numpy(inputs.node_labels(ids, wl.n_classes)).cuda()
        run = M.PartitionRunner(P, model, masks, dropout_q=wl.dropout, dropout_seed=inputs.SEED_DROPOUT,
                                dtype=wl.dtype, pool=pool, loss=wl.loss)
        runs.append((run, X, y, part_id))
        nnz_total += P.num_nnz
        log(f"[bench] partition {part_id}: {P.num_nodes} nodes, {P.num_nnz} directed edges "
            f"(features and buffers in {time.time() - t0:.1f} s)")
    c = 1.0 / wl.n_nodes
    trainer = T.Trainer(model, [T.PartitionData(run, X, y, inputs.SEED_MASKS + part_id) for run, X, y, part_id in runs],
                        c, wl.optimizer, wl.lr)
    # directed entries that survive a DropEdge-K mask, averaged over each partition's K masks (the masks are picked
    # uniformly): the second unit the throughput is quoted in
    kept_total = 0.0
    for _, P, masks in parts:
        if masks is None:
            kept_total += P.num_nnz
        else:
            kept = [int(np.unpackbits(masks.host_bits(k).view(np.uint8), bitorder="little")[:P.num_edges].sum())
                    for k in range(masks.count)]
            kept_total += 2.0 * float(np.mean(kept))
    for _ in range(warmup):
        trainer.step()
    torch.cuda.synchronize()
    B.profile_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]   # per-step spread only; `value` is wall time
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        trainer.step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    detail = B.profile_read()
    B.profile_enable(False)
    ms_per_step = 1e3 * dt / steps
    loss = float(runs[-1][0].loss.item())
    assert np.isfinite(loss), "loss is not finite"

    kernel_ms = sum(s["ms_total"] for s in detail.values())
    for name, s in sorted(detail.items(), key=lambda kv: -kv[1]["ms_total"]):
        n = max(s["launches"], 1)
        log(f"[shape] {name:62s} launches/step {s['launches'] / steps:5.1f}  avg ms {s['ms_total'] / n:8.4f}"
            f"  ms/step {s['ms_total'] / steps:8.3f}"
            f"  alg GB/s {s['alg_bytes'] / max(s['ms_total'], 1e-9) / 1e6:8.1f}"
            f"  alg TFLOP/s {s['alg_flops'] / max(s['ms_total'], 1e-9) / 1e9:7.2f}")
    log(f"[bench] kernels {kernel_ms / steps:.3f} ms/step of {ms_per_step:.3f} ms/step wall")

    traffic, traffic_note = load_traffic(wl, scale)

    def roofline(name: str):
        """One kernel instance at one launch shape: algorithmic bytes or flops of its launches over their summed
        duration (HIP events on the launching stream)."""
        s = detail[name]
        instance = name.split(" ")[0]
        avg_ms = s["ms_total"] / max(s["launches"], 1)
        out_r = {"kernel": name, "launches": s["launches"], "avg_ms": avg_ms}
        if instance.startswith("gemm_"):
            a = s["alg_flops"] / (s["ms_total"] * 1e-3) / 1e12
            peak = PEAK_MFMA_BF16_TFLOPS if "bf16" in instance else PEAK_MFMA_F32_TFLOPS
            out_r.update({"bound": "mfma", "achieved": a, "peak": peak, "unit": "TFLOP/s", "frac": a / peak})
        else:
            a = s["alg_bytes"] / (s["ms_total"] * 1e-3) / 1e9
            out_r.update({"bound": "hbm", "achieved": a, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": a / PEAK_HBM_GBS})
        out_r["traffic"] = traffic.get(instance) if traffic else None
        if out_r["traffic"] is None:
            out_r["traffic_note"] = traffic_note or "this kernel instance is not in the committed counter profile"
        else:
            # counter bytes (mean over the launches of this instance in the profiled run) over the live duration
            out_r["measured_traffic_GBps"] = out_r["traffic"] / (avg_ms * 1e-3) / 1e9
        if instance.startswith("aggregate_") and s["alg_flops"] > 0:
            # bytes the gather requests when no neighbour row is reused: entries * width * element size
            # (the kernel's flop count is 2 * entries * width)
            es = 2 if wl.dtype == "bf16" else 4
            out_r["gathered_GBps"] = s["alg_flops"] / 2 * es / (s["ms_total"] * 1e-3) / 1e9
        return out_r

    dominant = max(detail, key=lambda k: detail[k]["ms_total"])
    leg = {
        "value": nnz_total / (dt / steps), "unit": "edges/s", "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "dtype": wl.dtype,
        "step_ms_min_median_max": [step_ms[0], step_ms[len(step_ms) // 2], step_ms[-1]],
        "undirected_edges_per_s": 0.5 * nnz_total / (dt / steps),
        "kept_directed_edges_per_s": kept_total / (dt / steps),
        "config": {"workload": wl.name, "kind": wl.kind, "layers": wl.n_layers, "n_nodes": wl.n_nodes,
                   "partition_nodes": [r[0].n for r in runs], "partition_directed_edges": nnz_total,
                   "n_parts": wl.n_parts, "trained_parts": list(wl.train_parts), "d_feat": wl.d_feat,
                   "hidden": wl.hidden, "n_classes": wl.n_classes, "dropedge_K": wl.dropedge_K,
                   "reweighting": "DAR", "optimizer": wl.optimizer, "dropout": wl.dropout, "loss": wl.loss, "cut": cut},
        "roofline": roofline(dominant),
        "loss": loss,
    }
    aggs = [k for k in detail if k.startswith("aggregate_")]
    if aggs:
        top = max(aggs, key=lambda k: detail[k]["ms_total"])
        if top != dominant:
            leg["roofline_spmm"] = roofline(top)
        leg["spmm_ms_per_step"] = sum(detail[k]["ms_total"] for k in aggs) / steps
    leg["kernel_ms_per_step"] = {k: v["ms_total"] / steps for k, v in
                                 sorted(detail.items(), key=lambda kv: -kv[1]["ms_total"])}
    leg["kernel_avg_ms"] = {k: v["ms_total"] / max(v["launches"], 1) for k, v in detail.items()}
    # release the workload's device memory before the next leg
    del trainer, runs, parts, pool, model
    gc.collect()
    torch.cuda.empty_cache()
    return leg


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the graph (development only)")
    ap.add_argument("--cpu-sample-scale", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="cfg1 only: skip the cfg2, cfg4 and cfg3 legs")
    ap.add_argument("--cut", choices=["random", "dbh"], default="random",
                    help="vertex cut: the random cut (default, the benchmark configurations) or the degree-aware hash")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path is communication-free per partition; "
              "no collectives are built). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    from paper_2308_03209_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU fallback)"
    torch.cuda.set_device(0)
    wl = inputs.WORKLOADS[args.config]
    if args.scale != 1.0:
        wl = wl.scaled(args.scale)

    # one plain device copy of known size (1 GiB read + 1 GiB written): the reference that the
    # HBM byte counters of a profiler run are scaled by
    cal_src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    torch.cuda.empty_cache()

    leg = run_leg(wl, args.steps, args.warmup, args.cut, args.scale)
    out = {
        "metric": "partition edges/sec per fwd+bwd epoch",
        "value": leg["value"], "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": leg["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
    }
    for k in ("config", "roofline", "loss", "roofline_spmm", "spmm_ms_per_step", "kernel_ms_per_step", "kernel_avg_ms",
              "step_ms_min_median_max", "undirected_edges_per_s", "kept_directed_edges_per_s"):
        if k in leg:
            out[k] = leg[k]
    if args.config == 1 and args.scale == 1.0 and args.cut == "random" and not args.no_also:
        # the configurations whose aggregation is bound by HBM: same code path, fewer steps for the long one
        also = {}
        for index, steps, warmup in ((2, args.steps, args.warmup), (4, max(2, args.steps // 4), max(1, args.warmup // 2)),
                                     (3, max(3, args.steps // 4), 1)):
            log(f"[bench] ---- also: config {index} ----")
            also[f"cfg{index}"] = run_leg(inputs.WORKLOADS[index], steps, warmup, "random", 1.0)
        out["also"] = also
    if not args.no_cpu_baseline:
        sample = args.cpu_sample_scale
        if sample is None:
            sample = {0: 1.0, 1: 1.0, 2: 0.1, 3: 0.002, 4: 0.02, 5: 0.3, 6: 0.1, 7: 0.1}.get(wl.index, 0.05)
            if args.scale != 1.0:
                sample = min(1.0, sample / args.scale)
        log(f"[bench] timing the CPU oracle on a x{sample:g} sample ...")
        out["cpu_baseline"] = cpu_baseline(inputs.WORKLOADS[args.config] if args.scale == 1.0 else wl, sample, args.cut)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
