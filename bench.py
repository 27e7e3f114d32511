#!/usr/bin/env python3
"""Throughput of one full-batch training iteration (forward, reweighted loss, backward, update)
on one vertex-cut partition, on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--scale 1.0]

Prints ONE JSON line: partition edges per second per iteration (edges = directed adjacency
entries of the unmasked partition), the roofline of the kernel that dominates the iteration
(timed live with HIP events on the launching stream) and the CPU oracle timed on a bounded
sample of the same workload.  Inputs are synthetic (seeded power-law graph shaped like the
paper's dataset, N(0,1) features, uniform labels, Glorot weights) and resident in HBM before
the timed region.
"""
from __future__ import annotations

import argparse
import re
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F32_TFLOPS = 157.3
PEAK_MFMA_BF16_TFLOPS = 2500.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(wl, sample_scale: float, cut: str = "random"):
    """Time the oracle (as it stands) on one iteration over partition 0 of a down-scaled copy of
    the workload with the same average degree and model widths."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import dropedge as o_dropedge
    from oracle import epoch as o_epoch
    from oracle import partition as o_partition
    from paper_2308_03209_amd import inputs

    ws = wl.scaled(sample_scale)
    src, dst = inputs.workload_graph(ws)
    O = o_partition.build_partition(ws.n_nodes, src, dst, ws.n_parts, 0, inputs.SEED_CUT, method=cut)
    ids = O["local2global"]
    dims = ws.layer_dims()
    X = inputs.node_features(ids, ws.d_feat)
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
    return {"value": O["nnz"] / dt, "unit": "edges/s", "cores": threads, "kind": "oracle",
            "sample": f"one iteration on partition 0 of the workload scaled x{sample_scale:g} in nodes and edges "
                      f"({O['n_nodes']} nodes, {O['nnz']} directed edges, same widths), {dt:.1f} s; numpy fp64, "
                      f"BLAS threads for the dense products, one thread for the per-row aggregation loops"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the graph (development only)")
    ap.add_argument("--cpu-sample-scale", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cut", choices=["random", "dbh"], default="random",
                    help="vertex cut: the random cut (default, the benchmark configurations) or the degree-aware hash")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path is communication-free per partition; "
              "no collectives are built). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2308_03209_amd import binding as B
    from paper_2308_03209_amd import inputs
    from paper_2308_03209_amd import model as M
    from paper_2308_03209_amd import train as T

    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU fallback)"
    torch.cuda.set_device(0)
    wl = inputs.WORKLOADS[args.config]
    if wl.index == 3 and args.scale > 0.5:
        print("bench.py: config 3's 1.6-billion-edge graph needs a streamed generator that is not built; "
              "run it with --scale <= 0.5 (the in-memory generator takes minutes there)", file=sys.stderr)
        return 2
    if args.scale != 1.0:
        wl = wl.scaled(args.scale)
    log(f"[bench] workload {wl.name}: seeds graph={inputs.SEED_GRAPH + wl.index} perm={inputs.SEED_PERM + wl.index} "
        f"cut={inputs.SEED_CUT} masks={inputs.SEED_MASKS} features={inputs.SEED_FEATURES} labels={inputs.SEED_LABELS} "
        f"params={inputs.SEED_PARAMS}")
    t0 = time.time()
    src, dst = inputs.workload_graph(wl, progress=lambda text: log(f"[bench] graph: {text} ({time.time() - t0:.0f} s)"))
    log(f"[bench] graph: {wl.n_nodes} nodes, {len(src)} undirected edges ({time.time() - t0:.1f} s)")
    dims = wl.layer_dims()
    model = M.Model(wl.kind, dims)
    model.load(inputs.model_params(wl.kind, dims))
    runs = []
    nnz_total = 0
    parts = []
    for part_id in wl.train_parts:
        t0 = time.time()
        P = B.build_partition(wl.n_nodes, src, dst, wl.n_parts, part_id, inputs.SEED_CUT,
                              flags=B.CUT_DBH if args.cut == "dbh" else 0)
        masks = None
        if wl.dropedge_K:
            t1 = time.time()
            masks = B.dropedge_k(P, wl.dropedge_K, wl.dropedge_p, inputs.SEED_MASKS + part_id)   # synchronises
            log(f"[bench] partition {part_id}: {wl.dropedge_K} DropEdge masks drawn and compacted on the device in "
                f"{1e3 * (time.time() - t1):.1f} ms")
        parts.append((part_id, P, masks, time.time() - t0))
    # partitions are trained one after the other, so their activation buffers are shared
    pool = M.BufferPool(max(P.num_nodes for _, P, _, _ in parts)) if len(parts) > 1 else None
    tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    for part_id, P, masks, t_build in parts:
        t0 = time.time() - t_build
        ids = P.host_array(B.ARR_LOCAL2GLOBAL)
        X = torch.from_numpy(inputs.node_features(ids, wl.d_feat)).to(tdtype).cuda()
        if wl.loss == "sigmoid_bce":
            y = torch.from_numpy(inputs.node_multilabels(ids, wl.n_classes)).cuda()
        else:
            y = torch.from_numpy(inputs.node_labels(ids, wl.n_classes)).cuda()
        run = M.PartitionRunner(P, model, masks, dropout_q=wl.dropout, dropout_seed=inputs.SEED_DROPOUT,
                                dtype=wl.dtype, pool=pool, loss=wl.loss)
        runs.append((run, X, y, part_id))
        nnz_total += P.num_nnz
        log(f"[bench] partition {part_id}: {P.num_nodes} nodes, {P.num_nnz} directed edges "
            f"({time.time() - t0:.1f} s to build and upload)")
    del src, dst
    c = 1.0 / wl.n_nodes

    trainer = T.Trainer(model, [T.PartitionData(run, X, y, inputs.SEED_MASKS + part_id) for run, X, y, part_id in runs],
                        c, wl.optimizer, wl.lr)

    def step(epoch: int) -> None:
        assert trainer.iteration == epoch
        trainer.step()

    # one plain device copy of known size (1 GiB read + 1 GiB written): the reference that the
    # HBM byte counters of a profiler run are scaled by
    cal_src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    for e in range(args.warmup):
        step(e)
    torch.cuda.synchronize()
    B.profile_enable(True)
    t0 = time.perf_counter()
    for e in range(args.steps):
        step(args.warmup + e)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    detail = B.profile_read()
    B.profile_enable(False)
    # per-shape records -> kernel families: the kernel's name without template arguments and shape
    # (all instances of the dense-transform kernel are one family)
    stats = {}
    for name, rec in detail.items():
        fam = stats.setdefault(re.sub(r"<.*?>", "", name.split(" ")[0]),
                               dict(launches=0, ms_total=0.0, alg_bytes=0.0, alg_flops=0.0))
        for k in fam:
            fam[k] += rec[k]
    ms_per_step = 1e3 * dt / args.steps
    value = nnz_total / (dt / args.steps)
    loss = float(runs[-1][0].loss.item())
    assert np.isfinite(loss), "loss is not finite"

    kernel_ms = sum(s["ms_total"] for s in stats.values())
    for name, s in sorted(detail.items(), key=lambda kv: -kv[1]["ms_total"]):
        n = max(s["launches"], 1)
        log(f"[shape] {name:40s} launches/step {s['launches'] / args.steps:5.1f}  avg ms {s['ms_total'] / n:8.4f}"
            f"  alg GB/s {s['alg_bytes'] / max(s['ms_total'], 1e-9) / 1e6:8.1f}"
            f"  alg TFLOP/s {s['alg_flops'] / max(s['ms_total'], 1e-9) / 1e9:7.2f}")
    for name, s in sorted(stats.items(), key=lambda kv: -kv[1]["ms_total"]):
        n = max(s["launches"], 1)
        log(f"[bench] {name:24s} launches/step {s['launches'] / args.steps:6.1f}  ms/step {s['ms_total'] / args.steps:8.3f}"
            f"  avg ms {s['ms_total'] / n:8.4f}  alg GB/s {s['alg_bytes'] / max(s['ms_total'], 1e-9) / 1e6:9.1f}"
            f"  alg TFLOP/s {s['alg_flops'] / max(s['ms_total'], 1e-9) / 1e9:8.2f}")
    log(f"[bench] kernels {kernel_ms / args.steps:.3f} ms/step of {ms_per_step:.3f} ms/step wall")

    # HBM-side bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this same
    # command (scaled by a plain copy's reading); committed with the profile summary
    traffic = {}
    tpath = os.path.join(ROOT, "profiles", f"cfg{wl.index}_traffic.json")
    if args.scale == 1.0 and os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("bytes_per_launch", {})

    def roofline(name: str):
        s = stats[name]
        if name.startswith("gemm_"):
            a = s["alg_flops"] / (s["ms_total"] * 1e-3) / 1e12
            peak = PEAK_MFMA_BF16_TFLOPS if "bf16" in name else PEAK_MFMA_F32_TFLOPS
            return {"kernel": name, "bound": "mfma", "achieved": a, "peak": peak, "unit": "TFLOP/s",
                    "frac": a / peak, "traffic": traffic.get(name), "launches": s["launches"],
                    "avg_ms": s["ms_total"] / max(s["launches"], 1)}
        a = s["alg_bytes"] / (s["ms_total"] * 1e-3) / 1e9
        out_r = {"kernel": name, "bound": "hbm", "achieved": a, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                 "frac": a / PEAK_HBM_GBS, "traffic": traffic.get(name), "launches": s["launches"],
                 "avg_ms": s["ms_total"] / max(s["launches"], 1)}
        if out_r["traffic"]:
            # counter-measured bytes over the live duration: how busy the memory system really is
            out_r["measured_traffic_GBps"] = out_r["traffic"] / (out_r["avg_ms"] * 1e-3) / 1e9
        if name == "aggregate_kernel" and s["alg_flops"] > 0:
            # bytes the gather requests when no neighbour row is reused: nnz * width * element size
            # (the kernel's flop count is 2 * nnz * width)
            es = 2 if wl.dtype == "bf16" else 4
            out_r["gathered_GBps"] = s["alg_flops"] / 2 * es / (s["ms_total"] * 1e-3) / 1e9
        return out_r

    dominant = max(stats, key=lambda k: stats[k]["ms_total"])
    out = {
        "metric": "partition edges/sec per fwd+bwd epoch",
        "value": value, "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "kind": wl.kind, "layers": wl.n_layers, "n_nodes": wl.n_nodes,
                   "partition_nodes": [r[0].n for r in runs], "partition_directed_edges": nnz_total,
                   "n_parts": wl.n_parts, "trained_parts": list(wl.train_parts), "d_feat": wl.d_feat,
                   "hidden": wl.hidden, "n_classes": wl.n_classes, "dropedge_K": wl.dropedge_K,
                   "reweighting": "DAR", "optimizer": wl.optimizer, "dropout": wl.dropout, "loss": wl.loss, "cut": args.cut},
        "roofline": roofline(dominant),
        "loss": loss,
    }
    if "aggregate_kernel" in stats and dominant != "aggregate_kernel":
        out["roofline_spmm"] = roofline("aggregate_kernel")
    out["kernel_ms_per_step"] = {k: v["ms_total"] / args.steps for k, v in stats.items()}
    if not args.no_cpu_baseline:
        sample = args.cpu_sample_scale
        if sample is None:
            sample = {0: 1.0, 1: 0.8, 2: 0.1, 3: 0.002, 4: 0.02, 5: 0.3, 6: 0.1, 7: 0.1}.get(wl.index, 0.05) * (1.0 if args.scale == 1.0 else 1.0)
            sample = min(1.0, sample / args.scale) if args.scale != 1.0 else sample
        log(f"[bench] timing the CPU oracle on a x{sample:g} sample ...")
        out["cpu_baseline"] = cpu_baseline(inputs.WORKLOADS[args.config] if args.scale == 1.0 else wl, sample, args.cut)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
