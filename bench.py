"""Benchmark of the layer-wise full-graph inference path on one MI355X.

A step is one dgi_infer call: every layer of the model over every node of the graph, in destination
batches chosen by the library (dynamic batch-size control).  The default workload is the 3-layer GCN on
the 2.4 M-node / 126 M-edge synthetic power-law graph (inputs generated on the GPU from seeds and
resident in HBM before the timed region).  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--scale 1.0] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def algorithmic_bytes(n, e, width, elem, indptr_bytes, heads=0, out_width=None, out_elem=None, self_width=0):
    """Bytes the aggregation of one layer must move when nothing is reused: per edge one source row and
    its index (plus the GAT score terms), per destination node its indptr entry and its output row (for
    the fused kernel the output row is the layer output, plus the node's own input row for GraphSAGE)."""
    per_edge = width * elem + 4 + 4 * heads
    per_node = indptr_bytes + (width * elem if out_width is None else out_width * out_elem) + self_width * elem
    return e * per_edge + n * per_node


def measured_traffic(workload, layer):
    """HBM bytes per launch of the dominant kernel as measured offline with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE, each scaled by a plain copy of known size).  The figure lives in a text summary under
    profiles/ as a line `TRAFFIC_BYTES_PER_LAUNCH | <workload> | layer <k> | <bytes>`; None if absent."""
    path = os.path.join(ROOT, "profiles")
    if not os.path.isdir(path):
        return None
    for name in sorted(os.listdir(path)):
        if not name.endswith(".txt"):
            continue
        for line in open(os.path.join(path, name)):
            f = [x.strip() for x in line.split("|")]
            if len(f) == 4 and f[0] == "TRAFFIC_BYTES_PER_LAUNCH" and f[1] == workload and f[2] == "layer %d" % layer:
                return float(f[3])
    return None


def cpu_baseline(cfg, target_seconds=30.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: every layer of the model on
    the first R destination rows of the full graph (synthetic N(0,1) inputs of each layer's width stand in
    for the hidden layers), all host threads.  R is sized from a short calibration pass so that the sample
    takes about `target_seconds`.  Reported as aggregated edges per second."""
    import numpy as np
    import torch
    from dgi_inputs import configs, generators
    from oracle import oracle

    n = cfg["num_nodes"]
    ip = cfg["indptr"].cpu().numpy().astype(np.int64)
    ix = cfg["indices"].cpu().numpy()
    layers = configs.to_numpy_layers(cfg["layers"])
    threads = oracle.num_threads()
    inputs = []
    for li, L in enumerate(layers):
        d_in = L["W_neigh"].shape[0]
        inputs.append(cfg["x"].float().cpu().numpy() if li == 0 else generators.normal_features(n, d_in, 777 + li).numpy())

    def run(count):
        rows = np.arange(count, dtype=np.int64)
        t = 0.0
        for L, h in zip(layers, inputs):
            t0 = time.perf_counter()
            oracle.layer_forward(ip, ix, L, h, rows=rows)
            t += time.perf_counter() - t0
        return t, int(ip[count] - ip[0])

    probe = min(n, 20_000)
    t_probe, _ = run(probe)
    count = int(min(n, max(probe, probe * target_seconds / max(t_probe, 1e-3))))
    total, edges = run(count)
    agg_edges = edges * len(layers)
    rows = np.arange(count)
    return {"value": agg_edges / total, "unit": "edges/s", "cores": threads, "kind": "oracle",
            "sample": "all %d layers on the first %d destination rows (%d edges per layer) of the full graph, %.1f s"
                      % (len(layers), rows.size, edges, total)}


def input_set_total(indptr, indices, batch):
    """Sum over consecutive-id batches of the number of distinct source rows the batch reads (the quantity
    node reordering is meant to shrink); torch tensors on the GPU."""
    import torch
    n = indptr.numel() - 1
    total = 0
    for b in range(0, n, batch):
        e = min(n, b + batch)
        total += int(torch.unique(indices[int(indptr[b]):int(indptr[e])]).numel())
    return total


def ablation(args, cfg, g, structs, x, out, B):
    """Reordering / batching ablation: shuffled ids vs the library's reorderings, at fixed and dynamic
    destination-batch sizes.  Reordering time is reported separately (once per graph)."""
    import torch
    n = cfg["num_nodes"]
    variants = [("shuffled ids", g, None, 0.0)]
    for method in ("bfs_rcm", "degree"):
        t0 = time.perf_counter()
        g2, perm = B.graph_reorder(g, method)
        torch.cuda.synchronize()
        variants.append((method, g2, perm, time.perf_counter() - t0))
        print("[bench] reorder %s: %.1f s" % (method, variants[-1][3]), file=sys.stderr, flush=True)
    runs = []
    for name, gv, perm, t_reorder in variants:
        ip, ix = gv.csr()
        ip_d, ix_d = torch.from_numpy(ip).cuda(), torch.from_numpy(ix).cuda()
        inputs = {bs: input_set_total(ip_d, ix_d, bs) for bs in (1 << 16, 1 << 20)}
        del ip_d, ix_d
        for bs in (1 << 16, 1 << 20, 0):
            B.infer(gv, structs, x, out, batch_size=bs, perm_new_of_old=perm)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            st = None
            for _ in range(args.steps):
                st = B.infer(gv, structs, x, out, batch_size=bs, perm_new_of_old=perm, want_stats=True)
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t0) / args.steps
            runs.append({"ids": name, "batch_size": bs or "dynamic", "ms": round(sec * 1e3, 3),
                         "agg_ms": [round(v, 3) for v in st["agg_ms"]], "gemm_ms": [round(v, 3) for v in st["gemm_ms"]],
                         "batches": st["batches"], "distinct_inputs_over_batches": inputs.get(bs),
                         "reorder_seconds": round(t_reorder, 2)})
            print("[bench] %s" % json.dumps(runs[-1]), file=sys.stderr, flush=True)
        gv.release_workspace()
    print(json.dumps({"ablation": cfg["name"], "num_nodes": n, "num_edges": int(cfg["indices"].numel()), "steps": args.steps,
                      "note": "ms includes permuting X in and the output back for the reordered variants", "runs": runs}))


def host_resident(args, cfg, g, structs, B):
    """The paper's own regime (Algorithm 2 with the embeddings outside the GPU): x, the hidden layers and the
    output live in pinned host memory; every batch reads its input set over the host link.  The rate printed
    here includes those transfers; it is a separate line, never the headline value."""
    import torch
    n, e = cfg["num_nodes"], int(cfg["indices"].numel())
    x = B.pinned_empty(tuple(cfg["x"].shape), cfg["x"].dtype)   # exactly sized (torch's pinned allocator rounds up to 2^k)
    reorder_seconds = 0.0
    if args.reorder != "none":
        # Section 4.2: renumber the nodes once so that batches of consecutive ids share inputs; x goes in in the new
        # numbering (new row perm[v] = old row v) and the output comes out in it (a caller would index it through perm)
        t0 = time.perf_counter()
        g, perm = B.graph_reorder(g, args.reorder, seed=0)
        torch.cuda.synchronize()
        reorder_seconds = time.perf_counter() - t0
        xp = torch.empty_like(cfg["x"])
        xp[perm.long()] = cfg["x"]
        x.copy_(xp)
        del xp
    else:
        x.copy_(cfg["x"])
    out = B.pinned_empty((n, structs[-1].out_dim), torch.float32)
    budget = int(args.device_budget_gb * 1e9)
    kw = dict(batch_size=args.batch_size, mem_budget_bytes=budget, stream_always=not args.allow_device_resident)
    for _ in range(max(args.warmup, 1)):
        B.infer_host(g, structs, x, out, **kw)
    t0 = time.perf_counter()
    stats = [B.infer_host(g, structs, x, out, **kw) for _ in range(args.steps)]
    sec = (time.perf_counter() - t0) / args.steps
    st = stats[-1]
    moved = sum(st["input_bytes"]) + sum(st["output_bytes"]) + sum(st["transform_bytes"])
    print(json.dumps({
        "metric": "full-graph layer-wise inference: aggregated edges per second", "value": len(structs) * e / sec, "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": max(args.warmup, 1), "ms_per_step": sec * 1e3, "higher_is_better": True,
        "data": "synthetic", "config": {"workload": cfg["name"] + " [embeddings in pinned host memory]", "num_nodes": n, "num_edges": e,
                                        "device_budget_bytes": st["budget_bytes"], "batch_size": args.batch_size or "dynamic",
                                        "node_ids": args.reorder, "reorder_seconds": round(reorder_seconds, 3)},
        "host_link": {"bytes_per_step": moved, "GBps_over_whole_step": moved / sec / 1e9,
                      "GBps_while_loading": sum(st["input_bytes"]) / max(sum(st["load_ms"]) * 1e-3, 1e-9) / 1e9},
        "per_layer": {k: [round(v, 3) if isinstance(v, float) else v for v in st[k]]
                      for k in ("load_ms", "compute_ms", "store_ms", "batches", "input_rows", "input_bytes", "output_bytes", "transform_bytes")},
        "oom_retries": st["oom_retries"], "peak_batch_bytes": st["peak_batch_bytes"], "device_resident": st["device_resident"],
        "slots": st["slots"]}))


def sampling(args, cfg, g, structs, x, out, B):
    """Sampling inference (Section 2; the paper's experiments use fan-out 10): every layer draws its sample on the
    device and runs the ordinary schedule on the sampled graph.  Separate line, never the headline value."""
    import torch
    n, e = cfg["num_nodes"], int(cfg["indices"].numel())
    for _ in range(max(args.warmup, 1)):
        B.infer_sampled(g, structs, x, out, args.fanout, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        B.infer_sampled(g, structs, x, out, args.fanout, 2 + i)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    t0 = time.perf_counter()
    gs = B.graph_sample(g, args.fanout, 1, 0)
    torch.cuda.synchronize()
    t_sample = time.perf_counter() - t0
    kept = gs.info()["num_edges"]
    gs.free()
    print(json.dumps({"metric": "sampling inference: seconds per full-graph pass", "value": sec, "unit": "s", "higher_is_better": False,
                      "n_gpus": 1, "steps": args.steps, "warmup": max(args.warmup, 1), "data": "synthetic",
                      "config": {"workload": cfg["name"] + " [fan-out %d]" % args.fanout, "num_nodes": n, "num_edges": e,
                                 "sampled_edges_per_layer": kept},
                      "sample_one_layer_ms": t_sample * 1e3, "sampled_edges_per_second": len(structs) * kept / sec}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--batch-size", type=int, default=0, help="destination rows per batch; 0 = dynamic")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ablation", action="store_true", help="reordering x batch-size ablation instead of the timed run")
    ap.add_argument("--fanout", type=int, default=0, help="sampling inference with this fan-out per layer (prints its own JSON line)")
    ap.add_argument("--host-resident", action="store_true",
                    help="embeddings in pinned host memory, batches streamed in (dgi_infer_host); prints its own JSON line")
    ap.add_argument("--reorder", choices=["none", "degree", "bfs_rcm"], default="none",
                    help="--host-resident: renumber the nodes with the library's reordering first (Section 4.2)")
    ap.add_argument("--allow-device-resident", action="store_true",
                    help="--host-resident: let the library keep the hidden layers on the device when everything fits the budget")
    ap.add_argument("--device-budget-gb", type=float, default=0.0, help="device memory for a batch in --host-resident mode (0 = 90 %% of free)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (known traffic, for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from dgi_inputs import configs
    from paper_2211_15082_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = "cuda"
    t_gen = time.perf_counter()
    cfg = configs.make_config(args.config, scale=args.scale, device=dev, verbose=True)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    torch.cuda.empty_cache()  # hand the generator's scratch back so the library sees the free memory
    n = cfg["num_nodes"]
    e = int(cfg["indices"].numel())
    g = B.graph_load(cfg["indptr"], cfg["indices"])
    info = g.info()
    storage = "bf16" if cfg["x"].dtype == torch.bfloat16 else "f32"
    structs, keep = [], []
    for i, L in enumerate(cfg["layers"]):
        fs = storage if i == 0 else cfg["layers"][i - 1].get("out_storage", "f32")
        s, k = B.make_layer(L, device=dev, feat_dtype=fs)
        structs.append(s)
        keep.append(k)
    x = cfg["x"].contiguous()
    out = torch.empty(n, structs[-1].out_dim, dtype=torch.float32, device=dev)

    if args.ablation:
        ablation(args, cfg, g, structs, x, out, B)
        return
    if args.fanout > 0:
        sampling(args, cfg, g, structs, x, out, B)
        return
    if args.host_resident:
        del out
        host_resident(args, cfg, g, structs, B)
        return
    for _ in range(args.warmup):
        B.infer(g, structs, x, out, batch_size=args.batch_size)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stats = []
    for _ in range(args.steps):
        stats.append(B.infer(g, structs, x, out, batch_size=args.batch_size, want_stats=True))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec = (t1 - t0) / args.steps
    if args.calibration_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    n_layers = len(structs)
    agg_edges = n_layers * e
    step_ms = sorted(s_["total_ms"] for s_ in stats)  # per-call HIP-event time, first enqueue to last completion
    deg = torch.diff(cfg["indptr"].to(torch.int64)).double()
    q = torch.quantile(deg[torch.randperm(n, device=dev)[:min(n, 4_000_000)]], torch.tensor([0.5, 0.9, 0.99, 0.999], dtype=torch.float64, device=dev))
    degree_stats = {"mean": round(float(deg.mean()), 2), "max": int(deg.max()), "zero_rows": int((deg == 0).sum()),
                    "p50": int(q[0]), "p90": int(q[1]), "p99": int(q[2]), "p99.9": int(q[3])}

    # dominant kernel: the aggregation launch with the largest total time
    agg_ms = [sum(s["agg_ms"][l] for s in stats) for l in range(n_layers)]
    agg_launches = [sum(s["agg_launches"][l] for s in stats) for l in range(n_layers)]
    gemm_ms = [sum(s["gemm_ms"][l] for s in stats) / args.steps for l in range(n_layers)]
    dom = max(range(n_layers), key=lambda l: agg_ms[l])
    width = stats[0]["gather_width"][dom]
    L = cfg["layers"][dom]
    is_gat = L["agg"] == "gat"
    elem = 2 if (storage == "bf16" and (dom == 0 or cfg["layers"][dom - 1].get("out_storage") == "bf16")) else 4
    ipb = 8 if info["indptr_type"] == 1 else 4
    fused = bool(stats[0]["fused"][dom])
    if fused:
        # the fused kernel gathers the edges of the non-hub rows; hub rows arrive pre-aggregated (fp32) from the
        # hub pre-pass, whose time is reported separately
        out_elem = 2 if L.get("out_storage") == "bf16" else 4
        bytes_layer = algorithmic_bytes(n, e - info["num_hub_edges"], width, elem, ipb, out_width=int(L["W_neigh"].shape[1]),
                                        out_elem=out_elem, self_width=width if L.get("W_self") is not None else 0)
        bytes_layer += info["num_hub_rows"] * width * 4
    else:
        bytes_layer = algorithmic_bytes(n, e, width, elem, ipb, heads=L.get("heads", 1) if is_gat else 0)
    avg_launch_ms = agg_ms[dom] / max(agg_launches[dom], 1)
    achieved = bytes_layer * args.steps / (agg_ms[dom] * 1e-3) / 1e9  # GB/s over all launches of that kernel
    result = {
        "metric": "full-graph layer-wise inference: aggregated edges per second",
        "value": agg_edges / sec,
        "unit": "edges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": sec * 1e3,
        "inference_seconds": sec,
        "ms_per_step_median": step_ms[len(step_ms) // 2], "ms_per_step_min": step_ms[0],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if storage == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": cfg["name"], "num_nodes": n, "num_edges": e, "max_in_degree": info["max_in_degree"],
                   "in_degree": degree_stats, "hub_rows": info["num_hub_rows"], "hub_edges": info["num_hub_edges"], "scale": args.scale, "batch_size": args.batch_size or "dynamic",
                   "batches_per_layer": stats[-1]["batches"], "transform_first": stats[-1]["transform_first"], "fused": stats[-1]["fused"],
                   "generate_seconds": round(t_gen, 2)},
        "per_layer_ms": {"layer": [round(sum(s["layer_ms"][l] for s in stats) / args.steps, 3) for l in range(n_layers)],
                         "aggregate": [round(a / args.steps, 3) for a in agg_ms], "gemm": [round(v, 3) for v in gemm_ms],
                         "hub_prepass": [round(sum(s["hub_ms"][l] for s in stats) / args.steps, 3) for l in range(n_layers)]},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(cfg["name"], dom + 1),
                     "kernel": "%s launch of layer %d (gather width %d, %d-byte elements)"
                               % ("fused aggregate+transform" if fused else "aggregation", dom + 1, width, elem),
                     "algorithmic_bytes_per_launch": bytes_layer * args.steps / max(agg_launches[dom], 1),
                     "avg_launch_ms": avg_launch_ms, "launches": agg_launches[dom],
                     "launches_per_layer_pass": agg_launches[dom] / args.steps},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
