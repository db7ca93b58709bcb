"""Benchmark of the layer-wise full-graph inference path on one MI355X.

A step is one dgi_infer call: every layer of the model over every node of the graph, in destination
batches chosen by the library (dynamic batch-size control).  The default workload is the largest one a single GPU
holds: the 3-layer GraphSAGE-mean model with bf16 storage on the 111 M-node / 1.6 B-edge synthetic power-law graph
(inputs generated on the GPU from seeds and resident in HBM before the timed region).  Prints one JSON line; the
other full-size workloads (configs 2, 3, 5) are measured in the same process with shorter runs and reported inside it
under "other_configs".

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--scale 1.0] [--no-cpu-baseline] [--no-other-configs]
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


# what "dtype" stands for, spelled out
ARITHMETIC = {
    "bf16": "inputs, weights and hidden layers stored bf16; sums and products accumulated in fp32 (aggregates reach the bf16 "
            "matrix instruction as a bf16 value plus its rounding remainder, 16 significant bits)",
    "f32": "fp32 storage and accumulation; the GEMMs outside the fused kernel run on the bf16 matrix instruction with both "
           "operands split exactly into three bf16 terms and six products per fp32 product (error at the fp32 instruction's level)",
}


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


def cpu_baseline(cfg, target_seconds=20.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: every layer of the model on
    the first R destination rows of the full graph, all host threads.  The oracle is handed the sub-problem those
    rows span (the rows, their in-neighbour lists relabelled, the feature rows they read), so that a 111 M-node
    feature matrix never has to be copied to the host; layer 1 reads the real input rows, later layers N(0,1) rows
    of their width.  R is sized from a short calibration pass so that the sample takes about `target_seconds`.
    Reported as aggregated edges per second."""
    import numpy as np
    import torch
    from dgi_inputs import configs
    from oracle import oracle

    n = cfg["num_nodes"]
    indptr, indices = cfg["indptr"], cfg["indices"]
    layers = configs.to_numpy_layers(cfg["layers"])
    threads = oracle.num_threads()

    def run(count):
        e1 = int(indptr[count])
        src = indices[:e1].to(torch.int64)
        rows = torch.arange(count, device=src.device)
        U = torch.unique(torch.cat([rows, src]))                       # sorted: the first `count` entries are the rows
        ip = torch.full((U.numel() + 1,), e1, dtype=torch.int64)
        ip[:count + 1] = indptr[:count + 1].to(torch.int64).cpu()
        ix = torch.searchsorted(U, src).to(torch.int32).cpu().numpy()
        ip = ip.numpy()
        t = 0.0
        r = np.arange(count, dtype=np.int64)
        for li, L in enumerate(layers):
            d_in = L["W_neigh"].shape[0]
            if li == 0:
                h = cfg["x"][U].float().cpu().numpy()
            else:
                h = np.random.default_rng(777 + li).standard_normal((U.numel(), d_in), dtype=np.float32)
            t0 = time.perf_counter()
            oracle.layer_forward(ip, ix, L, h, rows=r)
            t += time.perf_counter() - t0
        return t, e1

    probe = min(n, 20_000)
    t_probe, _ = run(probe)
    count = int(min(n, max(probe, probe * target_seconds / max(t_probe, 1e-3))))
    count = min(count, 4_000_000)   # bounds the host memory of the sample
    total, edges = run(count)
    agg_edges = edges * len(layers)
    return {"value": agg_edges / total, "unit": "edges/s", "cores": threads, "kind": "oracle",
            "sample": "all %d layers on the first %d destination rows (%d edges per layer) of the full graph, %.1f s"
                      % (len(layers), count, edges, total)}


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
    for method in ("bfs_rcm", "community", "degree"):
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


def partial(args, cfg, g, structs, x, B):
    """Partial inference (Section 3.3; the paper's figure of time against the number of targets): random target sets of
    growing size, the per-layer sets the library annotates, the rows each layer computes, and the time next to that of
    full inference.  Separate line, never the headline value."""
    import torch
    n, e = cfg["num_nodes"], int(cfg["indices"].numel())
    out_dim = structs[-1].out_dim
    full = torch.empty(n, out_dim, dtype=torch.float32, device="cuda")
    B.infer(g, structs, x, full)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        B.infer(g, structs, x, full)
    torch.cuda.synchronize()
    full_ms = (time.perf_counter() - t0) / args.steps * 1e3
    del full
    runs = []
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    for count in [int(c) for c in args.partial.split(",")]:
        count = min(count, n)
        targets = torch.randperm(n, device="cuda", generator=gen)[:count].to(torch.int32)
        out = torch.empty(count, out_dim, dtype=torch.float32, device="cuda")
        st = B.infer_partial(g, structs, x, targets, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            st = B.infer_partial(g, structs, x, targets, out)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        runs.append({"targets": count, "ms": round(ms, 3), "set_size": st["set_size"], "rows_computed": st["rows_computed"],
                     "shortcut_all_nodes_up_to_layer": st["all_nodes_from_layer"], "sub_nodes": st["sub_nodes"], "sub_edges": st["sub_edges"]})
        print("[bench] %s" % json.dumps(runs[-1]), file=sys.stderr, flush=True)
        del out, targets
    print(json.dumps({"metric": "partial inference: milliseconds per call against the number of targets", "unit": "ms", "higher_is_better": False,
                      "n_gpus": 1, "steps": args.steps, "data": "synthetic",
                      "config": {"workload": cfg["name"] + " [partial inference]", "num_nodes": n, "num_edges": e},
                      "full_inference_ms": round(full_ms, 3), "runs": runs}))


def hot_sources(cfg):
    """How much of a gather the popular source rows account for: the share of all edges whose source is among the K
    nodes of largest out-degree, for K rows that fit a workgroup's LDS, one XCD's L2 and the memory-side cache."""
    import torch
    n, e = cfg["num_nodes"], int(cfg["indices"].numel())
    out_deg = torch.zeros(n, dtype=torch.int64, device=cfg["indices"].device)
    step = 1 << 28
    for a in range(0, e, step):   # bincount in pieces: a 1.6 G-edge index array would need 13 GB as int64
        out_deg += torch.bincount(cfg["indices"][a:a + step].long(), minlength=n)
    top = torch.sort(out_deg, descending=True).values
    cum = torch.cumsum(top, 0)
    row_bytes = int(cfg["x"].shape[1]) * cfg["x"].element_size()
    res = {"workload": cfg["name"], "num_nodes": n, "num_edges": e, "input_row_bytes": row_bytes, "max_out_degree": int(top[0]), "top_sources": []}
    for what, cap in (("64 KB of LDS", 64 << 10), ("4 MB L2 of one XCD", 4 << 20), ("256 MB memory-side cache", 256 << 20)):
        for rb in sorted({row_bytes, 256, 1024}):
            k = max(1, min(n, cap // rb))
            res["top_sources"].append({"fits": what, "row_bytes": rb, "rows": k, "edge_share": round(float(cum[k - 1]) / e, 5)})
    print(json.dumps(res))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--batch-size", type=int, default=0, help="destination rows per batch; 0 = dynamic")
    ap.add_argument("--order", choices=["auto", "agg_first", "transform_first", "agg_first_fused", "agg_first_split"], default="auto",
                    help="force every layer's execution order (dgi_layer_t.order); auto = the library's choice")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", dest="other_configs", action="store_false",
                    help="skip the short runs of the other full-size workloads that the headline line carries as context")
    ap.add_argument("--ablation", action="store_true", help="reordering x batch-size ablation instead of the timed run")
    ap.add_argument("--partial", default="", metavar="COUNTS",
                    help="partial inference of random target sets of these sizes, e.g. 100,1000,10000,100000,1000000 (prints its own JSON line)")
    ap.add_argument("--hot-sources", action="store_true",
                    help="print the share of edges whose source is among the top-K out-degree nodes, K sized to LDS / L2 / the memory-side cache")
    ap.add_argument("--fanout", type=int, default=0, help="sampling inference with this fan-out per layer (prints its own JSON line)")
    ap.add_argument("--host-resident", action="store_true",
                    help="embeddings in pinned host memory, batches streamed in (dgi_infer_host); prints its own JSON line")
    ap.add_argument("--reorder", choices=["none", "degree", "bfs_rcm", "community"], default="none",
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
    if args.hot_sources:
        hot_sources(cfg)
        return
    n = cfg["num_nodes"]
    e = int(cfg["indices"].numel())
    g = B.graph_load(cfg["indptr"], cfg["indices"])
    info = g.info()
    storage = "bf16" if cfg["x"].dtype == torch.bfloat16 else "f32"
    structs, keep = [], []
    for i, L in enumerate(cfg["layers"]):
        fs = storage if i == 0 else cfg["layers"][i - 1].get("out_storage", "f32")
        s, k = B.make_layer(dict(L, order=args.order), device=dev, feat_dtype=fs)
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
    if args.partial:
        del out
        partial(args, cfg, g, structs, x, B)
        return
    if args.host_resident:
        del out
        host_resident(args, cfg, g, structs, B)
        return
    first_call_ms, sec, stats = timed_steps(B, g, structs, x, out, args.warmup, args.steps, args.batch_size)
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
    del deg
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
        "first_call_ms": first_call_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if storage == "bf16" else "f32",
        "arithmetic": ARITHMETIC[storage],
        "data": "synthetic",
        "config": {"workload": cfg["name"], "num_nodes": n, "num_edges": e, "max_in_degree": info["max_in_degree"],
                   "in_degree": degree_stats, "hub_rows": info["num_hub_rows"], "hub_edges": info["num_hub_edges"], "scale": args.scale, "batch_size": args.batch_size or "dynamic",
                   "batches_per_layer": stats[-1]["batches"], "transform_first": stats[-1]["transform_first"], "fused": stats[-1]["fused"],
                   "generate_seconds": round(t_gen, 2)},
        "per_layer_ms": per_layer_ms(stats, args.steps),
        "roofline": roofline(cfg, info, stats, args.steps, storage),
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg)
    if args.other_configs:
        # the other full-size workloads, same process, same measurement (shorter runs): context for the headline line
        g.free()
        del g, x, out, cfg, structs, keep
        torch.cuda.empty_cache()
        result["other_configs"] = {}
        for k in (2, 3, 5):
            if k == args.config:
                continue
            result["other_configs"]["cfg%d" % k] = other_config(B, configs, k, dev)
        if args.config != 5:  # the block-model graph once more, renumbered by the library (Section 4.2)
            result["other_configs"]["cfg5_reordered"] = other_config(B, configs, 5, dev, reorder="community")
    print(json.dumps(result))


def timed_steps(B, g, structs, x, out, warmup, steps, batch_size, perm=None):
    """(first call in ms: it allocates the library's arena; seconds per step over `steps` timed calls; their stats)."""
    import torch
    first_call_ms = None
    if warmup >= 1:  # the first of the untimed warm-up calls, timed on its own
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.infer(g, structs, x, out, batch_size=batch_size, perm_new_of_old=perm)
        torch.cuda.synchronize()
        first_call_ms = (time.perf_counter() - t0) * 1e3
    for _ in range(max(warmup - 1, 0)):
        B.infer(g, structs, x, out, batch_size=batch_size, perm_new_of_old=perm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stats = []
    for _ in range(steps):
        stats.append(B.infer(g, structs, x, out, batch_size=batch_size, want_stats=True, perm_new_of_old=perm))
    torch.cuda.synchronize()
    return first_call_ms, (time.perf_counter() - t0) / steps, stats


def per_layer_ms(stats, steps):
    n_layers = len(stats[0]["layer_ms"])
    return {k2: [round(sum(s[k1][l] for s in stats) / steps, 3) for l in range(n_layers)]
            for k1, k2 in (("layer_ms", "layer"), ("agg_ms", "aggregate"), ("gemm_ms", "gemm"), ("hub_ms", "hub_prepass"))}


def roofline(cfg, info, stats, steps, storage):
    """HBM roofline of the dominant kernel: the aggregation (or fused aggregation + transform) launch with the largest
    total time.  achieved = algorithmic bytes of its launches / their HIP-event durations."""
    n, e = cfg["num_nodes"], int(cfg["indices"].numel())
    n_layers = len(cfg["layers"])
    agg_ms = [sum(s["agg_ms"][l] for s in stats) for l in range(n_layers)]
    agg_launches = [sum(s["agg_launches"][l] for s in stats) for l in range(n_layers)]
    # (layers that run the same kernel on the same graph differ by noise only: the last of those within 3 % of the
    # slowest is taken, so that the choice, and the offline traffic figure looked up for it, do not flip between runs)
    dom = max(l for l in range(n_layers) if agg_ms[l] >= 0.97 * max(agg_ms))
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
    achieved = bytes_layer * steps / (agg_ms[dom] * 1e-3) / 1e9  # GB/s over all launches of that kernel
    return {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(cfg["name"], dom + 1),
            "kernel": "%s launch of layer %d (gather width %d, %d-byte elements)"
                      % ("fused aggregate+transform" if fused else "aggregation", dom + 1, width, elem),
            "algorithmic_bytes_per_launch": bytes_layer * steps / max(agg_launches[dom], 1),
            "avg_launch_ms": agg_ms[dom] / max(agg_launches[dom], 1), "launches": agg_launches[dom],
            "launches_per_layer_pass": agg_launches[dom] / steps,
            "note": "achieved = requested bytes (every edge priced at one full source row + its index, every node at its "
                    "indptr entry and output row, nothing reused) / kernel time.  On a power-law graph popular source rows "
                    "are served by the L2s and the 256 MB memory-side cache, so this is a requested-byte rate against the "
                    "HBM peak, not DRAM utilisation; `traffic` is L2-miss traffic (FETCH_SIZE / WRITE_SIZE, measured "
                    "offline with rocprofv3 --pmc, see profiles/), which that cache can serve as well."}


def other_config(B, configs, k, dev, steps=5, warmup=2, reorder=None):
    import torch
    cfg = configs.make_config(k, device=dev)
    torch.cuda.empty_cache()
    g = B.graph_load(cfg["indptr"], cfg["indices"])
    perm, reorder_s = None, 0.0
    if reorder:
        t0 = time.perf_counter()
        g2, perm = B.graph_reorder(g, reorder)
        torch.cuda.synchronize()
        reorder_s = time.perf_counter() - t0
        g.free()
        g = g2
    info = g.info()
    structs, keep = zip(*[B.make_layer(L, device=dev) for L in cfg["layers"]])
    structs = list(structs)
    x = cfg["x"].contiguous()
    out = torch.empty(cfg["num_nodes"], structs[-1].out_dim, dtype=torch.float32, device=dev)
    first_ms, sec, stats = timed_steps(B, g, structs, x, out, warmup, steps, 0, perm)
    e = int(cfg["indices"].numel())
    r = roofline(cfg, info, stats, steps, "f32")
    if reorder:
        r["traffic"] = None   # the offline counter figure belongs to the graph as generated
    res = {"workload": cfg["name"] + (" [ids renumbered by dgi_graph_reorder(%s), %.2f s once per graph; x and the output stay in the caller's order]" % (reorder, reorder_s) if reorder else ""),
           "num_nodes": cfg["num_nodes"], "num_edges": e, "steps": steps, "warmup": warmup, "dtype": "f32", "arithmetic": ARITHMETIC["f32"],
           "ms_per_step": sec * 1e3, "first_call_ms": first_ms, "edges_per_s": len(structs) * e / sec,
           "per_layer_ms": per_layer_ms(stats, steps),
           "dominant_kernel": {k2: r[k2] for k2 in ("kernel", "achieved", "frac", "avg_launch_ms", "traffic")}}
    g.free()
    del g, x, out, cfg
    torch.cuda.empty_cache()
    return res


if __name__ == "__main__":
    main()
