#!/usr/bin/env python3
"""Benchmark of the masked full-neighbourhood GNN hot path on ONE MI355X.

A step is one pass of the whole hot path over one synthetic partition: active-set construction
(frontier expansion), then per layer masked aggregation + feature transform, the loss, and the
matching backward pass.  Inputs are resident in HBM before the timed region.  One JSON line on
stdout:
  value     aggregated edges per second = (edges visited by all forward and backward aggregations
            of a step, counted for the paper's order of a layer's halves) / (wall time of a step)
  roofline  the dominant kernel (the forward aggregation that gathers the most bytes): algorithmic bytes
            per launch over the launch's duration from HIP events recorded on the launch stream in the timed steps
  call_ms   every C-ABI call between two events on the stream it is enqueued on; the weight-gradient
            products run on a second stream beside the backward aggregations, so the sum of the entries
            exceeds the step (ms_per_step is the wall time)
  cpu_baseline  the CPU oracle timed on this machine's host cores on a bounded sample (reported for
            context; it is not the target)

python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1] [--scale s]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}

CONFIG_INDEX = {"cfg0": 0, "cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4}

# Traffic between L2 and the memory fabric of the dominant call per launch, from the two rocprofv3 --pmc runs
# summarised in profiles/spmm_blocked_fwd_cfg1.md and profiles/spmm_rows_and_gemm_cfg4.md (FETCH_SIZE and WRITE_SIZE in
# KiB, summed over the call's kernels, scaled by what the same counters read for a 1 GiB copy: 2.0 and 1.0).  Known
# for configs[1] (layer 2; layer 1 in the paper's order, --aggregate-first) and configs[4] at full scale.
MEASURED_TRAFFIC_KIB = {"cfg1": {2: {"fetch": 230305 + 15972532 + 935683,       # seg + stream + sum_parts kernels
                                     "write": 8191 + 1864000 + 233000},
                                 1: {"fetch": 231169 + 40302620 + 2297897, "write": 8192 + 4427085 + 562475}},
                        "cfg4": {2: {"fetch": 7994957, "write": 1742670}}}       # one spmm_rows_kernel launch
FETCH_SCALE, WRITE_SCALE = 2.0, 1.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_partition(name, scale):
    """The seeded synthetic partition of the named workload (cfg4: sampled on the GPU first)."""
    import graphgen as gg
    t0 = time.time()
    w = gg.make_workload(name, scale=scale)
    log(f"[bench] generated {name} (scale {scale}) in {time.time() - t0:.1f}s: global n={w.global_graph.n_rows} "
        f"nnz={w.global_graph.nnz}")
    return w


def sampled_partition_cfg4(w):
    """configs[4], steps a0 and a-1 on the GPU: boundary sampling, then extraction of the local one-hop graph with
    (distance, id) numbering.  Returns a host-side Partition (for the CPU baseline), the device graph and the two times."""
    import torch
    import graphgen as gg
    import paper_2311_06837_amd as P
    g, T = w.global_graph, w.targets_global.astype(np.int32)          # targets ascending
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Td = torch.from_numpy(T).cuda()
    ws = P.Workspace()
    bits = P.gnn_make_bitmap(Td, g.n_rows)
    for _ in range(2):                                                 # first pass warms the allocator, second is timed
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rp, ci = P.gnn_sample_boundary(G, bits, Td, w.fanout, w.sample_seed, ws=ws)
        torch.cuda.synchronize()
        t_sample = time.perf_counter() - t0
        local, l2g, hop = P.gnn_extract_sampled_partition(G, Td, rp, ci, ws=ws)     # symmetric graph: gT = g
        torch.cuda.synchronize()
        t_extract = time.perf_counter() - t0 - t_sample
    kept = int(ci.numel())
    l2g_h = l2g.cpu().numpy().astype(np.int64)
    lg = gg.CSR(local.n_rows, local.n_rows, local.row_ptr.cpu().numpy(), local.col_idx.cpu().numpy())
    part = gg.Partition(lg, lg, l2g_h, np.arange(T.size, dtype=np.int32), g.degrees()[l2g_h].astype(np.int32))
    return part, local, t_sample, t_extract, kept


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg1", choices=sorted(CONFIG_INDEX))
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the vertex count (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--host-partition", action="store_true",
                    help="run the step on the host-built partition (ascending-id numbering, every call gets a row list) "
                         "instead of the one built on the GPU from the unpartitioned graph (active sets, extraction with "
                         "(distance, id) numbering, feature gather: every R_l is an id prefix); full-halo workloads only")
    ap.add_argument("--extract-on-gpu", action="store_true", help="the default; kept for old command lines")
    ap.add_argument("--aggregate-first", action="store_true",
                    help="keep the paper's order (aggregate, then weights) in every layer; by default a GraphSAGE layer that "
                         "narrows its input multiplies by the weights first and gathers the narrower rows")
    ap.add_argument("--weights-first-all", action="store_true",
                    help="every narrowing layer in the exchanged order, also those whose input rows are shorter than 512 bytes")
    ap.add_argument("--one-stream", action="store_true",
                    help="enqueue the weight-gradient products on the step's stream instead of a second one")
    ap.add_argument("--layer-sampling", default=None, metavar="RULE:PARAM[:SEED]",
                    help="layer-wise sampling as per-layer edge masks, rebuilt every step: fanout:F (neighbours kept per "
                         "row and layer) or dropedge:P (every edge kept with probability P per layer); off by default")
    ap.add_argument("--res-layers", type=int, default=0, metavar="L",
                    help="run the deep residual GraphSAGE (ResSAGE+) with L layers of the workload's hidden width on the "
                         "workload's graph instead of its own model (GraphSAGE workloads); --recompute: activation recomputation")
    ap.add_argument("--recompute", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    args.extract_on_gpu = not args.host_partition
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding or collectives are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import graphgen as gg
    import paper_2311_06837_amd as P

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = build_partition(args.workload, args.scale)
    t_sample, kept, t_extract, sampled_graph = None, None, None, None
    if w.partition is None:
        part, sampled_graph, t_sample, t_extract, kept = sampled_partition_cfg4(w)
        log(f"[bench] GPU sampling {t_sample * 1e3:.2f} ms, GPU extraction of the sampled partition {t_extract * 1e3:.2f} ms")
    else:
        part = w.partition
    dtype = torch.float32 if w.dtype == "f32" else torch.bfloat16
    sage = w.model == "sage"
    n = part.graph.n_rows
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    params = gg.layer_weights(w.dims, sage, w.seed)
    dparams = [{k: dev(v) for k, v in p.items()} for p in params]
    ld0 = P.row_stride(w.dims[0], dtype)
    H0 = gg.features(n, w.dims[0], w.seed, ld=ld0)
    n_layers = len(w.dims) - 1

    if args.res_layers:
        return bench_res_model(args, w, part, sampled_graph, dtype)

    # Step (a-1) of the path, outside the timed step like the sampling: the partition's one-hop graph extracted on
    # the GPU from the unpartitioned graph, vertices renumbered by (distance, id).  Timed always (full-halo
    # workloads); used for the run with --extract-on-gpu.
    gpu_part = None
    if w.partition is not None:
        Gg = P.Graph.from_numpy(w.global_graph.row_ptr, w.global_graph.col_idx)
        Tg = dev(w.targets_global.astype(np.int32))
        ews = P.Workspace()
        for rep_i in range(2):       # first pass warms the allocator, second is timed
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            gdist, gring, _, ghop = P.gnn_build_active_sets(Gg, Tg, n_layers, ws=ews)
            local, new_id = P.gnn_extract_partition(Gg, gring, int(ghop[-1]), gdist, n_layers, ws=ews)
            torch.cuda.synchronize()
            t_extract = time.perf_counter() - t0
        assert local.n_rows == n and local.nnz == part.graph.nnz, "GPU extraction disagrees with the host-built partition"
        log(f"[bench] GPU extraction of the partition (active sets of the unpartitioned graph + sub-graph): {t_extract * 1e3:.2f} ms")
        if args.extract_on_gpu:
            gpu_part = (local, gring[:n].clone())
        del Gg, gdist, new_id
        if not args.extract_on_gpu:
            del local, gring

    if gpu_part is not None:
        G, l2g = gpu_part
        GT = G                                   # the workloads' graphs are symmetric
        t_dev = torch.arange(len(part.targets), dtype=torch.int32, device="cuda")
        gdeg = None
        if w.model == "gcn":
            gdeg = dev(w.global_graph.degrees().astype(np.int32))[l2g.long()]
        model = P.MaskedGNN(G, GT, t_dev, w.model, dparams, dtype=dtype, global_degree=gdeg, prefix_numbered=True,
                            transform_first=False if args.aggregate_first else (True if args.weights_first_all else "auto"), side_stream=not args.one_stream)
        # the host partition numbers its vertices by ascending id; its feature rows are permuted into ring order
        pos = torch.from_numpy(np.searchsorted(part.local_to_global, l2g.cpu().numpy().astype(np.int64)).astype(np.int32)).cuda()
        H0d = torch.zeros(n, ld0, dtype=dtype, device="cuda")
        P.gnn_gather_rows(dev(H0).to(dtype), pos, w.dims[0], H0d)
        model.set_input(H0d)
    else:
        G = sampled_graph if sampled_graph is not None else P.Graph.from_numpy(part.graph.row_ptr, part.graph.col_idx)
        GT = G if part.graph_t is part.graph else P.Graph.from_numpy(part.graph_t.row_ptr, part.graph_t.col_idx)
        model = P.MaskedGNN(G, GT, dev(part.targets), w.model, dparams, dtype=dtype,
                            global_degree=dev(part.global_degree) if w.model == "gcn" else None,
                            prefix_numbered=sampled_graph is not None,   # the GPU extraction numbers by (distance, id)
                            transform_first=False if args.aggregate_first else (True if args.weights_first_all else "auto"), side_stream=not args.one_stream)
        model.set_input(dev(H0).to(dtype))
    if args.layer_sampling:
        f = args.layer_sampling.split(":")
        seed_ls = int(f[2]) if len(f) > 2 else 1
        if f[0] == "fanout":
            model.layer_sampling = ("fanout", int(f[1]), seed_ls)
        else:
            pk = float(f[1])
            model.layer_sampling = ("threshold", (1 << 64) - 1 if pk >= 1.0 else max(0, int(pk * (1 << 64)) - 1), seed_ls)
    labels = dev(gg.labels(len(part.targets), w.dims[-1], w.seed))
    log(f"[bench] partition: n={n} nnz={part.graph.nnz} |T|={len(part.targets)} model={w.model} dims={w.dims} dtype={w.dtype}")

    for _ in range(args.warmup):
        model.step(labels)
    torch.cuda.synchronize()
    model.trace = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        model.step(labels)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    trace, model.trace = model.trace, None
    ms_per_step = wall / args.steps * 1e3

    per_call = {}
    for name, a, b in trace:
        per_call.setdefault(name, []).append(a.elapsed_time(b))
    call_ms = {k: float(np.mean(v)) for k, v in per_call.items()}
    edges = model.aggregated_edges()
    total_edges = sum(e["fwd"] + e["bwd"] for e in edges.values())
    hop = [int(x) for x in model.hop]
    L = model.L
    es = 4 if dtype == torch.float32 else 2

    # a first layer in the exchanged order splits its feature transform into two calls each way
    lin_f = lambda l: call_ms.get(f"linear_fwd_{l}", 0.0) + call_ms.get(f"linear_pre_{l}", 0.0)
    lin_b = lambda l: (call_ms.get(f"linear_bwd_{l}", 0.0) + call_ms.get(f"linear_bwd_{l}_neigh", 0.0) +
                       call_ms.get(f"linear_bwd_{l}_input", 0.0) + call_ms.get(f"linear_bwd_{l}_input_self", 0.0))

    # per-layer report
    layers = {}
    for l in range(1, L + 1):
        t_f = call_ms.get(f"spmm_fwd_{l}", 0.0)
        t_b = call_ms.get(f"spmm_bwd_{l}", 0.0) + call_ms.get(f"spmm_bwd_{l}_ring", 0.0)
        e = edges[l]
        F = model.agg_width(l)
        nl = model.n_rows_of_layer(l)
        gather_bytes = e["fwd"] * (4 + F * es) + nl * (8 + F * es)
        layers[str(l)] = {
            "rows": nl, "edges_fwd": e["fwd"], "edges_bwd": e["bwd"], "F": F,
            "spmm_fwd_ms": round(t_f, 4), "spmm_bwd_ms": round(t_b, 4),
            "linear_fwd_ms": round(lin_f(l), 4), "linear_bwd_ms": round(lin_b(l), 4),
            "edges_per_s_spmm": (e["fwd"] + e["bwd"]) / ((t_f + t_b) * 1e-3) if t_f + t_b > 0 else None,
            "spmm_fwd_gather_GBs": gather_bytes / (t_f * 1e-3) / 1e9 if t_f > 0 else None,
        }

    # roofline of the dominant kernel: the forward aggregation that gathers the most bytes (the later layer on a tie:
    # the plain call rather than the first layer's add-on-top form)
    dom = max(range(1, L + 1), key=lambda l: (edges[l]["fwd"] * model.agg_width(l), l))
    Fd = model.agg_width(dom)
    nd = model.n_rows_of_layer(dom)
    n_in = model.n_rows_of_layer(dom - 1) if dom > 1 else int(hop[L + 1])
    alg_bytes = edges[dom]["fwd"] * (4 + Fd * es) + nd * (8 + Fd * es)           # gather model
    compulsory = edges[dom]["fwd"] * 4 + n_in * Fd * es + nd * (8 + Fd * es)     # every input row read once
    t_dom = call_ms[f"spmm_fwd_{dom}"] * 1e-3
    src_dom, dst_dom = (model.P[dom], model.H[dom]) if dom in model.tf_layers else (model.H[dom - 1], model.A[dom])
    blocked = P.binding.spmm_workspace_bytes(G, nd, src_dom, dst_dom, Fd) > 0
    kernels = ("spmm_stream_kernel (+ spmm_seg_kernel before and spmm_sum_parts_kernel after it: column-blocked route)"
               if blocked else "spmm_rows_kernel")
    kib = MEASURED_TRAFFIC_KIB.get(args.workload, {}).get(dom) if args.scale == 1.0 else None
    if dom == 1 and 1 in model.tf_layers:        # (the layer-1 figures are those of the 602-wide gather)
        kib = None
    traffic = None
    if kib:
        traffic = (kib["fetch"] * FETCH_SCALE + kib["write"] * WRITE_SCALE) * 1024
    # `achieved` counts the ALGORITHMIC bytes of the gather model (every neighbour row of every edge); on the
    # column-blocked route most of them are served by the L2 of the compute die, so it can exceed the HBM peak.
    # `traffic` is what actually crossed from L2 to the memory fabric, `traffic_GBs` the same per second.
    roofline = {
        "kernel": f"{kernels}; gnn_masked_spmm_fwd, layer {dom}, F={Fd}",
        "bound": "hbm", "achieved": alg_bytes / t_dom / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": alg_bytes / t_dom / 1e9 / HBM_PEAK_GBS,
        "traffic": traffic, "traffic_GBs": None if traffic is None else traffic / t_dom / 1e9,
        "bytes_per_launch": alg_bytes, "launch_ms": t_dom * 1e3,
        "compulsory_bytes_per_launch": compulsory, "compulsory_GBs": compulsory / t_dom / 1e9,
    }
    # the feature-transform GEMMs against the MFMA peak of their data type
    gemm = {}
    for l in range(1, L + 1):
        K, N = w.dims[l - 1], w.dims[l]
        nl = model.n_rows_of_layer(l)
        srcs = 2 if sage else 1
        f_fwd = 2.0 * nl * K * N * srcs
        f_bwd = f_fwd * (2 if l > 1 else 1)
        tf, tb = lin_f(l) * 1e-3, lin_b(l) * 1e-3
        peak = MFMA_PEAK_TFLOPS[w.dtype]
        b_fwd = nl * (K * srcs + N) * es
        # backward, every operand once: the (already masked) output gradient and the layer inputs in, the input gradients out
        b_bwd = nl * (N + K * srcs) * es + (nl * K * srcs * es if l > 1 else 0)
        # the roof that binds a product this skinny: the slower of "operands at the HBM peak" and "flops at the MFMA peak"
        roof_f = max(b_fwd / (HBM_PEAK_GBS * 1e9), f_fwd / (peak * 1e12))
        roof_b = max(b_bwd / (HBM_PEAK_GBS * 1e9), f_bwd / (peak * 1e12))
        gemm[str(l)] = {"M": nl, "K": K * srcs, "N": N,
                        "fwd_TFLOPs": f_fwd / tf / 1e12 if tf > 0 else None, "fwd_frac_mfma": f_fwd / tf / 1e12 / peak if tf > 0 else None,
                        "fwd_GBs": b_fwd / tf / 1e9 if tf > 0 else None,
                        "fwd_binds": "hbm" if b_fwd / (HBM_PEAK_GBS * 1e9) > f_fwd / (peak * 1e12) else "mfma",
                        "fwd_frac_roof": roof_f / tf if tf > 0 else None,
                        "bwd_TFLOPs": f_bwd / tb / 1e12 if tb > 0 else None, "bwd_frac_mfma": f_bwd / tb / 1e12 / peak if tb > 0 else None,
                        "bwd_GBs": b_bwd / tb / 1e9 if tb > 0 else None,
                        "bwd_binds": "hbm" if b_bwd / (HBM_PEAK_GBS * 1e9) > f_bwd / (peak * 1e12) else "mfma",
                        "bwd_frac_roof": roof_b / tb if tb > 0 else None}

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        rows1 = model.ring_ids[: model.n_rows_of_layer(1)]
        if gpu_part is not None:     # same vertices in the host partition's numbering (H0 and part.graph use it)
            rows1 = pos[rows1.long()]
        cpu = cpu_baseline(part, w, params, H0, rows1.cpu().numpy())

    out = {
        "metric": "aggregated_edges_per_sec", "value": total_edges / (wall / args.steps), "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{CONFIG_INDEX[args.workload]}]: {gg.WORKLOADS[args.workload]}",
                   "scale": args.scale, "n_local": n, "nnz_local": part.graph.nnz, "targets": len(part.targets),
                   "hop_offsets": hop, "layers": L},
        "epoch_ms": sum(v for k, v in call_ms.items() if k != "active_sets"),
        "active_sets_ms": call_ms.get("active_sets"),
        "sampling_ms": None if t_sample is None else t_sample * 1e3, "sampled_edges": kept,
        "extract_ms": None if t_extract is None else t_extract * 1e3,
        "partition_built_on": "gpu ((distance, id) numbering)" if (gpu_part is not None or sampled_graph is not None)
                              else "host (ascending-id numbering)",
        "aggregated_edges_per_step": total_edges,
        "layers_weights_first": sorted(model.tf_layers),
        "layer_sampling": args.layer_sampling,
        "layer_mask_ms": sum(v for k, v in call_ms.items() if k.startswith("layer_mask")) if args.layer_sampling else None,
        "per_layer": layers, "roofline": roofline, "roofline_gemm": gemm, "cpu_baseline": cpu,
        "call_ms": {k: round(v, 4) for k, v in call_ms.items()},
    }
    print(json.dumps(out))


def bench_res_model(args, w, part, sampled_graph, dtype):
    """The deep residual GraphSAGE on the workload's partition (host-built numbering unless the partition was sampled
    on the GPU): same metric, the forward aggregation of a middle layer as the dominant call."""
    import torch
    import graphgen as gg
    import paper_2311_06837_amd as P
    assert w.model == "sage" and args.res_layers >= 2
    L, hid = args.res_layers, w.dims[1]
    dims = [w.dims[0]] + [hid] * (L - 1) + [w.dims[-1]]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    # the partition's halo was cut for the workload's own depth: deeper models see the same vertices (the late active
    # sets are the whole partition, as in configs[3])
    G = sampled_graph if sampled_graph is not None else P.Graph.from_numpy(part.graph.row_ptr, part.graph.col_idx)
    params = [{k: dev(v) for k, v in p.items()} for p in gg.res_layer_weights(dims, w.seed)]
    model = P.ResSAGEPlus(G, G, dev(part.targets), params, dtype=dtype, recompute=args.recompute,
                          prefix_numbered=sampled_graph is not None)
    n = part.graph.n_rows
    model.set_input(dev(gg.features(n, w.dims[0], w.seed, ld=P.row_stride(w.dims[0], dtype))).to(dtype))
    labels = dev(gg.labels(len(part.targets), w.dims[-1], w.seed))
    for _ in range(args.warmup):
        model.step(labels)
    torch.cuda.synchronize()
    model.trace = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        model.step(labels)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    trace, model.trace = model.trace, None
    per_call = {}
    for name, a, b in trace:
        per_call.setdefault(name, []).append(a.elapsed_time(b))
    call_ms = {k: float(np.mean(v)) for k, v in per_call.items()}
    edges = model.aggregated_edges()
    total_edges = sum(e["fwd"] + e["bwd"] + e["again"] for e in edges.values())
    es = 4 if dtype == torch.float32 else 2
    dom = max(range(2, L + 1), key=lambda l: call_ms.get(f"spmm_fwd_{l}", 0.0))
    nd = model.n_rows_of_layer(dom)
    alg_bytes = edges[dom]["fwd"] * (4 + hid * es) + nd * (8 + hid * es)
    t_dom = call_ms[f"spmm_fwd_{dom}"] * 1e-3
    group = lambda pre: sum(v for k, v in call_ms.items() if k.startswith(pre))
    out = {
        "metric": "aggregated_edges_per_sec", "value": total_edges / (wall / args.steps), "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"deep residual GraphSAGE (ResSAGE+), {L} layers, hidden {hid}, on the partition of "
                               f"configs[{CONFIG_INDEX[args.workload]}]: {gg.WORKLOADS[args.workload]}",
                   "scale": args.scale, "n_local": n, "nnz_local": part.graph.nnz, "targets": len(part.targets),
                   "layers": L, "recompute": bool(args.recompute)},
        "epoch_ms": sum(v for k, v in call_ms.items() if k != "active_sets"),
        "activation_bytes": model.activation_bytes(),
        "aggregated_edges_per_step": total_edges,
        "ms_by_kind": {"spmm_fwd": group("spmm_fwd"), "spmm_bwd": group("spmm_bwd"), "linear_fwd": group("linear_fwd"),
                       "linear_bwd": group("linear_bwd"), "layer_norm_fwd": group("ln_fwd"), "layer_norm_bwd": group("ln_bwd"),
                       "residual": group("residual"), "active_sets": call_ms.get("active_sets"), "softmax_ce": call_ms.get("softmax_ce")},
        "roofline": {"kernel": f"spmm_rows_kernel; gnn_masked_spmm_fwd, layer {dom}, F={hid}", "bound": "hbm",
                     "achieved": alg_bytes / t_dom / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": alg_bytes / t_dom / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "bytes_per_launch": alg_bytes, "launch_ms": t_dom * 1e3},
        "cpu_baseline": None,
    }
    print(json.dumps(out))


def cpu_baseline(part, w, params, H0, rows_all):
    """The oracle as it stands, on this machine's host cores: layer-1 masked aggregation + feature transform
    (forward) on a seeded sample of the layer's rows (rows_all, local ids of the host partition), sized for
    about 10-30 s."""
    import oracle
    K, N = w.dims[0], w.dims[1]
    deg = np.diff(part.graph.row_ptr)[rows_all].astype(np.int64)
    # budget: about 2e11 fp64 multiply-adds of aggregation (roughly 10-20 s on 16 cores with the gathers)
    budget = 2.0e11 / max(K, 1)
    rng = np.random.default_rng(12345)
    order = rng.permutation(rows_all.size)
    take = int(np.searchsorted(np.cumsum(deg[order]), budget)) + 1
    take = max(1, min(take, rows_all.size))
    rows = np.sort(rows_all[order[:take]]).astype(np.int32)
    sample_edges = int(deg[order[:take]].sum())
    X = np.ascontiguousarray(H0[:, :K], dtype=np.float64)
    if w.dtype == "bf16":
        oracle.round_bf16(X)
    n = part.graph.n_rows
    length = np.diff(part.graph.row_ptr)
    if w.model == "gcn":
        s = oracle.norm_scales("sym", part.global_degree)
        rs, cs = s, s
    else:
        rs, cs = oracle.norm_scales("mean", length), None
    A = np.zeros((n, K))
    Hn = np.zeros((n, N))
    p = params[0]
    t0 = time.perf_counter()
    oracle.spmm_fwd(part.graph.row_ptr, part.graph.col_idx, rows, X, A, K, rs, cs)
    t_agg = time.perf_counter() - t0
    oracle.linear_fwd(rows, A, X if w.model == "sage" else None, K, p["W_neigh"], p.get("W_self"), p["bias"], Hn, True)
    t_all = time.perf_counter() - t0
    log(f"[bench] cpu oracle: {take} rows, {sample_edges} edges, aggregation {t_agg:.2f}s, with transform {t_all:.2f}s")
    return {"value": sample_edges / t_all, "unit": "edges/s", "cores": oracle.n_threads(), "kind": "oracle",
            "sample": f"layer-1 forward (masked aggregation + feature transform) of {take} seeded rows of R_1 "
                      f"({sample_edges} edges) of the same partition, fp64, gcc -O2 -fopenmp",
            "seconds": t_all, "aggregation_only_edges_per_s": sample_edges / t_agg}


if __name__ == "__main__":
    main()
