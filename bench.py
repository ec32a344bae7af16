#!/usr/bin/env python3
"""Benchmark of the masked full-neighbourhood GNN hot path on ONE MI355X.

A step is one pass of the whole hot path over one synthetic partition: active-set construction
(frontier expansion), then per layer masked aggregation + feature transform, the loss, and the
matching backward pass.  Inputs are resident in HBM before the timed region.  One JSON line on
stdout:
  value     aggregated edges per second = (edges visited by all forward and backward aggregations
            of a step, counted for the paper's order of a layer's halves) / (wall time of a step)
  roofline  the dominant kernel (the forward aggregation that gathers the most bytes), against the HBM
            peak; `frac` is never above 1 by construction, see roofline_of_call()
  roofline_gemm / roofline_sets / roofline_sampling / roofline_extract   the other steps of the path
  call_ms   every C-ABI call between two events on the stream it is enqueued on; the weight-gradient
            products run on a second stream beside the backward aggregations, so the sum of the entries
            exceeds the step (ms_per_step is the wall time)
  cpu_baseline  the CPU oracle timed on this machine's host cores on a bounded sample (reported for
            context; it is not the target)
  others    the same record for the other single-GPU workloads (configs[2], [3], [4]), fewer steps

python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1] [--others cfg2,cfg3,cfg4 | --no-others]

Counter-derived figures (`traffic`, `mfma_busy`) come from profiles/counters_sidecar.json, which
bench_counters.py writes from rocprofv3 --pmc runs of this file's --pmc-probe mode; they are used only
when the sidecar was measured on the same kernel sources (hash of csrc/ and include/), else null.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
SIDECAR = os.path.join(ROOT, "profiles", "counters_sidecar.json")
CONFIG_INDEX = {"cfg0": 0, "cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def source_sha() -> str:
    """Hash of the kernel sources and the header: identifies the build a counter sidecar belongs to."""
    h = hashlib.sha256()
    files = [os.path.join(ROOT, "include", "gnnhot.h")]
    csrc = os.path.join(ROOT, "paper_2311_06837_amd", "csrc")
    files += sorted(os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith((".hip", ".h")))
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def load_sidecar():
    """The counter sidecar if it exists AND was measured on these sources; else None (figures become null)."""
    try:
        d = json.load(open(SIDECAR))
    except (OSError, ValueError):
        return None
    if d.get("source_sha") != source_sha():
        log(f"[bench] {SIDECAR} was measured on other kernel sources ({d.get('source_sha')}): counter figures are null")
        return None
    return d


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
    (distance, id) numbering.  Returns a host-side Partition (for the CPU baseline), the device graph and the two times
    (best of three passes each; the first pass also warms the allocator)."""
    import torch
    import graphgen as gg
    import paper_2311_06837_amd as P
    g, T = w.global_graph, w.targets_global.astype(np.int32)          # targets ascending
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Td = torch.from_numpy(T).cuda()
    ws = P.Workspace()
    bits = P.gnn_make_bitmap(Td, g.n_rows)
    t_sample, t_extract = float("inf"), float("inf")
    for _ in range(4):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rp, ci = P.gnn_sample_boundary(G, bits, Td, w.fanout, w.sample_seed, ws=ws)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        local, l2g, hop = P.gnn_extract_sampled_partition(G, Td, rp, ci, ws=ws)     # symmetric graph: gT = g
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        t_sample, t_extract = min(t_sample, t1 - t0), min(t_extract, t2 - t1)
    kept = int(ci.numel())
    l2g_h = l2g.cpu().numpy().astype(np.int64)
    lg = gg.CSR(local.n_rows, local.n_rows, local.row_ptr.cpu().numpy(), local.col_idx.cpu().numpy())
    part = gg.Partition(lg, lg, l2g_h, np.arange(T.size, dtype=np.int32), g.degrees()[l2g_h].astype(np.int32))
    return part, local, t_sample, t_extract, kept


def roofline_of_call(kernels, what, t_s, gather_bytes, compulsory_bytes, blocked, counters):
    """HBM roofline record of one aggregation call.

    gather model   every neighbour row of every edge comes from memory (no reuse): index + row per edge, row_ptr +
                   output row per active row.  What a gather kernel WITHOUT designed reuse must move.
    compulsory     every input row, index and output row exactly once (perfect reuse): the lower bound.
    `achieved` / `frac` (never above 1):
      one-launch route   gather-model bytes / time, capped at what the counters say crossed the fabric when a same-build
                         counter reading exists and is smaller (reuse the caches found on their own)
      column-blocked     its point is reuse inside the compute dies' L2s, so gather-model bytes are not memory bytes:
                         counter bytes (L2 <-> fabric) / time when a same-build reading exists, else the compulsory bytes
                         / time (a floor).  The gather-model rate is reported separately as gather_GBs.
    """
    traffic = None
    extra = {}
    if counters:
        traffic = counters.get("traffic_bytes")
        extra = {k: counters[k] for k in ("fetch_bytes_by_request_size", "write_bytes", "fetch_size_KiB", "write_size_KiB",
                                          "tcc_hit", "tcc_miss", "l2_hit_rate") if k in counters}
    if blocked:
        basis = "counters (L2<->fabric bytes of the same build)" if traffic else "compulsory bytes (no same-build counter reading)"
        ach_bytes = traffic if traffic else compulsory_bytes
    else:
        ach_bytes, basis = gather_bytes, "gather model"
        if traffic and traffic < gather_bytes:
            ach_bytes, basis = traffic, "counters (below the gather model: cache reuse)"
        if ach_bytes / t_s / 1e9 > HBM_PEAK_GBS:    # rows re-read from L2: only the lower bound can be claimed
            ach_bytes, basis = compulsory_bytes, "compulsory bytes (the gather model exceeds the HBM peak and no counter reading says less)"
    ach = ach_bytes / t_s / 1e9
    return {
        "kernel": f"{kernels}; {what}", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": ach / HBM_PEAK_GBS, "frac_basis": basis,
        "traffic": traffic, "traffic_GBs": None if traffic is None else traffic / t_s / 1e9,
        "bytes_per_launch": ach_bytes, "launch_ms": t_s * 1e3,
        "gather_bytes_per_launch": gather_bytes, "gather_GBs": gather_bytes / t_s / 1e9,
        "compulsory_bytes_per_launch": compulsory_bytes, "compulsory_GBs": compulsory_bytes / t_s / 1e9,
        "frac_compulsory": compulsory_bytes / t_s / 1e9 / HBM_PEAK_GBS, **extra,
    }


def simple_roofline(kernel, t_s, alg_bytes, counters=None, note=None):
    out = {"kernel": kernel, "bound": "hbm", "achieved": alg_bytes / t_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": alg_bytes / t_s / 1e9 / HBM_PEAK_GBS, "bytes_per_launch": alg_bytes, "launch_ms": t_s * 1e3,
           "traffic": counters.get("traffic_bytes") if counters else None}
    if note:
        out["note"] = note
    return out


class Setup:
    """Everything of one workload that lives on the GPU before the timed region."""
    pass


def setup_workload(args, name):
    import torch
    import graphgen as gg
    import paper_2311_06837_amd as P

    w = build_partition(name, args.scale)
    S = Setup()
    S.w, S.name = w, name
    S.t_sample = S.kept = S.t_extract = S.sampled_graph = None
    if w.partition is None:
        S.part, S.sampled_graph, S.t_sample, S.t_extract, S.kept = sampled_partition_cfg4(w)
        log(f"[bench] GPU sampling {S.t_sample * 1e3:.2f} ms, GPU extraction of the sampled partition {S.t_extract * 1e3:.2f} ms")
    else:
        S.part = w.partition
    part = S.part
    S.dtype = torch.float32 if w.dtype == "f32" else torch.bfloat16
    S.sage = w.model == "sage"
    S.n = n = part.graph.n_rows
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    S.params = gg.layer_weights(w.dims, S.sage, w.seed)
    dparams = [{k: dev(v) for k, v in p.items()} for p in S.params]
    ld0 = P.row_stride(w.dims[0], S.dtype)
    S.H0 = gg.features(n, w.dims[0], w.seed, ld=ld0)
    S.n_layers = len(w.dims) - 1
    S.edges_traversed = None
    if args.res_layers:
        return S

    # Step (a-1) of the path, outside the timed step like the sampling: the partition's one-hop graph extracted on
    # the GPU from the unpartitioned graph, vertices renumbered by (distance, id).
    S.gpu_part, S.pos = None, None
    if w.partition is not None:
        Gg = P.Graph.from_numpy(w.global_graph.row_ptr, w.global_graph.col_idx)
        Tg = dev(w.targets_global.astype(np.int32))
        ews = P.Workspace()
        S.t_extract = float("inf")
        for rep_i in range(3):       # first pass warms the allocator
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            gdist, gring, _, ghop = P.gnn_build_active_sets(Gg, Tg, S.n_layers, ws=ews, gt=Gg)   # symmetric: its own transpose
            local, new_id = P.gnn_extract_partition(Gg, gring, int(ghop[-1]), gdist, S.n_layers, ws=ews)
            torch.cuda.synchronize()
            S.t_extract = min(S.t_extract, time.perf_counter() - t0)
        assert local.n_rows == n and local.nnz == part.graph.nnz, "GPU extraction disagrees with the host-built partition"
        log(f"[bench] GPU extraction of the partition (active sets of the unpartitioned graph + sub-graph): {S.t_extract * 1e3:.2f} ms")
        S.edges_traversed = int(w.global_graph.degrees()[part.local_to_global].astype(np.int64).sum())
        if not args.host_partition:
            S.gpu_part = (local, gring[:n].clone())
        del Gg, gdist, new_id, local, gring

    tf = False if args.aggregate_first else (True if args.weights_first_all else "auto")
    if S.gpu_part is not None:
        G, l2g = S.gpu_part
        t_dev = torch.arange(len(part.targets), dtype=torch.int32, device="cuda")
        gdeg = None
        if w.model == "gcn":
            gdeg = dev(w.global_graph.degrees().astype(np.int32))[l2g.long()]
        model = P.MaskedGNN(G, G, t_dev, w.model, dparams, dtype=S.dtype, global_degree=gdeg, prefix_numbered=True,
                            transform_first=tf, side_stream=not args.one_stream, fused_forward=args.fused,
                            grad_first=False if args.chain_rule_order else "auto")
        # the host partition numbers its vertices by ascending id; its feature rows are permuted into ring order
        S.pos = torch.from_numpy(np.searchsorted(part.local_to_global, l2g.cpu().numpy().astype(np.int64)).astype(np.int32)).cuda()
        H0d = torch.zeros(n, ld0, dtype=S.dtype, device="cuda")
        P.gnn_gather_rows(dev(S.H0).to(S.dtype), S.pos, w.dims[0], H0d)
        model.set_input(H0d)
    else:
        G = S.sampled_graph if S.sampled_graph is not None else P.Graph.from_numpy(part.graph.row_ptr, part.graph.col_idx)
        GT = G if part.graph_t is part.graph else P.Graph.from_numpy(part.graph_t.row_ptr, part.graph_t.col_idx)
        model = P.MaskedGNN(G, GT, dev(part.targets), w.model, dparams, dtype=S.dtype,
                            global_degree=dev(part.global_degree) if w.model == "gcn" else None,
                            prefix_numbered=S.sampled_graph is not None,   # the GPU extraction numbers by (distance, id)
                            transform_first=tf, side_stream=not args.one_stream, fused_forward=args.fused,
                            grad_first=False if args.chain_rule_order else "auto")
        model.set_input(dev(S.H0).to(S.dtype))
    if args.layer_sampling:
        f = args.layer_sampling.split(":")
        seed_ls = int(f[2]) if len(f) > 2 else 1
        if f[0] == "fanout":
            model.layer_sampling = ("fanout", int(f[1]), seed_ls)
        else:
            pk = float(f[1])
            model.layer_sampling = ("threshold", (1 << 64) - 1 if pk >= 1.0 else max(0, int(pk * (1 << 64)) - 1), seed_ls)
    S.G, S.model = G, model
    S.labels = dev(gg.labels(len(part.targets), w.dims[-1], w.seed))
    log(f"[bench] partition: n={n} nnz={part.graph.nnz} |T|={len(part.targets)} model={w.model} dims={w.dims} dtype={w.dtype}")
    return S


def dominant_layer(model, edges):
    """The forward aggregation that gathers the most bytes (the later layer on a tie: the plain call rather than the
    first layer's add-on-top form)."""
    return max(range(1, model.L + 1), key=lambda l: (edges[l]["fwd"] * model.agg_width(l), l))


def run_workload(args, name, steps, warmup, cpu_flops):
    import torch
    import graphgen as gg
    import paper_2311_06837_amd as P

    S = setup_workload(args, name)
    w, part, model, dtype = S.w, S.part, getattr(S, "model", None), S.dtype
    if args.res_layers:
        return bench_res_model(args, w, part, S.sampled_graph, dtype, steps, warmup)
    n, G = S.n, S.G

    for _ in range(warmup):
        model.step(S.labels)
    torch.cuda.synchronize()
    model.trace = []
    t0 = time.perf_counter()
    for _ in range(steps):
        model.step(S.labels)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    trace, model.trace = model.trace, None
    ms_per_step = wall / steps * 1e3

    def mean_ms(tr):
        per_call = {}
        for nm, a, b in tr:
            per_call.setdefault(nm, []).append(a.elapsed_time(b))
        return {k: float(np.mean(v)) for k, v in per_call.items()}
    call_ms = mean_ms(trace)
    # Outside the timed region: two more steps with every call on the one stream, so that the events around a weight-
    # gradient product time that product alone (in the timed steps it shares the GPU with an aggregation).
    alone_ms, costs = call_ms, model.product_costs()
    if model.side is not None:
        side_stream, model.side = model.side, None
        costs = model.product_costs()      # the one-stream step forms some gradients in fewer, larger calls
        model.step(S.labels)
        model.trace = []
        for _ in range(2):
            model.step(S.labels)
        torch.cuda.synchronize()
        alone_ms, model.trace = mean_ms(model.trace), None
        model.side = side_stream
    edges = model.aggregated_edges()
    total_edges = sum(e["fwd"] + e["bwd"] for e in edges.values())
    hop = [int(x) for x in model.hop]
    L = model.L
    es = 4 if dtype == torch.float32 else 2
    sidecar = load_sidecar()
    side = (sidecar or {}).get("workloads", {}).get(name, {}) if args.scale == 1.0 else {}

    # a layer in the exchanged order splits its feature transform into two calls each way
    lin_f = lambda l: call_ms.get(f"linear_fwd_{l}", 0.0) + call_ms.get(f"linear_pre_{l}", 0.0)
    lin_b = lambda l: (call_ms.get(f"linear_bwd_{l}", 0.0) + call_ms.get(f"linear_bwd_{l}_neigh", 0.0) +
                       call_ms.get(f"linear_bwd_{l}_input", 0.0) + call_ms.get(f"linear_bwd_{l}_input_self", 0.0))

    layers = {}
    for l in range(1, L + 1):
        t_f = call_ms.get(f"spmm_fwd_{l}", 0.0) + call_ms.get(f"fused_fwd_{l}", 0.0)   # fused: aggregation and transform together
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

    # ---- roofline of the dominant kernel
    dom = dominant_layer(model, edges)
    Fd = model.agg_width(dom)
    nd = model.n_rows_of_layer(dom)
    n_in = model.n_rows_of_layer(dom - 1) if dom > 1 else int(hop[L + 1])
    gather_bytes = edges[dom]["fwd"] * (4 + Fd * es) + nd * (8 + Fd * es)
    compulsory = edges[dom]["fwd"] * 4 + n_in * Fd * es + nd * (8 + Fd * es)
    t_dom = (call_ms.get(f"spmm_fwd_{dom}") or call_ms[f"fused_fwd_{dom}"]) * 1e-3
    if dom in model.fused_layers:
        blocked, kernels = False, "fused_agg_linear_kernel (aggregation and feature transform in one kernel)"
    else:
        src_dom, dst_dom = (model.P[dom], model.H[dom]) if dom in model.tf_layers else (model.H[dom - 1], model.A[dom])
        blocked = P.binding.spmm_workspace_bytes(G, nd, src_dom, dst_dom, Fd) > 0
        kernels = ("spmm_stream_kernel (+ spmm_seg_kernel before and spmm_sum_parts_kernel after it: column-blocked route)"
                   if blocked else "spmm_rows_kernel")
    c_dom = side.get("spmm_fwd_dom") if side.get("dominant_layer") == dom else None
    roofline = roofline_of_call(kernels, f"gnn_masked_spmm_fwd, layer {dom}, F={Fd}", t_dom, gather_bytes, compulsory, blocked, c_dom)

    # ---- the feature-transform products against the roof that binds each of them: the slower of "operands once at
    # the HBM peak" and "flops at the MFMA peak of the data type".  Timed alone on the GPU (see above).
    peak = MFMA_PEAK_TFLOPS[w.dtype]
    gemm_calls = {}
    for nm, c in costs.items():
        t = alone_ms.get(nm, 0.0) * 1e-3
        if t <= 0:
            continue
        t_hbm, t_mfma = c["bytes"] / (HBM_PEAK_GBS * 1e9), c["flops"] / (peak * 1e12)
        gemm_calls[nm] = {"layer": c["layer"], "direction": c["direction"], "ms": t * 1e3, "TFLOPs": c["flops"] / t / 1e12,
                          "GBs": c["bytes"] / t / 1e9, "binds": "hbm" if t_hbm > t_mfma else "mfma",
                          "roof_ms": max(t_hbm, t_mfma) * 1e3, "frac_roof": max(t_hbm, t_mfma) / t,
                          "frac_mfma": c["flops"] / t / 1e12 / peak}
    gemm = {"timing": "HIP events around each product call with the call alone on the GPU (extra one-stream steps after the "
                      "timed region); a layer's figure = sum of its calls' roof times / sum of their durations",
            "calls": gemm_calls}
    for l in range(1, L + 1):
        rec = {"K": w.dims[l - 1], "N": w.dims[l], "rows": model.n_rows_of_layer(l),
               "order": "transform first" if l in model.tf_layers else "aggregate first",
               "input_gradient": "from the aggregated output gradient, one two-source product" if l in model.gf_layers else
                                 ("none" if l == 1 else "per source, then aggregated")}
        for d in ("fwd", "bwd"):
            sel = [c for c in gemm_calls.values() if c["layer"] == l and c["direction"] == d]
            if sel:
                tt, rr = sum(c["ms"] for c in sel), sum(c["roof_ms"] for c in sel)
                ff = sum(c["TFLOPs"] * c["ms"] for c in sel)
                rec[f"{d}_ms"] = tt
                rec[f"{d}_frac_roof"] = rr / tt
                rec[f"{d}_TFLOPs"] = ff / tt
                rec[f"{d}_frac_mfma"] = ff / tt / peak
                rec[f"{d}_binds"] = max(sel, key=lambda c: c["roof_ms"])["binds"]
        if l == dom:
            for key in ("linear_fwd_dom", "linear_bwd_dom"):
                if key in side:
                    rec[key + "_counters"] = side[key]
        gemm[str(l)] = rec

    # ---- set expansion: 4 B per frontier edge (rows of rings 0 .. L-1), 8 B row bounds per frontier vertex, 8 B (distance and
    # ring-list entry) per reached vertex
    rp = model.g.row_ptr.long()
    ring = model.ring_ids.long()
    n_front = int(hop[L])
    frontier_edges = int((rp[ring[:n_front] + 1] - rp[ring[:n_front]]).sum().item())
    reached = int(hop[L + 1])
    sets_bytes = 4 * frontier_edges + 8 * n_front + 8 * reached
    t_sets = call_ms["active_sets"] * 1e-3
    roof_sets = simple_roofline(f"as_expand / as_count / as_emit kernels; gnn_build_active_sets, L={L}", t_sets, sets_bytes,
                                side.get("active_sets"))
    roof_sets.update({"frontier_edges": frontier_edges, "reached_vertices": reached, "levels": L,
                      "edges_per_s": frontier_edges / t_sets})
    roof_sampling = None
    if S.t_sample is not None:
        deg_t = w.global_graph.degrees()[w.targets_global].astype(np.int64)
        cand = int(deg_t.sum())
        nt = int(w.targets_global.size)
        samp_bytes = 4 * cand + 8 * nt + 4 * S.kept + 4 * (nt + 1)
        roof_sampling = simple_roofline("sb_count_kernel + sb_fill_kernel; gnn_sample_boundary (count and fill pass, host "
                                        "allocation of the output between them)", S.t_sample, samp_bytes, side.get("sampling"))
        roof_sampling.update({"candidate_edges": cand, "kept_edges": S.kept, "targets": nt, "edges_per_s": cand / S.t_sample})
    roof_extract = None
    if S.t_extract is not None:
        if S.edges_traversed is not None:      # full halo: active sets of the unpartitioned graph + induced sub-graph
            ex_bytes = 4 * S.edges_traversed + 8 * n + 4 * part.graph.nnz + 8 * n
            what = "gnn_build_active_sets on the unpartitioned graph + gnn_extract_partition (count and fill pass)"
        else:                                  # sampled: kept rows -> rings -> local rows
            ex_bytes = 4 * S.kept + 8 * n + 4 * part.graph.nnz + 8 * n
            what = "gnn_expand_row_ptr + gnn_build_active_sets + gnn_extract_sampled_partition (count and fill pass)"
        roof_extract = simple_roofline(what, S.t_extract, ex_bytes, None,
                                       note="wall time of the whole chain incl. two host round trips for output sizes")

    cpu = None
    if cpu_flops > 0:
        rows1 = model.ring_ids[: model.n_rows_of_layer(1)]
        if S.pos is not None:     # same vertices in the host partition's numbering (H0 and part.graph use it)
            rows1 = S.pos[rows1.long()]
        cpu = cpu_baseline(part, w, S.params, S.H0, rows1.cpu().numpy(), cpu_flops)

    out = {
        "metric": "aggregated_edges_per_sec", "value": total_edges / (wall / steps), "unit": "edges/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{CONFIG_INDEX[name]}]: {gg.WORKLOADS[name]}",
                   "scale": args.scale, "n_local": n, "nnz_local": part.graph.nnz, "targets": len(part.targets),
                   "hop_offsets": hop, "layers": L},
        "epoch_ms": sum(v for k, v in call_ms.items() if k != "active_sets"),
        "active_sets_ms": call_ms.get("active_sets"),
        "sampling_ms": None if S.t_sample is None else S.t_sample * 1e3, "sampled_edges": S.kept,
        "extract_ms": None if S.t_extract is None else S.t_extract * 1e3,
        "partition_built_on": "gpu ((distance, id) numbering)" if (S.gpu_part is not None or S.sampled_graph is not None)
                              else "host (ascending-id numbering)",
        "aggregated_edges_per_step": total_edges,
        "layers_weights_first": sorted(model.tf_layers), "layers_gradient_aggregated_first": sorted(model.gf_layers),
        "layers_fused_forward": sorted(model.fused_layers),
        "layer_sampling": args.layer_sampling,
        "layer_mask_ms": sum(v for k, v in call_ms.items() if k.startswith("layer_mask")) if args.layer_sampling else None,
        "per_layer": layers, "roofline": roofline, "roofline_gemm": gemm, "roofline_sets": roof_sets,
        "roofline_sampling": roof_sampling, "roofline_extract": roof_extract, "cpu_baseline": cpu,
        "counters_sidecar": None if not side else {"source_sha": sidecar["source_sha"], "file": "profiles/counters_sidecar.json"},
        "call_ms": {k: round(v, 4) for k, v in call_ms.items()},
    }
    del model, S
    torch.cuda.empty_cache()
    return out


# ---------------------------------------------------------------------------------------------------------------
# counter probe: the calls whose counters profiles/ reports, each repeated a few times from a thread of its own, so
# that a rocprofv3 --pmc run of this mode can be split by the Thread_Id column (see bench_counters.py)
# ---------------------------------------------------------------------------------------------------------------
def pmc_probe(args, name, manifest_path, repeats=3):
    import torch
    import paper_2311_06837_amd as P

    args.one_stream = True
    S = setup_workload(args, name)
    model, w = S.model, S.w
    model.step(S.labels)            # every buffer of the step holds real values; also the lazy module loads
    torch.cuda.synchronize()
    edges = model.aggregated_edges()
    dom = dominant_layer(model, edges)
    L = model.L
    groups = {}

    def in_thread(tag, fn):
        box = {}

        def body():
            torch.cuda.set_device(0)
            box["tid"] = threading.get_native_id()
            for _ in range(repeats):
                fn()
            torch.cuda.synchronize()
        th = threading.Thread(target=body)
        th.start()
        th.join()
        groups[tag] = {"thread_id": box["tid"], "repeats": repeats}

    p = model.params[dom - 1]
    K, N = model.dims[dom - 1], model.dims[dom]
    nl = model.n_rows_of_layer(dom)
    sage = model.kind == "sage"
    assert dom not in model.tf_layers, "the probe expects the dominant call in the paper's order"
    in_thread("active_sets", lambda: model.build_active_sets())
    in_thread("spmm_fwd_dom", lambda: P.gnn_masked_spmm_fwd(model.g, model.rows, nl, model.H[dom - 1], model.A[dom], K, model.rs,
                                                            model.cs, ws=model.ws))
    in_thread("linear_fwd_dom", lambda: P.gnn_linear_fwd(model.rows, nl, model.A[dom], model.H[dom - 1] if sage else None, K,
                                                         p["W_neigh"], p.get("W_self"), p["bias"], model.H[dom], relu=(dom < L),
                                                         ws=model.ws))
    gr = model.grads[dom - 1]
    if dom > 1:
        in_thread("linear_bwd_dom", lambda: P.gnn_linear_bwd(model.rows, nl, model.dH[dom], None, False, model.A[dom],
                                                             model.H[dom - 1] if sage else None, K, p["W_neigh"], p.get("W_self"),
                                                             gr["dW_neigh"], gr.get("dW_self"), gr["dbias"], model.dA[dom],
                                                             model.dH[dom - 1] if sage else None, ws=model.ws))
    if w.partition is None:        # configs[4]: the sampler
        g = w.global_graph
        Gg = P.Graph.from_numpy(g.row_ptr, g.col_idx)
        Td = torch.from_numpy(w.targets_global.astype(np.int32)).cuda()
        bits = P.gnn_make_bitmap(Td, g.n_rows)
        sws = P.Workspace()
        P.gnn_sample_boundary(Gg, bits, Td, w.fanout, w.sample_seed, ws=sws)
        in_thread("sampling", lambda: P.gnn_sample_boundary(Gg, bits, Td, w.fanout, w.sample_seed, ws=sws))
    # a plain copy of known size: what the byte counters read for it scales the readings of the other groups
    n_copy, f_copy = 1 << 20, 256
    src = torch.empty(n_copy, f_copy, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    ids = torch.arange(n_copy, dtype=torch.int32, device="cuda")
    P.gnn_gather_rows(src, ids, f_copy, dst)
    in_thread("copy_calibration", lambda: P.gnn_gather_rows(src, ids, f_copy, dst))
    groups["copy_calibration"].update({"bytes_read": n_copy * f_copy * 4 + n_copy * 4, "bytes_written": n_copy * f_copy * 4})
    json.dump({"workload": name, "source_sha": source_sha(), "dominant_layer": dom, "groups": groups,
               "shapes": {"rows": nl, "K": K, "N": N, "edges_fwd": edges[dom]["fwd"], "sage": sage, "dtype": w.dtype}},
              open(manifest_path, "w"))
    log(f"[bench] probe manifest -> {manifest_path}")


def eas_bench(args, name):
    """The paper's expansion-aware traversal (section 5.3.1) on the workload's unpartitioned graph, one cell (hops, fanout,
    rule) of its sensitivity grid per entry of --eas: traversal and extraction times and the size of the halo."""
    import torch
    import paper_2311_06837_amd as P
    w = build_partition(name, args.scale)
    g = w.global_graph
    G = P.Graph.from_numpy(g.row_ptr, g.col_idx)
    Td = torch.from_numpy(w.targets_global.astype(np.int32)).cuda()
    ws = P.Workspace()
    cells = []
    for cell in args.eas.split(","):
        f = cell.split(":")
        hops, fanout, rule = int(f[0]), int(f[1]), (f[2] if len(f) > 2 else "degree")
        best_t, best_e = float("inf"), float("inf")
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            dist, ring, off, hop = P.gnn_eas_traverse(G, Td, hops, fanout, rule=rule, seed=w.sample_seed, ws=ws)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            local, _ = P.gnn_extract_partition(G, ring, int(hop[-1]), dist, hops, ws=ws)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            best_t, best_e = min(best_t, t1 - t0), min(best_e, t2 - t1)
        deg = g.degrees().astype(np.int64)
        ring_h = ring[: int(hop[-1])].cpu().numpy()
        front = ring_h[: int(hop[hops])]
        e_front = int(deg[front].sum())
        # the degree rule reads the whole graph once per hop (connection counts); both rules read the frontier rows
        alg = 4 * e_front + (4 * g.nnz * hops if rule == "degree" else 0) + 8 * int(hop[-1])
        cells.append({"hops": hops, "fanout": fanout, "rule": rule, "traverse_ms": best_t * 1e3, "extract_ms": best_e * 1e3,
                      "halo_vertices": int(hop[-1]) - int(hop[1]), "local_vertices": int(hop[-1]), "local_edges": local.nnz,
                      "ring_sizes": [int(hop[j + 1]) - int(hop[j]) for j in range(hops + 1)],
                      "frontier_edges": e_front, "algorithmic_GBs": alg / best_t / 1e9,
                      "frac_hbm_peak": alg / best_t / 1e9 / HBM_PEAK_GBS})
        log(f"[bench] eas {cell}: traverse {best_t * 1e3:.2f} ms, extract {best_e * 1e3:.2f} ms, local n={int(hop[-1])} nnz={local.nnz}")
    return {"metric": "eas_traversal_ms", "unit": "ms", "n_gpus": 1, "data": "synthetic",
            "config": {"workload": f"expansion-aware traversal on the unpartitioned graph of configs[{CONFIG_INDEX[name]}]",
                       "n": g.n_rows, "nnz": g.nnz, "targets": int(w.targets_global.size)},
            "cells": cells}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg1", choices=sorted(CONFIG_INDEX))
    ap.add_argument("--others", default=None, metavar="cfgA,cfgB",
                    help="workloads reported under the `others` key of the same JSON line (default: cfg2,cfg3,cfg4 when the "
                         "headline is cfg1 and no special mode is on; each with at most 5 timed steps and a smaller CPU sample)")
    ap.add_argument("--no-others", action="store_true")
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
                    help="enqueue the weight-gradient products on the step's stream instead of a second one (then every "
                         "call_ms entry is that call alone on the GPU)")
    ap.add_argument("--fused", action="store_true",
                    help="GraphSAGE layers of a shape gnn_fused_layer_fwd takes run aggregation and feature transform as one kernel "
                         "(the aggregate never leaves the chip); off by default")
    ap.add_argument("--chain-rule-order", action="store_true",
                    help="backward pass: input gradients per half and an accumulating aggregation (the order the chain rule gives) "
                         "instead of one product from the aggregated output gradient")
    ap.add_argument("--layer-sampling", default=None, metavar="RULE:PARAM[:SEED]",
                    help="layer-wise sampling as per-layer edge masks, rebuilt every step: fanout:F (neighbours kept per "
                         "row and layer) or dropedge:P (every edge kept with probability P per layer); off by default")
    ap.add_argument("--res-layers", type=int, default=0, metavar="L",
                    help="run the deep residual GraphSAGE (ResSAGE+) with L layers on the workload's graph instead of its own "
                         "model (GraphSAGE workloads); --res-hidden: its hidden width (default: the workload's); "
                         "--recompute: activation recomputation")
    ap.add_argument("--res-hidden", type=int, default=0)
    ap.add_argument("--recompute", action="store_true")
    ap.add_argument("--eas", default=None, metavar="H:F[:RULE],...",
                    help="time the expansion-aware traversal (hops H, fanout F, rule degree|hash) and the extraction of its "
                         "sub-graph on the workload's unpartitioned graph, one JSON line with a record per cell")
    ap.add_argument("--pmc-probe", default=None, metavar="MANIFEST.json",
                    help="counter probe for rocprofv3 --pmc runs (driven by bench_counters.py): the dominant aggregation, its "
                         "layer's feature transforms, set expansion, sampling and a plain copy, each from a thread of its own")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding or collectives are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.pmc_probe:
        return pmc_probe(args, args.workload, args.pmc_probe)
    if args.eas:
        print(json.dumps(eas_bench(args, args.workload)))
        return
    special = bool(args.res_layers or args.layer_sampling or args.host_partition or args.aggregate_first or
                   args.weights_first_all or args.scale != 1.0 or args.fused or args.chain_rule_order)
    others = []
    if not args.no_others:
        if args.others:
            others = [o for o in args.others.split(",") if o]
        elif args.workload == "cfg1" and not special:
            others = ["cfg2", "cfg3", "cfg4"]
    out = run_workload(args, args.workload, args.steps, args.warmup, 0.0 if args.no_cpu_baseline else 2.0e11)
    if others:
        out["others"] = {}
        for o in others:
            assert o in CONFIG_INDEX and o != args.workload
            r = run_workload(args, o, min(args.steps, 5), min(args.warmup, 2), 0.0 if args.no_cpu_baseline else 5.0e10)
            r.pop("call_ms", None)
            out["others"][o] = r
    print(json.dumps(out))


def bench_res_model(args, w, part, sampled_graph, dtype, steps, warmup):
    """The deep residual GraphSAGE on the workload's partition (host-built numbering unless the partition was sampled
    on the GPU): same metric, the forward aggregation of a middle layer as the dominant call."""
    import torch
    import graphgen as gg
    import paper_2311_06837_amd as P
    assert w.model == "sage" and args.res_layers >= 2
    L, hid = args.res_layers, (args.res_hidden or w.dims[1])
    dims = [w.dims[0]] + [hid] * (L - 1) + [w.dims[-1]]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    # the partition's halo was cut for the workload's own depth: deeper models see the same vertices (the late active
    # sets are the whole partition, as in configs[3])
    es = 4 if dtype == torch.float32 else 2
    need = part.graph.n_rows * P.row_stride(hid, dtype) * es * (L * (1 if args.recompute else 3) + 8)
    have = torch.cuda.get_device_properties(0).total_memory
    if need > 0.9 * have:       # say so instead of driving the allocator into the wall
        return {"metric": "aggregated_edges_per_sec", "value": None, "unit": "edges/s", "n_gpus": 1,
                "config": {"workload": f"deep residual GraphSAGE (ResSAGE+), {L} layers, hidden {hid}, on the partition of "
                                       f"configs[{CONFIG_INDEX[args.workload]}]", "layers": L, "hidden": hid,
                           "recompute": bool(args.recompute), "n_local": part.graph.n_rows},
                "does_not_fit": {"needed_bytes": int(need), "device_bytes": int(have)}}
    G = sampled_graph if sampled_graph is not None else P.Graph.from_numpy(part.graph.row_ptr, part.graph.col_idx)
    params = [{k: dev(v) for k, v in p.items()} for p in gg.res_layer_weights(dims, w.seed)]
    model = P.ResSAGEPlus(G, G, dev(part.targets), params, dtype=dtype, recompute=args.recompute,
                          prefix_numbered=sampled_graph is not None)
    n = part.graph.n_rows
    model.set_input(dev(gg.features(n, w.dims[0], w.seed, ld=P.row_stride(w.dims[0], dtype))).to(dtype))
    labels = dev(gg.labels(len(part.targets), w.dims[-1], w.seed))
    for _ in range(warmup):
        model.step(labels)
    torch.cuda.synchronize()
    model.trace = []
    t0 = time.perf_counter()
    for _ in range(steps):
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
    dom = max(range(2, L + 1), key=lambda l: call_ms.get(f"spmm_fwd_{l}", 0.0))
    nd = model.n_rows_of_layer(dom)
    alg_bytes = edges[dom]["fwd"] * (4 + hid * es) + nd * (8 + hid * es)
    t_dom = (call_ms.get(f"spmm_fwd_{dom}") or call_ms[f"fused_fwd_{dom}"]) * 1e-3
    group = lambda pre: sum(v for k, v in call_ms.items() if k.startswith(pre))
    return {
        "metric": "aggregated_edges_per_sec", "value": total_edges / (wall / steps), "unit": "edges/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"deep residual GraphSAGE (ResSAGE+), {L} layers, hidden {hid}, on the partition of "
                               f"configs[{CONFIG_INDEX[args.workload]}]: {gg.WORKLOADS[args.workload]}",
                   "scale": args.scale, "n_local": n, "nnz_local": part.graph.nnz, "targets": len(part.targets),
                   "layers": L, "hidden": hid, "recompute": bool(args.recompute)},
        "epoch_ms": sum(v for k, v in call_ms.items() if k != "active_sets"),
        "activation_bytes": model.activation_bytes(),
        "aggregated_edges_per_step": total_edges,
        "ms_by_kind": {"spmm_fwd": group("spmm_fwd"), "spmm_bwd": group("spmm_bwd"), "linear_fwd": group("linear_fwd"),
                       "linear_bwd": group("linear_bwd"), "layer_norm_fwd": group("ln_fwd"), "layer_norm_bwd": group("ln_bwd"),
                       "residual": group("residual"), "active_sets": call_ms.get("active_sets"), "softmax_ce": call_ms.get("softmax_ce")},
        "roofline": res_roofline(f"spmm_rows_kernel; gnn_masked_spmm_fwd, layer {dom}, F={hid}", alg_bytes,
                                 edges[dom]["fwd"] * 4 + model.n_rows_of_layer(dom - 1) * hid * es + nd * (8 + hid * es), t_dom),
        "cpu_baseline": None,
    }


def res_roofline(kernel, gather_bytes, compulsory_bytes, t_s):
    """No counter reading exists for these shapes.  The gather model (every neighbour row from memory) is what the
    launch is priced on while it stays below the HBM peak; wide rows are re-read from L2 often enough that the model
    overshoots the peak - then only the lower bound (every operand once) can be claimed."""
    g = gather_bytes / t_s / 1e9
    over = g > HBM_PEAK_GBS
    ach = compulsory_bytes / t_s / 1e9 if over else g
    return {"kernel": kernel, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "frac_basis": "compulsory bytes (the gather model exceeds the HBM peak: neighbour rows come from L2)" if over
                          else "gather model",
            "traffic": None, "bytes_per_launch": compulsory_bytes if over else gather_bytes, "launch_ms": t_s * 1e3,
            "gather_GBs": g, "compulsory_GBs": compulsory_bytes / t_s / 1e9}


def cpu_baseline(part, w, params, H0, rows_all, flops_budget):
    """The oracle as it stands, on this machine's host cores: layer-1 masked aggregation + feature transform
    (forward) on a seeded sample of the layer's rows (rows_all, local ids of the host partition), sized by a budget of
    fp64 multiply-adds of aggregation (2e11: roughly 10-20 s on 16 cores with the gathers)."""
    import oracle
    K, N = w.dims[0], w.dims[1]
    deg = np.diff(part.graph.row_ptr)[rows_all].astype(np.int64)
    budget = flops_budget / max(K, 1)
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
