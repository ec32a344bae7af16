#!/usr/bin/env python3
"""Hardware-counter readings for bench.py, taken with rocprofv3 on the MI355X machine.

For every workload this runs `python3 bench.py --workload W --pmc-probe MANIFEST` under `rocprofv3 --pmc ...`, once per
counter pass (rocprofv3 does not split counters over passes; each pass stays inside the per-block limits), and
optionally once under `rocprofv3 --kernel-trace --stats` on the plain benchmark.  The probe issues each call of interest
from a thread of its own and writes the thread ids to the manifest, so the per-dispatch rows of rocprofv3's CSV are
attributed to calls by their Thread_Id column.  Results:

  <out>/counters_sidecar.json   per workload and call: counter sums per launch, scaled byte counts, kernel list; stamped
                                with the hash of the kernel sources (bench.source_sha) - copy it to profiles/, bench.py
                                reads it from there and ignores it when the sources have changed since
  <out>/counters_<W>.md         the same as a short text summary, with the full commands
  <out>/stats_<W>.md            per-kernel durations of the plain benchmark (with --stats)

Byte counts.  FETCH_SIZE / WRITE_SIZE are rocprofv3's derived counters (KiB per dispatch).  Both are scaled by what
they read for a plain copy of known size in the same pass (the probe's `copy_calibration` group: gnn_gather_rows with
the identity list, 1 GiB in, 1 GiB out).  The request-size pass (TCC_EA0_RDREQ_sum, _32B, _64B, _128B) gives the read
bytes without any scale: 32 n32 + 64 n64 + 128 n128.  These are requests from the L2s to the memory fabric; part of
them may be served by the last-level (Infinity) cache, so they bound the HBM traffic from above.

python bench_counters.py [--workloads cfg1,cfg2,cfg3,cfg4] [--out gpurun_out/counters] [--stats] [--passes bytes,req,sq]
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import signal
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PASSES = {
    "fetch": ["FETCH_SIZE"],
    "write": ["WRITE_SIZE", "TCC_HIT_sum", "TCC_MISS_sum"],
    "req": ["TCC_EA0_RDREQ_sum", "TCC_EA0_RDREQ_32B_sum", "TCC_EA0_RDREQ_64B_sum", "TCC_EA0_RDREQ_128B_sum"],
    "sq": ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_INSTS_VALU_MFMA_MOPS_F32",
           "SQ_WAVES", "SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE", "GRBM_GUI_ACTIVE"],
}
N_SIMD = 256 * 4       # MI355X: 256 compute units, 4 SIMDs each
N_XCC = 8              # GRBM_GUI_ACTIVE comes summed over the eight compute dies (16 "cycles" per ns on a long kernel), so
                       # the cycles of ONE die's clock are a eighth of it.  Cross-check: SQ_INSTS_VALU_MFMA_MOPS_BF16 * 512 flop /
                       # 32768 flop per 32x32x16 instruction * 32 cycles equals SQ_VALU_MFMA_BUSY_CYCLES to three digits.


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def run(cmd, env, limit_s, log_path):
    """One GPU step under a time limit of its own; the whole process group is killed at the limit."""
    log(f"[counters] {' '.join(cmd)}")
    with open(log_path, "w") as lf:
        p = subprocess.Popen(cmd, cwd=ROOT, env=env, stdout=lf, stderr=subprocess.STDOUT, start_new_session=True)
        try:
            rc = p.wait(timeout=limit_s)
        except subprocess.TimeoutExpired:
            os.killpg(p.pid, signal.SIGKILL)
            p.wait()
            rc = 124
    log(f"[counters]   -> rc {rc}")
    return rc


def read_pass(csv_dir, manifest):
    """-> {group: {"counters": {name: sum per launch}, "kernels": {kernel: {"per_launch": k, "avg_us": t, counters...}}}}"""
    files = glob.glob(os.path.join(csv_dir, "**", "*counter_collection.csv"), recursive=True)
    assert files, f"no counter_collection.csv under {csv_dir}"
    rows = [r for f in files for r in csv.DictReader(open(f))]
    by_tid = collections.defaultdict(list)
    for r in rows:
        by_tid[int(r["Thread_Id"])].append(r)
    out = {}
    for gname, ginfo in manifest["groups"].items():
        rs = by_tid.get(int(ginfo["thread_id"]), [])
        if not rs:
            raise RuntimeError(f"no dispatch of thread {ginfo['thread_id']} (group {gname}) in {csv_dir}: "
                               f"thread ids seen: {sorted(by_tid)[:8]}")
        rep = ginfo["repeats"]
        sums = collections.defaultdict(float)
        kern = collections.OrderedDict()
        seen = set()
        # a counter may come as one row per hardware instance (one per compute die): block counters are summed over the
        # instances, the clock-like GRBM_* counters take the largest instance (every die counts the same cycles)
        per = collections.OrderedDict()
        for r in rs:
            per.setdefault((r["Dispatch_Id"], r["Counter_Name"]), []).append(r)
        for (did, cname), lst in per.items():
            vals = [float(x["Counter_Value"]) for x in lst]
            val = max(vals) if cname.startswith("GRBM_") else sum(vals)
            r = lst[0]
            sums[cname] += val
            k = kern.setdefault(r["Kernel_Name"], {"dispatches": 0, "ns": 0.0, "counters": collections.defaultdict(float)})
            k["counters"][cname] += val
            if r["Dispatch_Id"] not in seen:
                seen.add(r["Dispatch_Id"])
                k["dispatches"] += 1
                k["ns"] += float(r["End_Timestamp"]) - float(r["Start_Timestamp"])
        out[gname] = {"counters": {c: v / rep for c, v in sums.items()},
                      "kernels": {kn: {"per_launch": k["dispatches"] / rep, "avg_us": k["ns"] / max(k["dispatches"], 1) / 1e3,
                                       "counters_per_dispatch": {c: v / max(k["dispatches"], 1) for c, v in k["counters"].items()}}
                                  for kn, k in kern.items()}}
    return out


def derive(groups, manifest):
    """Scaled byte counts and ratios per group, from the merged counters of all passes."""
    cal = groups.get("copy_calibration", {}).get("counters", {})
    ginfo = manifest["groups"]["copy_calibration"]
    fetch_scale = write_scale = None
    if cal.get("FETCH_SIZE"):
        fetch_scale = ginfo["bytes_read"] / (cal["FETCH_SIZE"] * 1024.0)
    if cal.get("WRITE_SIZE"):
        write_scale = ginfo["bytes_written"] / (cal["WRITE_SIZE"] * 1024.0)
    res = {}
    for g, d in groups.items():
        c = d["counters"]
        r = {"kernels": {k: {"per_launch": v["per_launch"], "avg_us": round(v["avg_us"], 2)} for k, v in d["kernels"].items()}}
        if "FETCH_SIZE" in c:
            r["fetch_size_KiB"] = c["FETCH_SIZE"]
        if "WRITE_SIZE" in c:
            r["write_size_KiB"] = c["WRITE_SIZE"]
        if "FETCH_SIZE" in c and "WRITE_SIZE" in c and fetch_scale and write_scale:
            r["fetch_scale"], r["write_scale"] = fetch_scale, write_scale
            r["write_bytes"] = c["WRITE_SIZE"] * 1024.0 * write_scale
            r["traffic_bytes"] = c["FETCH_SIZE"] * 1024.0 * fetch_scale + r["write_bytes"]
        if "TCC_EA0_RDREQ_sum" in c:
            n32, n64, n128 = c.get("TCC_EA0_RDREQ_32B_sum", 0.0), c.get("TCC_EA0_RDREQ_64B_sum", 0.0), c.get("TCC_EA0_RDREQ_128B_sum", 0.0)
            r["read_requests"] = {"all": c["TCC_EA0_RDREQ_sum"], "32B": n32, "64B": n64, "128B": n128}
            r["fetch_bytes_by_request_size"] = 32 * n32 + 64 * n64 + 128 * n128
        if "TCC_HIT_sum" in c:
            r["tcc_hit"], r["tcc_miss"] = c["TCC_HIT_sum"], c.get("TCC_MISS_sum", 0.0)
            tot = r["tcc_hit"] + r["tcc_miss"]
            r["l2_hit_rate"] = r["tcc_hit"] / tot if tot else None
        if "SQ_VALU_MFMA_BUSY_CYCLES" in c:
            # per kernel: busy cycles of the matrix pipes over (active cycles of the dispatch x SIMDs)
            per_k = {}
            for kn, kv in d["kernels"].items():
                cc = kv["counters_per_dispatch"]
                act = cc.get("GRBM_GUI_ACTIVE", 0.0)
                if act > 0 and "SQ_VALU_MFMA_BUSY_CYCLES" in cc:
                    per_k[kn] = {"mfma_busy": cc["SQ_VALU_MFMA_BUSY_CYCLES"] / (act / N_XCC * N_SIMD),
                                 "mfma_mops_bf16": cc.get("SQ_INSTS_VALU_MFMA_MOPS_BF16", 0.0),
                                 "mfma_mops_f32": cc.get("SQ_INSTS_VALU_MFMA_MOPS_F32", 0.0),
                                 "lds_bank_conflict_frac": (cc.get("SQ_LDS_BANK_CONFLICT", 0.0) / cc["SQ_LDS_IDX_ACTIVE"]
                                                            if cc.get("SQ_LDS_IDX_ACTIVE") else None),
                                 "lds_busy": (cc.get("SQ_LDS_IDX_ACTIVE", 0.0) / (act / N_XCC * 256) if cc.get("SQ_LDS_IDX_ACTIVE") else None),
                                 "waves": cc.get("SQ_WAVES", 0.0), "gui_active_cycles_one_die": act / N_XCC}
            r["sq_per_kernel"] = per_k
        res[g] = r
    return res


def write_md(path, wl, derived, commands, manifest):
    L = [f"# Hardware counters of the probed calls of {wl} (bench.py --pmc-probe; per launch, averaged over the probe's repeats)\n",
         f"Kernel sources: {manifest['source_sha']}; dominant layer {manifest['dominant_layer']}; shapes {json.dumps(manifest['shapes'])}\n",
         "Commands (each pass its own run, from the repository root on the MI355X box; bench_counters.py issues them):\n", "```"]
    L += commands
    L.append("```\n")
    for g, r in derived.items():
        L.append(f"## {g}\n")
        L.append("| kernel | dispatches per launch | avg us (under the counter run) |\n|---|---|---|")
        for k, v in r["kernels"].items():
            L.append(f"| `{k[:120]}` | {v['per_launch']:g} | {v['avg_us']:.1f} |")
        L.append("")
        for key in ("fetch_size_KiB", "write_size_KiB", "fetch_scale", "write_scale", "traffic_bytes", "fetch_bytes_by_request_size",
                    "write_bytes", "read_requests", "tcc_hit", "tcc_miss", "l2_hit_rate"):
            if key in r:
                v = r[key]
                L.append(f"* {key}: {json.dumps(v) if isinstance(v, dict) else (f'{v:.6g}' if isinstance(v, float) else v)}")
        for kn, kv in r.get("sq_per_kernel", {}).items():
            L.append(f"* `{kn[:100]}`: " + ", ".join(f"{a} {b:.4g}" for a, b in kv.items() if b is not None))
        L.append("")
    open(path, "w").write("\n".join(L) + "\n")


def stats_md(path, wl, stats_dir, cmd, bench_json):
    f = glob.glob(os.path.join(stats_dir, "**", "*kernel_stats.csv"), recursive=True)
    assert f, f"no kernel_stats.csv under {stats_dir}"
    rows = list(csv.DictReader(open(f[0])))
    L = [f"# rocprofv3 --kernel-trace --stats of the benchmark step of {wl}\n", "Command (from the repository root on the MI355X box):\n",
         "```", cmd, "```\n", "| kernel | calls | avg us | total ms | % |\n|---|---|---|---|---|"]
    for r in rows[:24]:
        L.append(f"| `{r['Name'][:120]}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {float(r['TotalDurationNs']) / 1e6:.2f} | "
                 f"{float(r['Percentage']):.2f} |")
    try:
        d = json.loads(open(bench_json).read().strip().splitlines()[-1])
        ro = d["roofline"]
        L.append("\nbench.py line of the same run (HIP events on the launch stream inside the timed steps):\n")
        L.append(f"* ms_per_step {d['ms_per_step']:.3f}, value {d['value']:.4e} {d['unit']}")
        L.append(f"* roofline: {ro['kernel']}: {ro['launch_ms']:.3f} ms per call, achieved {ro['achieved']:.0f} GB/s = {ro['frac']:.3f} of "
                 f"{ro['peak']:.0f} GB/s ({ro.get('frac_basis')}); gather model {ro.get('gather_GBs', 0):.0f} GB/s")
        L.append("* call_ms: " + json.dumps(d.get("call_ms")))
    except (OSError, ValueError, KeyError, IndexError) as e:
        L.append(f"\n(bench line not parsed: {e})")
    open(path, "w").write("\n".join(L) + "\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workloads", default="cfg1,cfg2,cfg3,cfg4")
    ap.add_argument("--out", default="gpurun_out/counters")
    ap.add_argument("--passes", default="fetch,write,req,sq")
    ap.add_argument("--stats", action="store_true", help="also one rocprofv3 --kernel-trace --stats run of the benchmark per workload")
    ap.add_argument("--limit", type=int, default=300, help="seconds per GPU step")
    args = ap.parse_args()
    import bench
    out = os.path.join(ROOT, args.out)
    os.makedirs(out, exist_ok=True)
    env = dict(os.environ)
    env.setdefault("GRAPHGEN_CACHE", "/tmp/graphgen_cache")
    env.setdefault("TMPDIR", "/tmp")
    sidecar = {"source_sha": bench.source_sha(), "made": time.strftime("%Y-%m-%d %H:%M:%S"), "workloads": {}}
    for wl in args.workloads.split(","):
        groups = {}
        commands = []
        manifest = None
        for pname in args.passes.split(","):
            d = os.path.join(out, f"{wl}_{pname}")
            man = os.path.join(out, f"{wl}_{pname}_manifest.json")
            cmd = ["rocprofv3", "--pmc", *PASSES[pname], "-d", os.path.relpath(d, ROOT), "-o", "p", "--output-format", "csv", "--",
                   "python3", "bench.py", "--workload", wl, "--pmc-probe", os.path.relpath(man, ROOT)]
            commands.append(" ".join(cmd))
            rc = run(cmd, env, args.limit, os.path.join(out, f"{wl}_{pname}.log"))
            if rc != 0:
                log(f"[counters] pass {pname} of {wl} failed (rc {rc}); stopping here")
                sys.exit(rc)
            manifest = json.load(open(man))
            assert manifest["source_sha"] == sidecar["source_sha"]
            for g, dd in read_pass(d, manifest).items():
                tgt = groups.setdefault(g, {"counters": {}, "kernels": {}})
                tgt["counters"].update(dd["counters"])
                for kn, kv in dd["kernels"].items():
                    t2 = tgt["kernels"].setdefault(kn, {"per_launch": kv["per_launch"], "avg_us": kv["avg_us"], "counters_per_dispatch": {}})
                    t2["counters_per_dispatch"].update(kv["counters_per_dispatch"])
        derived = derive(groups, manifest)
        derived_top = {"dominant_layer": manifest["dominant_layer"], "shapes": manifest["shapes"], **derived}
        sidecar["workloads"][wl] = derived_top
        write_md(os.path.join(out, f"counters_{wl}.md"), wl, derived, commands, manifest)
        json.dump(sidecar, open(os.path.join(out, "counters_sidecar.json"), "w"), indent=1)
        if args.stats:
            d = os.path.join(out, f"{wl}_stats")
            bj = os.path.join(out, f"{wl}_stats_bench.json")
            cmd = ["rocprofv3", "--kernel-trace", "--stats", "-d", os.path.relpath(d, ROOT), "-o", "bench", "--output-format", "csv", "--",
                   "python3", "bench.py", "--workload", wl, "--steps", "5", "--warmup", "2", "--no-others", "--no-cpu-baseline"]
            log_path = os.path.join(out, f"{wl}_stats.log")
            rc = run(cmd, env, args.limit, log_path)
            if rc != 0:
                sys.exit(rc)
            # the benchmark's JSON line is the last line of its stdout that starts with '{'
            lines = [ln for ln in open(log_path).read().splitlines() if ln.startswith("{")]
            open(bj, "w").write(lines[-1] if lines else "")
            stats_md(os.path.join(out, f"stats_{wl}.md"), wl, d, " ".join(cmd), bj)
    log(f"[counters] wrote {os.path.join(out, 'counters_sidecar.json')}")


if __name__ == "__main__":
    main()
