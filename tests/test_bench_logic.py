"""Host logic of the measurement scripts, on the CPU: the roofline record of an aggregation call, the gate that ties
counter figures to the kernel sources they were measured on, and the parsing of a counter pass.  No GPU call is made:
bench.py and bench_counters.py import without one."""
import csv
import json
import os

import pytest

import bench
import bench_counters


# ---- roofline_of_call: `frac` is a fraction of the published HBM peak and never above 1 ----------------------------------

def _call(t_s, gather, compulsory, blocked, counters):
    return bench.roofline_of_call("k", "what", t_s, gather, compulsory, blocked, counters)


def test_one_launch_route_without_counters_uses_the_gather_model():
    r = _call(1e-3, 4e9, 1e9, False, None)
    assert r["frac_basis"] == "gather model"
    assert r["achieved"] == pytest.approx(4000.0) and r["frac"] == pytest.approx(0.5)
    assert r["traffic"] is None and r["traffic_GBs"] is None
    assert r["bytes_per_launch"] == 4e9 and r["launch_ms"] == pytest.approx(1.0)


def test_one_launch_route_is_capped_by_a_smaller_counter_reading():
    r = _call(1e-3, 4e9, 1e9, False, {"traffic_bytes": 2e9, "l2_hit_rate": 0.5})
    assert r["frac_basis"].startswith("counters")
    assert r["achieved"] == pytest.approx(2000.0) and r["frac"] == pytest.approx(0.25)
    assert r["traffic"] == 2e9 and r["l2_hit_rate"] == 0.5
    # a reading above the model does not raise the claim
    r = _call(1e-3, 4e9, 1e9, False, {"traffic_bytes": 5e9})
    assert r["frac_basis"] == "gather model" and r["achieved"] == pytest.approx(4000.0)


def test_a_gather_model_above_the_peak_falls_back_to_the_lower_bound():
    r = _call(1e-3, 16e9, 3e9, False, None)
    assert r["frac_basis"].startswith("compulsory")
    assert r["achieved"] == pytest.approx(3000.0) and r["frac"] <= 1.0
    assert r["gather_GBs"] == pytest.approx(16000.0)       # still reported, beside the claim


def test_column_blocked_route_claims_counter_bytes_else_the_floor():
    r = _call(2e-3, 40e9, 4e9, True, {"traffic_bytes": 10e9})
    assert r["frac_basis"].startswith("counters") and r["achieved"] == pytest.approx(5000.0)
    r = _call(2e-3, 40e9, 4e9, True, None)
    assert r["frac_basis"].startswith("compulsory") and r["achieved"] == pytest.approx(2000.0)
    assert r["frac_compulsory"] == pytest.approx(0.25)


@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("counters", [None, {"traffic_bytes": 3e9}])
@pytest.mark.parametrize("gather", [2e9, 7.9e9, 30e9])
def test_frac_never_exceeds_one_when_the_floor_fits(blocked, counters, gather):
    r = _call(1e-3, gather, 1.5e9, blocked, counters)
    assert 0.0 < r["frac"] <= 1.0
    assert r["frac"] == pytest.approx(r["achieved"] / bench.HBM_PEAK_GBS)
    assert r["peak"] == 8000.0 and r["unit"] == "GB/s" and r["bound"] == "hbm"


# ---- the sidecar is used only for the sources it was measured on ---------------------------------------------------------

def test_source_sha_is_stable_and_hex():
    a, b = bench.source_sha(), bench.source_sha()
    assert a == b and len(a) == 16 and int(a, 16) >= 0


def test_sidecar_of_other_sources_is_ignored(tmp_path, monkeypatch):
    p = tmp_path / "sidecar.json"
    monkeypatch.setattr(bench, "SIDECAR", str(p))
    assert bench.load_sidecar() is None                              # no file
    p.write_text("{ not json")
    assert bench.load_sidecar() is None                              # unreadable
    p.write_text(json.dumps({"source_sha": "0" * 16, "workloads": {}}))
    assert bench.load_sidecar() is None                              # other build
    p.write_text(json.dumps({"source_sha": bench.source_sha(), "workloads": {"cfg1": 1}}))
    assert bench.load_sidecar()["workloads"] == {"cfg1": 1}


def test_committed_sidecar_matches_the_committed_sources():
    """The counter figures in the tree belong to the kernels in the tree (else the bench line reports them as null)."""
    if not os.path.exists(bench.SIDECAR):
        pytest.skip("no sidecar in the tree")
    d = json.load(open(bench.SIDECAR))
    assert d["source_sha"] == bench.source_sha()


def test_more_than_one_gpu_is_refused():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(bench.ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode == 2 and r.stdout == ""
    assert "exactly one GPU" in r.stderr


# ---- a counter pass: rows per hardware instance, several dispatches, repeats ---------------------------------------------

FIELDS = ["Thread_Id", "Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"]


def _write_pass(d, rows):
    os.makedirs(d, exist_ok=True)
    with open(os.path.join(d, "x_counter_collection.csv"), "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=FIELDS)
        w.writeheader()
        for r in rows:
            w.writerow(dict(zip(FIELDS, r)))


def test_read_pass_and_derive(tmp_path):
    manifest = {"groups": {
        "copy_calibration": {"thread_id": 11, "repeats": 2, "bytes_read": 2 * 1024 * 1024, "bytes_written": 1024 * 1024},
        "agg": {"thread_id": 12, "repeats": 1},
    }}
    rows = []
    # copy kernel: 2 dispatches (= 2 repeats), FETCH_SIZE split over two instances; the counter over-reads by 2x
    for did in (1, 2):
        rows += [(11, did, "copy", "FETCH_SIZE", 2048.0, 1000, 3000), (11, did, "copy", "FETCH_SIZE", 2048.0, 1000, 3000),
                 (11, did, "copy", "WRITE_SIZE", 1024.0, 1000, 3000)]
    # aggregation: one launch of two kernels; the clock counter takes the largest instance, block counters are summed
    rows += [(12, 3, "rows", "FETCH_SIZE", 4096.0, 0, 10000), (12, 3, "rows", "WRITE_SIZE", 512.0, 0, 10000),
             (12, 3, "rows", "GRBM_GUI_ACTIVE", 800.0, 0, 10000), (12, 3, "rows", "GRBM_GUI_ACTIVE", 640.0, 0, 10000),
             (12, 4, "tail", "FETCH_SIZE", 1024.0, 0, 2000), (12, 4, "tail", "WRITE_SIZE", 512.0, 0, 2000)]
    _write_pass(str(tmp_path / "p"), rows)
    groups = bench_counters.read_pass(str(tmp_path / "p"), manifest)
    cal = groups["copy_calibration"]
    assert cal["counters"]["FETCH_SIZE"] == pytest.approx(4096.0)        # per repeat, instances summed
    assert cal["kernels"]["copy"]["per_launch"] == 1 and cal["kernels"]["copy"]["avg_us"] == pytest.approx(2.0)
    agg = groups["agg"]
    assert agg["counters"]["FETCH_SIZE"] == pytest.approx(5120.0)
    assert agg["counters"]["GRBM_GUI_ACTIVE"] == pytest.approx(800.0)
    assert set(agg["kernels"]) == {"rows", "tail"} and agg["kernels"]["rows"]["avg_us"] == pytest.approx(10.0)

    d = bench_counters.derive(groups, manifest)
    # the copy moved 2 MiB in, 1 MiB out: the fetch counter read 4 MiB (scale 0.5), the write counter 1 MiB (scale 1)
    assert d["agg"]["fetch_scale"] == pytest.approx(0.5) and d["agg"]["write_scale"] == pytest.approx(1.0)
    assert d["agg"]["write_bytes"] == pytest.approx(1024.0 * 1024)
    assert d["agg"]["traffic_bytes"] == pytest.approx(5120 * 1024 * 0.5 + 1024 * 1024)
    assert d["copy_calibration"]["traffic_bytes"] == pytest.approx(3 * 1024 * 1024)


def test_read_pass_names_a_missing_group(tmp_path):
    manifest = {"groups": {"agg": {"thread_id": 99, "repeats": 1}}}
    _write_pass(str(tmp_path / "p"), [(12, 1, "k", "FETCH_SIZE", 1.0, 0, 1)])
    with pytest.raises(RuntimeError, match="group agg"):
        bench_counters.read_pass(str(tmp_path / "p"), manifest)
