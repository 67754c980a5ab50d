"""Host-side logic of bench.py that needs no GPU: the HBM-traffic record (written from rocprofv3
counter tables, reported only for the kernel sources it was measured on) and the byte / flop counts
the roofline fractions are formed from."""
import csv
import json
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench          # noqa: E402
import workloads      # noqa: E402


def _counter_table(path, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for i, (name, value) in enumerate(rows):
            w.writerow([i, name, "X", value])


def test_traffic_record_is_scaled_by_the_calibration_copy_and_dropped_when_sources_change(tmp_path, monkeypatch):
    record = tmp_path / "hbm_traffic.json"
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(record))
    name = workloads.CONFIG_NAMES[1]
    T, row = 4096, 1024 * 2
    # the calibration copy (the largest k_rows dispatch) reads T rows + 8 T bytes and writes T rows + 4 T
    # bytes; let the read counter see half of that (as FETCH_SIZE does on this part) and the write counter all
    read_kib = (T * row + 8 * T) / 1024.0 / 2.0
    write_kib = (T * row + 4 * T) / 1024.0
    rows_k = "void up::k_rows<false>(char const*, char*)"
    fetch = [(rows_k, read_kib), (rows_k, 100.0), (rows_k, 300.0), ("void up::k_sweep<1, 16, false, 128>(up::SweepArgs)", 1000.0),
             ("void up::k_sweep<2, 16, false, 128>(up::SweepArgs)", 500.0), ("up::k_finish(up::SweepArgs, int)", 20.0),
             ("void up::k_combine<8>(int const*)", 10.0), ("up::k_plan(int const*)", 1.0)]
    write = [(rows_k, write_kib), (rows_k, 200.0), (rows_k, 600.0), ("void up::k_sweep<1, 16, false, 128>(up::SweepArgs)", 50.0),
             ("void up::k_sweep<2, 16, false, 128>(up::SweepArgs)", 8.0), ("up::k_finish(up::SweepArgs, int)", 2.0),
             ("void up::k_combine<8>(int const*)", 0.5), ("up::k_plan(int const*)", 0.0)]
    _counter_table(tmp_path / "f.csv", fetch)
    _counter_table(tmp_path / "w.csv", write)
    bench.record_traffic(1, str(tmp_path / "f.csv"), str(tmp_path / "w.csv"), "profiles/some_summary.md")
    rec = json.load(open(record))
    assert rec["csrc_sha256"] == bench.csrc_digest()
    assert rec["scale"][name] == {"FETCH_SIZE": 2.0, "WRITE_SIZE": 1.0}
    ent = rec["bytes"][name]
    assert ent["row_stats"] == round((1000.0 * 2 + 50.0) * 1024)
    assert ent["sweep_select"] == round((500.0 * 2 + 8.0 + 20.0 * 2 + 2.0) * 1024)      # pass 2 and k_finish together
    assert ent["merge_stats"] == round((10.0 * 2 + 0.5) * 1024)
    assert ent["gather"] == round((200.0 * 2 + 400.0) * 1024)                            # the calibration copy left out
    got, prov = bench.measured_traffic(name, "gather")
    assert got == ent["gather"] and prov["stale"] is False and prov["profile"] == "profiles/some_summary.md"
    # a record taken on other sources is not reported
    rec["csrc_sha256"] = "0" * 64
    json.dump(rec, open(record, "w"))
    got, prov = bench.measured_traffic(name, "gather")
    assert got is None and prov["stale"] is True
    # ... and a new measurement does not keep the old workloads' figures next to its own
    rec["bytes"]["another_workload"] = {"gather": 1}
    json.dump(rec, open(record, "w"))
    bench.record_traffic(1, str(tmp_path / "f.csv"), str(tmp_path / "w.csv"), "profiles/some_summary.md")
    assert list(json.load(open(record))["bytes"]) == [name]
    assert bench.measured_traffic("no_such_workload", "gather") == (None, None)


def test_committed_traffic_record_matches_the_sources_in_the_tree():
    """The record that bench.py reports from was measured on the kernel sources as they stand (else the
    benchmark line carries no traffic figure)."""
    rec = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
    assert rec["csrc_sha256"] == bench.csrc_digest()
    for name, path in rec["profiles"].items():
        assert os.path.exists(os.path.join(ROOT, path)), path
        assert set(rec["bytes"][name]) == {"row_stats", "merge_stats", "sweep_select", "gather"}


def test_algorithmic_bytes_and_flops_of_the_headline_workload():
    """Config 4 by hand: K once (8 kv heads x 128 x 2 B per token) + a score per token; per kept row the
    hidden row in and out (5120 x 2 B each) + 12 B of index and positions; the query window of 128 rows
    x 40 heads x 256 B.  One Q.K^T pass: 2 x 128 x 131072 x 128 x 40 flops."""
    w = workloads.make_config(4, hidden_dim=8)
    w.hidden_dim = 5120
    kept = 32960
    assert bench.algorithmic_bytes(w, kept) == 131072 * (2048 + 4) + kept * (2 * 10240 + 12) + 128 * 40 * 256 == 945686784
    assert bench.product_flops(w) == 2 * 128 * 131072 * 128 * 40
