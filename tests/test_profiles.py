"""The machine-readable traffic file that bench.py reads (profiles/hbm_traffic.json)
and the table kept beside it (profiles/hbm_traffic_pmc.md) come from one run of
paper_1907_00434_amd.profile_summary and must say the same; the bytes the dense
kernels move must be their algorithmic bytes.  CPU only."""
import json
import os
import re

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
ROW = {"cfg1": "cfg1: aggregate+apply", "cfg2": "cfg2: aggregate+apply", "cfg3": "cfg3: ordered apply",
       "cfg4": "cfg4: aggregate+apply", "cfg5": "cfg5, word id = rank - 1"}


def table_rows():
    rows = []
    for line in open(os.path.join(PROFILES, "hbm_traffic_pmc.md")):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if line.startswith("|") and len(cells) == 8 and re.fullmatch(r"[0-9.]+", cells[5] or "x"):
            rows.append(cells)
    return rows


def test_traffic_file_and_table_agree():
    rec = json.load(open(os.path.join(PROFILES, "hbm_traffic.json")))
    rows = table_rows()
    assert set(rec["traffic_bytes"]) == set(ROW)
    for workload, nbytes in rec["traffic_bytes"].items():
        if workload == "cfg5":
            match = [r for r in rows if r[0] == "whole sparse call" and r[1] == ROW[workload]]
        else:
            match = [r for r in rows if r[1] == ROW[workload]]
        assert len(match) == 1, (workload, match)
        assert abs(float(match[0][5]) - nbytes / 1e6) <= 0.051, (workload, match[0][5], nbytes)
    assert re.fullmatch(r"[0-9a-f]{64}", rec["kernel_source_sha256"])


def test_dense_kernels_move_their_algorithmic_bytes():
    rec = json.load(open(os.path.join(PROFILES, "hbm_traffic.json")))["traffic_bytes"]
    for name in ("cfg2", "cfg3", "cfg4"):
        want = W.CONFIGS[name].algorithmic_bytes()
        assert abs(rec[name] / want - 1) < 0.005, (name, rec[name], want)


def test_bench_reads_the_file_only_for_the_kernels_it_was_taken_on():
    import bench
    rec = json.load(open(os.path.join(PROFILES, "hbm_traffic.json")))
    current = bench.kernel_source_digest() == rec["kernel_source_sha256"]
    got = bench.measured_traffic("cfg2")
    assert got == (rec["traffic_bytes"]["cfg2"] if current else None)
