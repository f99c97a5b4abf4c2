#!/usr/bin/env python3
"""Benchmark of the MI355X hot path: effective HBM GB/s of the K-way
aggregate + apply (and of the other calls) on seeded synthetic updates.

One "step" is one call of the workload's entry point over one batch of K
updates that are already resident in HBM.  The default workload is the
ResNet-50-sized configuration (K = 16 binary32 updates of 25,557,032 elements,
SGD with momentum); `--workload cfg1..cfg5` selects another one.  "Effective"
bandwidth is ALGORITHMIC bytes (each update once, model and momentum read and
written once) divided by time, so redundant traffic lowers it.

Prints one JSON line.  Besides the headline it carries `dense_roofline`, the
fraction of the 8 TB/s peak of every dense configuration with the smallest one
named (`min_dense_frac`), and `rows`, every other call on its configuration.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_SOURCES = ["paper_1907_00434_amd/csrc/dense.hip", "paper_1907_00434_amd/csrc/sparse.hip"]


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--no-rows", action="store_true",
                    help="skip the extra per-call measurements of the other configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--permute-ids", action="store_true",
                    help="cfg5: word ids are a seeded permutation of the Zipf ranks")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy a few times (reference for "
                         "hardware byte counters)")
    return ap.parse_args()


def kernel_source_digest():
    """sha256 over the kernel sources: ties a counter measurement to the code it
    was taken on."""
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload):
    """HBM bytes per launch from the hardware-counter summary kept under
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy), or None when
    there is none for this workload or the kernels have changed since."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    if rec.get("kernel_source_sha256") != kernel_source_digest():
        return None
    return rec.get("traffic_bytes", {}).get(workload)


class DenseJob:
    """Device-resident inputs of one dense configuration and its entry point."""

    def __init__(self, cfg, mlf, W, torch, call=None):
        self.cfg, self.mlf = cfg, mlf
        self.call = call or cfg.call
        self.d = W.dense_inputs(cfg, "cuda:0")
        d = self.d
        self.out = None
        if self.call == "aggregate":
            self.out = torch.empty(cfg.n, device="cuda:0")
        with_h = 16 if d["momentum"] is not None else 8
        state = {"aggregate": 4, "apply_ordered": with_h, "aggregate_apply": with_h,
                 "apply_grouped": with_h, "apply_grouped_norms": with_h,
                 "apply_grouped_update_norms": with_h}[self.call]
        if self.call in ("apply_grouped_norms", "apply_grouped_update_norms"):
            self.norms = torch.zeros(2, dtype=torch.float64, device="cuda:0")
            self.update_norms = torch.zeros(len(d["order"]), dtype=torch.float64, device="cuda:0")
            nbytes = max(mlf.mlf_norms_workspace_bytes(cfg.n), mlf.mlf_update_norms_workspace_bytes(cfg.n))
            self.norm_ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        # a scheduled batch: a quarter of the updates forwarded directly, the rest
        # in three aggregated groups (Sec. 5.2 of the paper)
        M = len(d["order"])
        self.group_len = [1] * (M // 4) + [(M - M // 4) // 3] * 2 + [M - M // 4 - 2 * ((M - M // 4) // 3)]
        self.bytes = (cfg.in_bytes * len(d["order"]) + state) * cfg.n
        self.units = len(d["order"]) * cfg.n          # update elements consumed per step
        self.kernel = "dense_kernel"
        self.state_bytes = (state - 4 if self.call == "aggregate" else state) // 2 * cfg.n

    def step(self):
        d, m = self.d, self.mlf
        if self.call == "aggregate":
            m.mlf_aggregate(d["updates"], d["order"], d["weights"], self.out)
        elif self.call == "apply_ordered":
            m.mlf_apply_ordered(d["model"], d["momentum"], d["updates"], d["order"], d["lr"], d["mu"])
        elif self.call == "apply_grouped":
            m.mlf_apply_grouped(d["model"], d["momentum"], d["updates"], d["order"], d["weights"],
                                self.group_len, d["lr"], d["mu"])
        elif self.call == "apply_grouped_norms":
            m.mlf_apply_grouped_norms(d["model"], d["momentum"], d["updates"], d["order"],
                                      d["weights"], self.group_len, d["lr"], d["mu"], self.norms,
                                      self.norm_ws)
        elif self.call == "apply_grouped_update_norms":
            m.mlf_apply_grouped_update_norms(d["model"], d["momentum"], d["updates"], d["order"],
                                             d["weights"], self.group_len, d["lr"], d["mu"], self.norms,
                                             self.update_norms, self.norm_ws)
        else:
            m.mlf_aggregate_apply(d["model"], d["momentum"], None, d["updates"], d["order"],
                                  d["weights"], d["lr"], d["mu"])


class SparseJob:
    """cfg5.  Algorithmic bytes: 12 per triple, one 4-byte read and write of
    every DISTINCT cell the batch touches, the totals read and written once.
    The distinct cells are counted on the device here (one flag per cell, set
    by the valid triples); the CPU-baseline leg recounts them with the oracle."""

    def __init__(self, cfg, mlf, W, torch, permute_ids=False):
        self.cfg, self.mlf = cfg, mlf
        self.call = "sparse_scatter_add" + (" (permuted word ids)" if permute_ids else "")
        self.d = W.sparse_inputs(cfg, "cuda:0", permute_ids=permute_ids)
        total = cfg.K * cfg.m
        nbytes = mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, total)
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda:0")
        seen = torch.zeros(cfg.V * cfg.T, dtype=torch.bool, device="cuda:0")
        for t in self.d["triples"]:
            ok = (t[:, 0] >= 0) & (t[:, 0] < cfg.V) & (t[:, 1] >= 0) & (t[:, 1] < cfg.T)
            seen[(t[ok, 0].long() * cfg.T + t[ok, 1].long())] = True
        self.distinct_cells = int(seen.sum().item())
        self.distinct_source = "device (flags over the flat indices of the valid triples)"
        del seen
        self.bytes = cfg.algorithmic_bytes(self.distinct_cells)
        self.bytes_per_triple_rule = 20 * total      # 12 B + one 4-byte read-modify-write per triple
        self.units = total                             # triples per step
        self.kernel = "scatter"

    def step(self):
        d = self.d
        self.mlf.mlf_sparse_scatter_add(d["counts"], d["totals"], self.cfg.V, self.cfg.T,
                                        d["triples"], workspace=self.ws)


class DivergenceJob:
    """Exact server-replica distance of two AlexNet-sized models."""

    def __init__(self, cfg, mlf, torch):
        self.cfg, self.mlf, self.call = cfg, mlf, "divergence"
        g = torch.Generator(device="cuda:0")
        g.manual_seed(cfg.seed)
        self.a = torch.randn(cfg.n, generator=g, device="cuda:0")
        self.b = self.a + torch.randn(cfg.n, generator=g, device="cuda:0") * 1e-3
        self.dist = torch.zeros(1, dtype=torch.float64, device="cuda:0")
        self.ws = torch.empty(mlf.mlf_norms_workspace_bytes(cfg.n), dtype=torch.uint8, device="cuda:0")
        self.bytes, self.units = 8 * cfg.n, cfg.n

    def step(self):
        self.mlf.mlf_divergence(self.a, self.b, self.dist, self.ws)


class TrafficMixJob:
    """A reference for cfg4's traffic mix: mlf_aggregate of three binary32 updates
    of cfg4's length reads 12 bytes and writes 4 per element (a quarter of the
    traffic is stores, as in cfg4's 16 read + 16 read-modify-write bytes), with
    128-bit loads throughout and nothing read back."""

    def __init__(self, cfg, mlf, torch):
        self.cfg, self.mlf, self.call = cfg, mlf, "aggregate of 3 binary32 updates (traffic-mix reference)"
        g = torch.Generator(device="cuda:0")
        g.manual_seed(cfg.seed)
        self.ups = [torch.randn(cfg.n, generator=g, device="cuda:0") for _ in range(3)]
        self.out = torch.empty(cfg.n, device="cuda:0")
        self.bytes, self.units = 16 * cfg.n, 3 * cfg.n

    def step(self):
        self.mlf.mlf_aggregate(self.ups, [0, 1, 2], None, self.out)


class DenseDeltaJob:
    """The LDA update as 8 dense int32 delta matrices (2 % of the cells non-zero).
    Bytes: every delta matrix once, and one read and one write of the cells
    whose summed delta is not zero (a cell whose deltas cancel needs neither)."""

    def __init__(self, cfg, mlf, torch, K=8):
        self.cfg, self.mlf, self.call = cfg, mlf, "counts_add_dense"
        g = torch.Generator(device="cuda:0")
        g.manual_seed(cfg.seed)
        cells = cfg.V * cfg.T
        self.mats = []
        for _ in range(K):
            vals = torch.randint(-5, 6, (cells,), generator=g, device="cuda:0", dtype=torch.int32)
            keep = torch.rand(cells, generator=g, device="cuda:0") < 0.02
            self.mats.append(torch.where(keep, vals, torch.zeros_like(vals)))
        total = torch.zeros(cells, dtype=torch.int32, device="cuda:0")
        for m_ in self.mats:
            total += m_
        self.changed_cells = int((total != 0).sum().item())
        del total
        self.counts = torch.zeros(cells, dtype=torch.int32, device="cuda:0")
        self.totals = torch.zeros(cfg.T, dtype=torch.int32, device="cuda:0")
        self.bytes = 4 * K * cells + 8 * self.changed_cells + 8 * cfg.T
        self.bytes_nominal = (4 * K + 8) * cells
        self.units = K * cells

    def step(self):
        self.mlf.mlf_counts_add_dense(self.counts, self.totals, self.cfg.V, self.cfg.T, self.mats)


def time_steps(torch, job, steps, warmup):
    """Wall time and HIP-event time (on the launch stream) of `steps` steps."""
    for _ in range(warmup):
        job.step()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        job.step()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    event_ms = start.elapsed_time(stop) / steps
    return wall_ms, event_ms


def time_each(torch, job, steps, between=None):
    """Median and minimum HIP-event time of single steps; `between` runs before
    each timed step (outside its events)."""
    pairs = []
    for _ in range(steps):
        if between is not None:
            between()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        job.step()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in pairs)
    return ms[len(ms) // 2], ms[0]


def cpu_baseline(job, W, torch):
    """The oracle, as it stands, on the WHOLE configuration of the headline
    workload: repeated for a few seconds with all host threads, then with one."""
    import numpy as np

    import oracle
    threads = min(16, len(os.sched_getaffinity(0)))
    cfg, d = job.cfg, job.d
    extra = {}
    if job.call.startswith("sparse_scatter_add"):
        tr = [W.to_host(t) for t in d["triples"]]
        counts = np.zeros(cfg.V * cfg.T, dtype=np.int32)
        totals = np.zeros(cfg.T, dtype=np.int32)
        n_units = sum(t.shape[0] for t in tr)
        distinct = oracle.touched_cells(cfg.V, cfg.T, tr, threads=threads)
        extra = {"distinct_cells": distinct, "distinct_cells_agree_with_device": distinct == job.distinct_cells}
        nbytes = 12 * n_units + 8 * distinct + 8 * cfg.T
        sample = f"the whole configuration: {n_units:,} triples into the {cfg.V}x{cfg.T} matrix"

        def run(th):
            oracle.scatter_add(counts, totals, cfg.V, cfg.T, tr, threads=th)
    else:
        ups = [W.to_host(u) for u in d["updates"]]
        w = W.to_host(d["model"])
        h = W.to_host(d["momentum"]) if d["momentum"] is not None else None
        n_units = len(d["order"]) * cfg.n
        nbytes = job.bytes
        sample = f"the whole configuration: all {cfg.n:,} elements of all {cfg.K} updates"

        def run(th):
            if job.call == "apply_ordered":
                oracle.apply_ordered(w, h, ups, d["order"], d["lr"], d["mu"], threads=th)
            elif job.call == "aggregate":
                oracle.aggregate(ups, d["order"], d["weights"], threads=th)
            else:
                oracle.aggregate_apply(w, h, ups, d["order"], d["weights"], d["lr"], d["mu"],
                                       threads=th)

    def timed(th, budget_s):
        run(th)                                        # touch pages once
        reps, t0 = 0, time.perf_counter()
        while True:
            run(th)
            reps += 1
            el = time.perf_counter() - t0
            if el >= budget_s or reps >= 50:
                return el / reps, reps

    t_multi, reps_multi = timed(threads, 6.0)
    t_single, reps_single = timed(1, 6.0)
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
    except OSError:
        pass
    return {
        "value": round(nbytes / t_multi / 1e9, 3), "unit": "GB/s", "cores": threads,
        "kind": "oracle", "sample": sample, "repetitions": reps_multi,
        "seconds_per_repetition": round(t_multi, 4),
        "elements_per_s": round(n_units / t_multi, 1),
        "single_thread_value": round(nbytes / t_single / 1e9, 3),
        "single_thread_repetitions": reps_single,
        "cpu_model": model, "host_cpus": os.cpu_count(), **extra,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU (no sharding, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_1907_00434_amd as mlf
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)

    def make(name, call=None):
        cfg = W.CONFIGS[name]
        if call == "divergence":
            return DivergenceJob(cfg, mlf, torch)
        if call == "counts_add_dense":
            return DenseDeltaJob(cfg, mlf, torch)
        if call == "traffic_mix":
            return TrafficMixJob(cfg, mlf, torch)
        if isinstance(cfg, W.SparseConfig):
            return SparseJob(cfg, mlf, W, torch, permute_ids=(call == "permuted" or args.permute_ids))
        return DenseJob(cfg, mlf, W, torch, call)

    job = make(args.workload)
    wall_ms, event_ms = time_steps(torch, job, args.steps, args.warmup)
    gbs = job.bytes / (wall_ms * 1e-3) / 1e9
    achieved = job.bytes / (event_ms * 1e-3) / 1e9
    cfg = job.cfg
    line = {
        "metric": "effective HBM GB/s (and % of peak) for K-way aggregate+apply; elements/s",
        "value": round(gbs, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if args.workload == "cfg5" or cfg.dtype == "f32" else "f32 (bf16 inputs)",
        "data": "synthetic",
        "percent_of_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "elements_per_s": round(job.units / (wall_ms * 1e-3), 1),
        "config": {
            "workload": f"{args.workload}: {job.call}",
            "K": cfg.K,
            **({"V": cfg.V, "T": cfg.T, "triples": cfg.K * cfg.m,
                "distinct_cells_touched": job.distinct_cells,
                "distinct_cells_counted_on": job.distinct_source,
                "bytes_at_20_per_triple (not used)": job.bytes_per_triple_rule}
               if args.workload == "cfg5"
               else {"n": cfg.n, "update_dtype": cfg.dtype, "momentum": cfg.momentum,
                     "lr": cfg.lr, "mu": cfg.mu}),
            "algorithmic_bytes_per_step": job.bytes,
        },
        "roofline": {
            "bound": "hbm",
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic(args.workload),
            "kernel": job.kernel,
            "avg_launch_ms": round(event_ms, 5),
        },
    }
    if args.workload == "cfg5":
        line["dtype"] = "int32"
    elif job.state_bytes <= 256 << 20:
        line["roofline"]["note"] = ("model and momentum (%.0f MB) stay in the 256 MiB memory-side cache between the "
                                    "back-to-back timed calls; the row with the caches evicted before each launch "
                                    "is the HBM-only figure" % (job.state_bytes / 1e6))

    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(job, W, torch)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if not args.no_rows:
        del job
        torch.cuda.empty_cache()
        rows = {}
        dense_frac = {}
        extension_frac = {}      # the variants that also return one norm per update
        plan = [("cfg1", None), ("cfg2", "aggregate"), ("cfg2", None), ("cfg3", None),
                ("cfg3", "apply_grouped"), ("cfg2", "apply_grouped"),
                ("cfg2", "apply_grouped_norms"), ("cfg3", "apply_grouped_norms"),
                ("cfg2", "apply_grouped_update_norms"), ("cfg3", "apply_grouped_update_norms"),
                ("cfg3", "divergence"), ("cfg4", None), ("cfg4", "traffic_mix"), ("cfg5", None), ("cfg5", "permuted"), ("cfg5", "counts_add_dense")]
        for name, call in plan:
            j = make(name, call)
            _, ev = time_steps(torch, j, 20, 3)
            key = f"{name}:{j.call}"
            med, best = time_each(torch, j, 20)
            rows[key] = {"ms": round(ev, 5), "median_ms": round(med, 5), "min_ms": round(best, 5),
                         "algorithmic_bytes": j.bytes,
                         "GB/s": round(j.bytes / ev / 1e6, 1),
                         "frac_of_peak": round(j.bytes / ev / 1e6 / HBM_PEAK_GBS, 4),
                         "units_per_s": round(j.units / (ev * 1e-3), 1)}
            if isinstance(j, SparseJob):
                rows[key]["distinct_cells_touched"] = j.distinct_cells
                rows[key]["GB/s_at_20_bytes_per_triple"] = round(j.bytes_per_triple_rule / ev / 1e6, 1)
            if isinstance(j, DenseDeltaJob):
                rows[key]["cells_with_nonzero_sum"] = j.changed_cells
                rows[key]["GB/s_at_nominal_bytes (every cell read and written)"] = round(j.bytes_nominal / ev / 1e6, 1)
            if isinstance(j, DenseJob) and name != "cfg1":
                if j.call.endswith("update_norms"):
                    extension_frac[key] = rows[key]["frac_of_peak"]
                else:
                    dense_frac[key] = rows[key]["frac_of_peak"]
            if name in ("cfg1", "cfg2") and call is None:
                # The state of cfg1 / cfg2 fits the caches: also time the call after a
                # read-only pass over 2 GiB, which evicts L2 and the memory-side cache
                # and leaves no dirty lines behind for the timed call to write back
                # (the HBM-only figure).
                thrash = torch.zeros(1 << 29, dtype=torch.float32, device="cuda:0")
                med, best = time_each(torch, j, 20, between=lambda: thrash.sum())
                cold = key + " (caches evicted before each launch)"
                rows[cold] = {
                    "median_ms": round(med, 5), "min_ms": round(best, 5),
                    "GB/s": round(j.bytes / med / 1e6, 1),
                    "frac_of_peak": round(j.bytes / med / 1e6 / HBM_PEAK_GBS, 4)}
                if name == "cfg2":
                    dense_frac[cold] = rows[cold]["frac_of_peak"]
                del thrash
            if name == "cfg1":
                # Back-to-back calls from Python are launch-bound at this size;
                # recorded into a HIP graph (20 calls per replay) they are not.
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    j.step()
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for _ in range(20):
                        j.step()
                graph.replay()
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(10):
                    graph.replay()
                b.record()
                torch.cuda.synchronize()
                per_call = a.elapsed_time(b) / 200
                rows[key + " (HIP graph of 20 calls)"] = {
                    "ms": round(per_call, 5), "GB/s": round(j.bytes / per_call / 1e6, 1),
                    "frac_of_peak": round(j.bytes / per_call / 1e6 / HBM_PEAK_GBS, 4)}
                del graph
            del j
            torch.cuda.empty_cache()
        line["rows"] = rows
        weakest = min(dense_frac, key=dense_frac.get)
        line["dense_roofline"] = {
            "unit": "fraction of 8 TB/s, algorithmic bytes / HIP-event time of 20 back-to-back launches "
                    "(median single launch for the evicted-cache row)",
            "frac": dense_frac,
            "min_dense_frac": dense_frac[weakest],
            "min_dense_row": weakest,
            "per_update_norm_variants (binary64 work per update element on top of the pass; "
            "not counted in min_dense_frac)": extension_frac,
        }

    print(json.dumps(line))


if __name__ == "__main__":
    main()
