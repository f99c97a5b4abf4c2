"""Turns rocprofv3 output directories into the short summaries kept under
profiles/ (text a few KB each; the raw CSV files stay where rocprofv3 wrote
them).  Runs on the CSV files alone, no GPU needed.

    python3 -m paper_1907_00434_amd.profile_summary trace   <trace dir> <bench.py output file>
    python3 -m paper_1907_00434_amd.profile_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir>
    python3 -m paper_1907_00434_amd.profile_summary counters <name> <title> <dir> [<dir> ...]

`trace` writes profiles/bench_default_kernel_trace.md from a
`rocprofv3 --kernel-trace --stats --output-format csv` run of bench.py and the
JSON line that run printed.  `traffic` writes profiles/hbm_traffic_pmc.md and
profiles/hbm_traffic.json (the file bench.py reads `roofline.traffic` from) from
two `--pmc` runs of profile_workloads, one counter each.  `counters` writes
profiles/<name>.md, one table of counters per kernel, from any number of `--pmc`
runs of profile_workloads.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
PROFILES = os.path.join(ROOT, "profiles")
KERNEL_SOURCES = ["paper_1907_00434_amd/csrc/dense.hip", "paper_1907_00434_amd/csrc/sparse.hip"]
SPARSE_KERNELS = ("clear_kernel", "sample_kernel", "plan_kernel", "coarse_partition_kernel",
                  "fine_partition_kernel", "accumulate_kernel")
KEY = ("Kernel name key: `dense_kernel<IN, OP, HAS_H, STREAM, NORMS, THREADS, VPT, HALF>`; OP 0 = aggregate, "
       "1 = aggregate+apply, 2 = ordered apply, 3 = grouped apply; STREAM 3 = model / momentum (or the aggregate's "
       "output) accessed with the no-reuse hint; NORMS 1 = the call's squared norms reduced in the same pass, "
       "2 = those and one per update; THREADS x VPT 64 x 1 = the shape for many updates on streamed state, launched "
       "with five workgroups per compute unit.")


def kernel_source_digest():
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def short(name):
    name = re.sub(r"^void ", "", name).replace("(anonymous namespace)::", "")
    m = re.match(r"([\w:]+(<[^()]*>)?)", name)
    return m.group(1) if m else name[:60]


def ours(name):
    return not any(x in name for x in ("at::", "rocprim", "hipcub", "elementwise", "distribution", "rocclr_fill"))


def find(directory, suffix):
    files = glob.glob(os.path.join(directory, "**", f"*{suffix}.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *{suffix}.csv under {directory}")
    return files[0]


def dense_workload(kernel):
    """(label, algorithmic bytes) of the dense kernels profile_workloads / bench.py launch."""
    import workloads as W
    m = re.match(r"dense_kernel()<(\w+), (\d), (true|false), (\d), (\d), (\d+), (\d+),", kernel)
    if not m:
        if kernel.startswith("divergence_kernel"):
            return "cfg3: exact divergence of two 61,100,840-element models", 8 * W.CONFIGS["cfg3"].n
        if kernel.startswith("dense_delta_kernel"):
            return "cfg5 shape: 8 dense int32 delta matrices 100,000 x 1,000 (nominal bytes)", 40 * 100_000 * 1_000
        return "", None
    kind, op, has_h, stream, norms = m.group(2), int(m.group(3)), m.group(4) == "true", int(m.group(5)), int(m.group(6))
    if kind == "F32" and op == 0 and norms == 0 and int(m.group(8)) == 2:
        # the only plain binary32 aggregate of few updates these programs launch (the wide tile)
        return ("cfg4-sized vectors: aggregate of 3 binary32 updates (traffic-mix reference)",
                16 * W.CONFIGS["cfg4"].n)
    call = ["aggregate", "aggregate+apply", "ordered apply", "grouped apply"][op]
    call += ["", " + norms", " + norms of every update"][norms]
    if kind.startswith("BF16"):
        cfg = "cfg4"
    elif op == 2 or (op == 3 and stream == 3):
        cfg = "cfg3"
    elif not has_h and op == 1:
        cfg = "cfg1"
    else:
        cfg = "cfg2"
    c = W.CONFIGS[cfg]
    state = 4 if op == 0 else (16 if has_h else 8)
    return f"{cfg}: {call}", (c.in_bytes * c.K + state) * c.n


def per_kernel(path, value):
    """kernel -> list of value(row) in dispatch order."""
    rows = list(csv.DictReader(open(path)))
    key = "Dispatch_Id" if "Dispatch_Id" in rows[0] else "Start_Timestamp"
    rows.sort(key=lambda r: int(r[key]))
    out = collections.OrderedDict()
    for r in rows:
        k = short(r["Kernel_Name"])
        if ours(k):
            out.setdefault((k, r.get("Counter_Name", "")), []).append(value(r))
    return out


def halves(kernel, values):
    """The sparse call runs with word id = rank - 1 first, then with permuted ids."""
    if any(kernel.startswith(s) for s in SPARSE_KERNELS) and len(values) % 2 == 0 and values:
        h = len(values) // 2
        return [("cfg5, word id = rank - 1", values[:h]), ("cfg5, word ids permuted", values[h:])]
    return [("", values)]


def write(name, text):
    os.makedirs(PROFILES, exist_ok=True)
    path = os.path.join(PROFILES, name)
    with open(path, "w") as f:
        f.write(text)
    print("wrote", path)


def trace(directory, bench_output):
    line = None
    for l in open(bench_output):
        if l.startswith("{"):
            line = json.loads(l)
    if line is None:
        raise SystemExit("no JSON line in " + bench_output)
    data = per_kernel(find(directory, "kernel_trace"),
                      lambda r: int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    table = []
    sparse_ms = collections.defaultdict(float)
    for (k, _), v in data.items():
        for label, part in halves(k, v):
            avg = sum(part) / len(part)
            wl, nbytes = (label, None) if label else dense_workload(k)
            if label:
                sparse_ms[label] += avg / 1e6
            table.append((avg * len(part), f"| `{k}` | {len(part)} | {avg:.0f} | {min(part)} | {max(part)} | {wl} | "
                          f"{nbytes if nbytes else ''} | {f'{nbytes / avg:.0f}' if nbytes else ''} |"))
    table.sort(key=lambda t: -t[0])
    head_kernel = next(k for (k, _) in data if re.match(r"dense_kernel<F32, 1, true, 0, 0,", k))
    hk = data[(head_kernel, "")]
    rows = line.get("rows", {})
    text = f"""# rocprofv3 kernel trace of the default benchmark run (all rows)

Command (on the MI355X box, from the repository root; TMPDIR=/tmp):

    rocprofv3 --kernel-trace --stats --output-format csv -d <trace dir> -- python3 bench.py --no-cpu-baseline

Summary written by `python3 -m paper_1907_00434_amd.profile_summary trace <trace dir> <output of that run>`.

The timed region is {line['warmup']} warm-up + {line['steps']} steps of `mlf_aggregate_apply` on cfg2 (K = 16 binary32 updates of
25,557,032 elements, momentum); the other rows are 3 + 20 + 20 launches each.  bench.py printed for this
run: `value` {line['value']} GB/s, `ms_per_step` {line['ms_per_step']} (wall), `roofline.avg_launch_ms` {line['roofline']['avg_launch_ms']}
(HIP events around the timed launches); the profiler's average for the same kernel, `{head_kernel}`,
over all its {len(hk)} dispatches is {sum(hk) / len(hk) / 1e6:.5f} ms.

{KEY}  The sparse call runs twice in this benchmark
(word id = Zipf rank - 1, then the same triples with the word ids permuted); its kernels' dispatches are
split accordingly.

| kernel | calls | avg ns | min ns | max ns | workload | algorithmic bytes | GB/s at avg |
|---|---:|---:|---:|---:|---|---:|---:|
""" + "\n".join(t[1] for t in table) + "\n"
    if sparse_ms:
        text += "\nSparse call (cfg5, 64,000,000 triples): its six kernels sum to " + " and ".join(
            f"{ms:.3f} ms ({label})" for label, ms in sparse_ms.items())
        r1, r2 = rows.get("cfg5:sparse_scatter_add"), rows.get("cfg5:sparse_scatter_add (permuted word ids)")
        if r1 and r2:
            text += (f"; bench.py rows of this run (HIP events around 20 calls): {r1['ms']:.3f} and {r2['ms']:.3f} ms.  "
                     f"Algorithmic bytes of the call: {r1['algorithmic_bytes']:,} (12 B per triple, 8 B per distinct "
                     f"cell touched ({r1['distinct_cells_touched']:,}), the totals once in each direction).\n")
        else:
            text += ".\n"
    write("bench_default_kernel_trace.md", text)


def traffic(fetch_dir, write_dir):
    import workloads as W
    kib = 1024 / 1e6
    F = per_kernel(find(fetch_dir, "counter_collection"), lambda r: float(r["Counter_Value"]))
    Wr = per_kernel(find(write_dir, "counter_collection"), lambda r: float(r["Counter_Value"]))
    avg = lambda v: sum(v) / len(v)
    copy = next(k for (k, c) in F if "copyBuffer" in k)
    cf, cw = avg(F[(copy, "FETCH_SIZE")]), avg(Wr[(copy, "WRITE_SIZE")])
    copy_mb = (1 << 30) / 1e6
    sf, sw = copy_mb / (cf * kib), copy_mb / (cw * kib)
    lines, sparse_total = [], collections.OrderedDict()
    per_workload = {}
    for (k, _), v in F.items():
        if "copyBuffer" in k or (k, "WRITE_SIZE") not in Wr:
            continue
        for (label, fpart), (_, wpart) in zip(halves(k, v), halves(k, Wr[(k, "WRITE_SIZE")])):
            rd, wr = sf * avg(fpart) * kib, sw * avg(wpart) * kib
            wl, nbytes = (label, None) if label else dense_workload(k)
            lines.append(f"| `{k}` | {wl} | {avg(fpart) * kib:.1f} | {rd:.1f} | {avg(wpart) * kib:.1f} | {rd + wr:.1f} | "
                         f"{f'{nbytes / 1e6:.1f}' if nbytes else ''} | {f'{(rd + wr) * 1e6 / nbytes:.3f}' if nbytes else ''} |")
            if label:
                t = sparse_total.setdefault(label, [0.0, 0.0])
                t[0] += rd
                t[1] += wr
            elif nbytes and wl[:4] in W.CONFIGS and " + " not in wl.replace("aggregate+apply", "") and \
                    wl.split(": ")[1] in ("aggregate+apply", "ordered apply"):
                per_workload[wl[:4]] = int(round((rd + wr) * 1e6))
    for label, (rd, wr) in sparse_total.items():
        lines.append(f"| whole sparse call | {label} | | {rd:.1f} | {wr:.1f} | {rd + wr:.1f} | | |")
    if sparse_total:
        rd, wr = next(iter(sparse_total.values()))
        per_workload["cfg5"] = int(round((rd + wr) * 1e6))
    text = f"""# HBM traffic of every kernel from rocprofv3 hardware counters (FETCH_SIZE, WRITE_SIZE)

Two runs of the same program, one counter each (on the MI355X box, from the repository root; TMPDIR=/tmp):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <FETCH_SIZE dir> -- python3 -m paper_1907_00434_amd.profile_workloads copy cfg1 cfg2 cfg3 cfg4 cfg5
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <WRITE_SIZE dir> -- python3 -m paper_1907_00434_amd.profile_workloads copy cfg1 cfg2 cfg3 cfg4 cfg5

Summary (and `hbm_traffic.json` beside it, which `bench.py` reads `roofline.traffic` from) written by
`python3 -m paper_1907_00434_amd.profile_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir>`.
Counter values are KiB per dispatch, averaged over the dispatches of a kernel.

Calibration: the `copy` workload is a plain 1 GiB -> 1 GiB device copy (`{copy}`, 1,073.7 MB read and
written).  FETCH_SIZE reads {cf:,.1f} KiB ({cf * kib:.1f} MB) for it and WRITE_SIZE {cw:,.1f} KiB ({cw * kib:.1f} MB).  Scale factors:
FETCH_SIZE x {sf:.3f}, WRITE_SIZE x {sw:.3f}.

{KEY}

| kernel | workload | FETCH_SIZE MB | scaled = read MB | WRITE_SIZE MB | traffic MB | algorithmic MB | traffic / algorithmic |
|---|---|---:|---:|---:|---:|---:|---:|
""" + "\n".join(lines) + """

(The norms variants add only their partial sums.  The sparse call runs twice; its dispatches are split into the
run with word id = rank - 1 and the run with permuted ids.  Its algorithmic bytes depend on the distinct cells the
batch touches, which bench.py counts: see `bench_default_kernel_trace.md`.)
"""
    write("hbm_traffic_pmc.md", text)
    record = {"kernel_source_sha256": kernel_source_digest(),
              "unit": "HBM bytes per launch of the workload's call: FETCH_SIZE and WRITE_SIZE, each scaled by the "
                      "reading for a plain 1 GiB copy",
              "fetch_scale": round(sf, 4), "write_scale": round(sw, 4),
              "traffic_bytes": per_workload}
    write("hbm_traffic.json", json.dumps(record, indent=1) + "\n")


def counters(name, title, dirs):
    text = f"""# {title}

One `rocprofv3 --pmc` run per table (on the MI355X box, from the repository root; TMPDIR=/tmp); the command is
given above each.  Summary written by
`python3 -m paper_1907_00434_amd.profile_summary counters {name} "<title>" <dir> ...`.
Values are sums over the chip, averaged over the dispatches of a kernel.  {KEY}

"""
    for d in dirs:
        data = per_kernel(find(d, "counter_collection"), lambda r: float(r["Counter_Value"]))
        names, table = [], collections.OrderedDict()
        for (k, c), v in data.items():
            if "copyBuffer" in k:
                continue
            if c not in names:
                names.append(c)
            for label, part in halves(k, v):
                table.setdefault((k, label), {})[c] = sum(part) / len(part)
        workloads = sorted({(label or dense_workload(k)[0])[:4] for (k, label) in table} - {""})
        text += (f"    rocprofv3 --pmc {' '.join(names)} --output-format csv -d <dir> -- "
                 f"python3 -m paper_1907_00434_amd.profile_workloads --reps 3 {' '.join(workloads)}\n\n")
        text += "| kernel | workload | " + " | ".join(names) + " |\n|---|---|" + "---:|" * len(names) + "\n"
        for (k, label), vals in table.items():
            wl = label if label else dense_workload(k)[0]
            text += f"| `{k}` | {wl} | " + " | ".join(f"{vals[c]:.4g}" if c in vals else "" for c in names) + " |\n"
        text += "\n"
    write(name + ".md", text)


def main(argv):
    if len(argv) >= 3 and argv[0] == "trace":
        trace(argv[1], argv[2])
    elif len(argv) >= 3 and argv[0] == "traffic":
        traffic(argv[1], argv[2])
    elif len(argv) >= 4 and argv[0] == "counters":
        counters(argv[1], argv[2], argv[3:])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv[1:])
