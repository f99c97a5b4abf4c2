"""Launches the calls of the named configurations a few times each, and nothing
else: the program to put after `rocprofv3 ... --` when per-kernel hardware
counters or a kernel trace of one configuration are wanted without the rest of
the benchmark around it.

    python3 -m paper_1907_00434_amd.profile_workloads [--reps N] cfg3 cfg5 ...

cfg2 / cfg4: aggregate_apply (cfg2 also the plain aggregate and the grouped apply
with norms and with per-update norms); cfg3: apply_ordered, apply_grouped,
apply_grouped_norms, apply_grouped_update_norms, divergence;
cfg5: sparse_scatter_add with word id = rank - 1, then with the ids permuted;
copy: a plain 1 GiB device copy (the reference for byte counters).
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("workloads", nargs="+", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "copy"])
    args = ap.parse_args()

    import torch

    import paper_1907_00434_amd as mlf
    import workloads as W

    dev = "cuda:0"
    torch.cuda.set_device(0)
    for name in args.workloads:
        if name == "copy":
            src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
            dst = torch.empty_like(src)
            for _ in range(args.reps):
                dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        elif name == "cfg5":
            cfg = W.CONFIGS[name]
            for permute in (False, True):
                d = W.sparse_inputs(cfg, dev, permute_ids=permute)
                ws = torch.empty(max(mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m), 256),
                                 dtype=torch.uint8, device=dev)
                for _ in range(args.reps):
                    mlf.mlf_sparse_scatter_add(d["counts"], d["totals"], cfg.V, cfg.T, d["triples"], workspace=ws)
                torch.cuda.synchronize()
                del d, ws
        else:
            cfg = W.CONFIGS[name]
            d = W.dense_inputs(cfg, dev)
            M = len(d["order"])
            groups = [1] * (M // 4) + [(M - M // 4) // 3] * 2 + [M - M // 4 - 2 * ((M - M // 4) // 3)]
            norms = torch.zeros(2, dtype=torch.float64, device=dev)
            ws = torch.empty(mlf.mlf_norms_workspace_bytes(cfg.n), dtype=torch.uint8, device=dev)
            for _ in range(args.reps):
                if name == "cfg3":
                    mlf.mlf_apply_ordered(d["model"], d["momentum"], d["updates"], d["order"], d["lr"], d["mu"])
                else:
                    mlf.mlf_aggregate_apply(d["model"], d["momentum"], None, d["updates"], d["order"],
                                            d["weights"], d["lr"], d["mu"])
            if name in ("cfg2", "cfg3"):
                for _ in range(args.reps):
                    mlf.mlf_apply_grouped(d["model"], d["momentum"], d["updates"], d["order"], d["weights"],
                                          groups, d["lr"], d["mu"])
                for _ in range(args.reps):
                    mlf.mlf_apply_grouped_norms(d["model"], d["momentum"], d["updates"], d["order"],
                                                d["weights"], groups, d["lr"], d["mu"], norms, ws)
                per_update = torch.zeros(M, dtype=torch.float64, device=dev)
                ws2 = torch.empty(mlf.mlf_update_norms_workspace_bytes(cfg.n), dtype=torch.uint8, device=dev)
                for _ in range(args.reps):
                    mlf.mlf_apply_grouped_update_norms(d["model"], d["momentum"], d["updates"], d["order"],
                                                       d["weights"], groups, d["lr"], d["mu"], norms,
                                                       per_update, ws2)
            if name == "cfg2":
                out = torch.empty(cfg.n, device=dev)
                for _ in range(args.reps):
                    mlf.mlf_aggregate(d["updates"], d["order"], d["weights"], out)
                del out
            if name == "cfg3":
                other = d["model"] + 1e-3
                for _ in range(args.reps):
                    mlf.mlf_divergence(d["model"], other, norms[:1], ws)
                del other
            torch.cuda.synchronize()
            del d, ws
        torch.cuda.empty_cache()
        print("ran", name, flush=True)


if __name__ == "__main__":
    main()
