"""The calls only enqueue kernels (no allocation, no memset, no synchronisation),
so they can be recorded into a HIP graph.  Each replay is checked against the
same number of eager calls, with ordinary eager work between the replays."""
import pytest
import torch

import paper_1907_00434_amd as mlf
import workloads as W

pytestmark = pytest.mark.gpu


def same_bits(a, b):
    return torch.equal(a.view(torch.int32), b.view(torch.int32))


@pytest.mark.parametrize("name,n", [("cfg2", 300_003), ("cfg3", 200_001), ("cfg4", 400_004)])
def test_dense_calls_replay_from_a_graph(name, n):
    cfg = W.scaled(W.CONFIGS[name], n=n)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    model, momentum = d["model"].clone(), d["momentum"].clone()
    out = torch.empty(cfg.n, device="cuda")

    def call(w, h):
        if cfg.call == "apply_ordered":
            mlf.mlf_apply_ordered(w, h, d["updates"], d["order"], d["lr"], d["mu"])
        else:
            mlf.mlf_aggregate_apply(w, h, out, d["updates"], d["order"], d["weights"],
                                    d["lr"], d["mu"])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up outside the capture
        call(model.clone(), momentum.clone())
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(model, momentum)

    w_ref, h_ref = d["model"].clone(), d["momentum"].clone()
    for replay in range(4):
        graph.replay()
        call(w_ref, h_ref)                                  # eager twin
        scratch = torch.randn(1 << 16, device="cuda").sum() # unrelated eager work
        torch.cuda.synchronize()
        assert same_bits(model, w_ref), f"model differs after replay {replay}"
        assert same_bits(momentum, h_ref), f"momentum differs after replay {replay}"
        assert torch.isfinite(scratch)


@pytest.mark.parametrize("use_workspace", [False, True])
def test_sparse_call_replays_from_a_graph(use_workspace):
    cfg = W.scaled(W.CONFIGS["cfg5"], V=5003, T=1000, K=3, m=150_000)
    d = W.sparse_inputs(cfg, "cuda", init="random", n_invalid=5)
    counts, totals = d["counts"].clone(), d["totals"].clone()
    rejected = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = None
    if use_workspace:
        nbytes = mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m)
        assert nbytes > 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def call(c, t, r):
        mlf.mlf_sparse_scatter_add(c, t, cfg.V, cfg.T, d["triples"], workspace=ws, n_rejected=r)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(counts.clone(), totals.clone(), rejected.clone())
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(counts, totals, rejected)

    c_ref, t_ref = d["counts"].clone(), d["totals"].clone()
    r_ref = torch.zeros(1, dtype=torch.int32, device="cuda")
    for replay in range(4):
        graph.replay()
        torch.cuda.synchronize()
        call(c_ref, t_ref, r_ref)          # the eager twin shares the scratch: run it after
        torch.cuda.synchronize()
        assert torch.equal(counts, c_ref), f"counts differ after replay {replay}"
        assert torch.equal(totals, t_ref) and torch.equal(rejected, r_ref)
    assert rejected.item() == 4 * 5 * cfg.K
