"""GPU parity: the dense HIP kernels against the CPU oracle, bit for bit, from
the same seeded inputs (binary32 paths are built without contraction, so the
bar is raw-bit equality; see the tolerance discussion in the design notes)."""
import numpy as np
import pytest
import torch

import paper_1907_00434_amd as mlf
import workloads as W
from parity import assert_same_bits, run_dense

pytestmark = pytest.mark.gpu

CALLS = ["aggregate", "apply_ordered", "aggregate_apply"]
RAGGED_N = [1, 3, 7, 8, 9, 255, 256, 257, 2047, 2048, 2049, 4099, 70001]


def recipe(name, **kw):
    return W.scaled(W.CONFIGS[name], **kw)


@pytest.mark.parametrize("call", CALLS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_sizes(call, dtype):
    for n in RAGGED_N:
        cfg = recipe("cfg2", n=n, K=5, dtype=dtype)
        d = W.dense_inputs(cfg, "cuda", momentum_init="random")
        run_dense(call, d, want_out=(n % 2 == 0))


@pytest.mark.parametrize("call", CALLS)
@pytest.mark.parametrize("K", [1, 2, 3, 7, 8, 9, 16, 17, 31, 32, 33, 64])
def test_number_of_updates(call, K):
    for dtype in ("f32", "bf16"):
        cfg = recipe("cfg3", n=6151, K=K, dtype=dtype, weighted=(K % 2 == 1))
        d = W.dense_inputs(cfg, "cuda", momentum_init="random")
        if d["weights"] is not None:   # non-trivial, non-dyadic weights
            d["weights"] = np.random.default_rng(K).uniform(0.1, 2.0, K).astype(np.float32)
        run_dense(call, d, want_out=True)


@pytest.mark.parametrize("call", CALLS)
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4"])
def test_config_recipes_over_many_tiles(call, name):
    """Each configuration's recipe (value distribution, K, weights, lr, mu) at a
    size that spans a few hundred tiles and ends in a ragged tail."""
    cfg = recipe(name, n=700_003)
    d = W.dense_inputs(cfg, "cuda")
    run_dense(call, d, want_out=True)


@pytest.mark.parametrize("call", ["apply_ordered", "aggregate_apply"])
@pytest.mark.parametrize("dtype,n", [("f32", 512 * (2 * 4096 + 37) + 3),
                                     ("bf16", 2048 * (4096 + 5) + 9)])
def test_tile_numbering_over_whole_and_partial_blocks(call, dtype, n):
    """Cache-resident state: workgroups take tiles in runs per XCD, block by
    block of 4,096 tiles, the last partial block in plain order.  Sizes with whole
    blocks, a partial block and a ragged tail; every element must be visited once."""
    cfg = recipe("cfg2", n=n, K=2, dtype=dtype)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    run_dense(call, d, want_out=True)


@pytest.mark.parametrize("call", CALLS)
def test_dropped_updates_and_null_pointers(call):
    cfg = recipe("cfg2", n=5000, K=8)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random", n_dropped=3)
    for j in range(cfg.K):
        if j not in d["order"]:
            d["updates"][j] = None          # a dropped worker's pointer may be NULL
    run_dense(call, d)


@pytest.mark.parametrize("call", CALLS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_misaligned_base_pointers(call, dtype):
    """Pointers aligned to the element but not to 16 bytes take the element-wise
    path and must give the same bits."""
    n = 3001
    cfg = recipe("cfg2", n=n + 3, K=4, dtype=dtype)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    for which in ("one update", "model", "momentum"):
        e = dict(d)
        e["updates"] = [u[(1 if which == "one update" and j == 2 else 0):][:n]
                        for j, u in enumerate(d["updates"])]
        e["model"] = d["model"][(3 if which == "model" else 0):][:n]
        e["momentum"] = d["momentum"][(1 if which == "momentum" else 0):][:n]
        ptrs = [t.data_ptr() for t in e["updates"]] + [e["model"].data_ptr(),
                                                       e["momentum"].data_ptr()]
        assert any(p % 16 for p in ptrs)
        run_dense(call, e, want_out=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_misaligned_large_enough_to_stride(dtype):
    """The element-wise region is walked by a bounded number of workgroups that
    stride over it: make it longer than one sweep of them."""
    n = 700_001
    cfg = recipe("cfg2", n=n + 1, K=3, dtype=dtype)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    d["model"] = d["model"][1:]
    d["momentum"] = d["momentum"][:n]
    d["updates"] = [u[:n] for u in d["updates"]]
    assert d["model"].data_ptr() % 16 != 0
    for call in CALLS:
        run_dense(call, d, want_out=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_state_larger_than_the_infinity_cache(dtype):
    """Model + momentum (+ out) above 256 MiB switch the kernels to streamed
    state accesses (and bfloat16 to its 4-element lane layout); ragged n."""
    cfg = recipe("cfg3", n=34_000_003, K=3, dtype=dtype)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    d["weights"] = np.array([0.5, 0.3, 1.7], np.float32)
    run_dense("apply_ordered", d)
    run_dense("aggregate_apply", d, want_out=True)
    del d
    cfg = recipe("cfg3", n=68_000_001, K=2, dtype=dtype)
    d = W.dense_inputs(cfg, "cuda")
    d["weights"] = np.array([0.7, 1.1], np.float32)
    run_dense("aggregate", d)
    del d
    torch.cuda.empty_cache()


def test_without_momentum_buffer_and_without_weights():
    for dtype in ("f32", "bf16"):
        cfg = recipe("cfg1", n=40_001, dtype=dtype)
        d = W.dense_inputs(cfg, "cuda")
        assert d["momentum"] is None
        run_dense("apply_ordered", d)
        run_dense("aggregate_apply", d, want_out=False)
        d["weights"] = None
        run_dense("aggregate", d)
        run_dense("aggregate_apply", d, want_out=True)


def test_special_values_survive():
    special = torch.tensor([0.0, -0.0, 1e-45, -1e-40, float("inf"), -float("inf"), 3.0,
                            1.17549435e-38, float("nan"), 2.0 ** -126], device="cuda")
    n = special.numel()
    junk = torch.full((n,), 5.0, device="cuda")
    out = torch.empty(n, device="cuda")
    mlf.mlf_aggregate([junk, special], [1], None, out)      # K = 1: a bit copy
    assert_same_bits(out, special.cpu().numpy(), "bit copy")
    d = {"updates": [special, special.flip(0).contiguous(), junk], "order": np.array([1, 0, 2], np.int32),
         "weights": np.array([0.5, 1.0, 2.0 ** -20], np.float32),
         "model": torch.linspace(-1, 1, n, device="cuda"),
         "momentum": torch.full((n,), 1e-39, device="cuda"), "lr": 0.5, "mu": 0.5}
    with np.errstate(all="ignore"):
        for call in CALLS:
            run_dense(call, d, want_out=True)


def test_left_to_right_sum_and_unfused_products(golden):
    g = golden("aggregate_hand_cases.txt")

    def dev(key):
        return torch.tensor([float(v) for v in g[key]], device="cuda")

    ups = [dev(f"rounding.U{j}") for j in range(3)]
    out = torch.empty(1, device="cuda")
    mlf.mlf_aggregate(ups, [int(v) for v in g["rounding.order_abc"]], None, out)
    assert out.item() == float(g["rounding.out_abc"][0])
    mlf.mlf_aggregate(ups, [int(v) for v in g["rounding.order_bca"]], None, out)
    assert out.item() == float(g["rounding.out_bca"][0])
    ups = [dev("product.U0"), dev("product.U1")]
    mlf.mlf_aggregate(ups, [0, 1], [float(v) for v in g["product.weights"]], out)
    assert out.item() == 0.0
    x = 1.0 + 2.0 ** -12
    w, h = torch.tensor([3.0], device="cuda"), torch.tensor([x], device="cuda")
    mlf.mlf_apply_ordered(w, h, [torch.tensor([1.0 + 2.0 ** -11], device="cuda")], [0], 1.0, x)
    assert h.item() == 0.0 and w.item() == 3.0


def test_paper_two_update_values_on_gpu(golden):
    g = {k: float(v[0]) for k, v in golden("apply_two_updates.txt").items()}
    ups = [torch.tensor([g["g1"]], device="cuda"), torch.tensor([g["g2"]], device="cuda")]
    for order, tag in (([0, 1], "order12"), ([1, 0], "order21")):
        w, h = torch.tensor([g["w0"]], device="cuda"), torch.tensor([g["h0"]], device="cuda")
        mlf.mlf_apply_ordered(w, h, ups, order, g["lr"], g["gamma"])
        assert w.item() == g[f"w2_{tag}"] and h.item() == g[f"h2_{tag}"]


def test_empty_inputs():
    u = torch.ones(10, device="cuda")
    out = torch.full((10,), 3.0, device="cuda")
    mlf.mlf_aggregate([u], [], None, out)                     # empty order: +0
    assert_same_bits(out, np.zeros(10, np.float32), "empty order")
    out.fill_(3.0)
    mlf.mlf_aggregate([u], [0], None, out, n=0)               # n = 0: untouched
    assert (out == 3.0).all()
    w, h = torch.full((10,), 1.0, device="cuda"), torch.full((10,), 0.5, device="cuda")
    mlf.mlf_apply_ordered(w, h, [u], [], 0.1, 0.5)            # no update: no-op
    assert (w == 1.0).all() and (h == 0.5).all()
    mlf.mlf_aggregate_apply(w, h, None, [u], [], None, 0.1, 0.5)   # zero-gradient step
    assert (h == 0.25).all() and (w == 1.25).all()


def test_fused_equals_aggregate_then_apply():
    cfg = recipe("cfg2", n=123_457)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    w1, h1 = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_aggregate_apply(w1, h1, None, d["updates"], d["order"], d["weights"], d["lr"], d["mu"])
    a = torch.empty(cfg.n, device="cuda")
    mlf.mlf_aggregate(d["updates"], d["order"], d["weights"], a)
    w2, h2 = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_ordered(w2, h2, [a], [0], d["lr"], d["mu"])
    assert torch.equal(w1.view(torch.int32), w2.view(torch.int32))
    assert torch.equal(h1.view(torch.int32), h2.view(torch.int32))


def test_launch_on_a_side_stream():
    cfg = recipe("cfg2", n=50_000, K=4)
    d = W.dense_inputs(cfg, "cuda")
    out_a = torch.empty(cfg.n, device="cuda")
    out_b = torch.empty(cfg.n, device="cuda")
    mlf.mlf_aggregate(d["updates"], d["order"], d["weights"], out_a)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    mlf.mlf_aggregate(d["updates"], d["order"], d["weights"], out_b, stream=s)
    s.synchronize()
    assert torch.equal(out_a.view(torch.int32), out_b.view(torch.int32))


# ---- one scheduled batch: direct prefix + aggregated groups ----------------------

def split_into_groups(M, seed, n_direct=None):
    """A direct prefix of singleton groups followed by random aggregated groups."""
    rng = np.random.default_rng(seed)
    n_direct = int(rng.integers(0, M + 1)) if n_direct is None else n_direct
    lens, left = [1] * n_direct, M - n_direct
    while left > 0:
        ln = int(rng.integers(1, left + 1))
        lens.append(ln)
        left -= ln
    return lens


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K", [1, 2, 5, 16, 17, 33, 64])
def test_grouped_apply(dtype, K):
    for n in (1, 9, 257, 6151, 70_001):
        cfg = recipe("cfg2", n=n, K=K, dtype=dtype)
        d = W.dense_inputs(cfg, "cuda", momentum_init="random", n_dropped=K // 5)
        d["weights"] = np.random.default_rng(K).uniform(0.1, 2.0, K).astype(np.float32)
        d["group_len"] = split_into_groups(len(d["order"]), seed=K * 1000 + n)
        run_dense("apply_grouped", d)


def test_grouped_apply_without_momentum_or_weights_and_misaligned():
    cfg = recipe("cfg1", n=40_004, K=7)
    d = W.dense_inputs(cfg, "cuda")
    d["weights"] = None
    d["group_len"] = [1, 1, 2, 3]
    run_dense("apply_grouped", d)
    d["model"] = d["model"][1:]
    d["updates"] = [u[:cfg.n - 1] for u in d["updates"]]
    run_dense("apply_grouped", d)


def test_grouped_apply_reduces_to_the_other_calls_on_the_gpu():
    cfg = recipe("cfg2", n=123_457)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    M = len(d["order"])
    w1, h1 = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_grouped(w1, h1, d["updates"], d["order"], None, [1] * M, d["lr"], d["mu"])
    w2, h2 = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_ordered(w2, h2, d["updates"], d["order"], d["lr"], d["mu"])
    assert torch.equal(w1.view(torch.int32), w2.view(torch.int32))
    assert torch.equal(h1.view(torch.int32), h2.view(torch.int32))
    w1, h1 = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_grouped(w1, h1, d["updates"], d["order"], d["weights"], [M], d["lr"], d["mu"])
    w2, h2 = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_aggregate_apply(w2, h2, None, d["updates"], d["order"], d["weights"], d["lr"], d["mu"])
    assert torch.equal(w1.view(torch.int32), w2.view(torch.int32))
    assert torch.equal(h1.view(torch.int32), h2.view(torch.int32))


def test_grouped_apply_full_size_alexnet_batch():
    """cfg3's 32 updates as a scheduled batch: 8 forwarded directly, then three
    aggregated groups of 8 (state above the Infinity Cache: streamed)."""
    cfg = W.CONFIGS["cfg3"]
    d = W.dense_inputs(cfg, "cuda")
    d["weights"] = np.full(cfg.K, 0.125, np.float32)
    d["weights"][d["order"][:8]] = 1.0
    d["group_len"] = [1] * 8 + [8, 8, 8]
    run_dense("apply_grouped", d)
    del d
    torch.cuda.empty_cache()


@pytest.mark.parametrize("K", [16, 30])
def test_orders_from_the_scheduling_heuristic(K):
    """Commit orders produced the way the paper's scheduler does (shortest
    transfer first, deadlines, look-ahead drops) instead of plain permutations."""
    from workloads.scheduler import scheduled_order
    for seed in (3, 4, 5):
        cfg = recipe("cfg3", n=50_003, K=K)
        d = W.dense_inputs(cfg, "cuda", momentum_init="random")
        d["order"] = scheduled_order(K, seed)
        run_dense("apply_ordered", d)
        d["weights"] = np.full(K, 1.0 / K, np.float32)
        M = len(d["order"])
        d["group_len"] = [1] * (M // 3) + [M - M // 3]
        run_dense("apply_grouped", d)
