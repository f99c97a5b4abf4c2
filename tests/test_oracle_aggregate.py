"""Pins for the oracle's ordered weighted sum (aggregator, Sec. 4 / Sec. 3.2 /
Sec. 5.2 of the paper).  None of these use the GPU library."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import workloads as W


def f32(vals):
    return np.array([float(v) for v in vals], dtype=np.float32)


def ints(vals):
    return [int(v) for v in vals]


def bits(a):
    return np.asarray(a, dtype=np.float32).view(np.uint32)


# ---- values worked out by hand / printed example ---------------------------

def test_paper_four_worker_example(golden):
    g = golden("aggregate_hand_cases.txt")
    ups = [f32(g[f"paper.g{j}"]) for j in (1, 2, 3, 4)]
    r = oracle.aggregate(ups, ints(g["paper.order"]))
    assert np.array_equal(bits(r), bits(f32(g["paper.r"])))


def test_hand_weighted_case(golden):
    g = golden("aggregate_hand_cases.txt")
    ups = [f32(g[f"weighted.U{j}"]) for j in range(3)]
    out = oracle.aggregate(ups, ints(g["weighted.order"]), f32(g["weighted.weights"]))
    assert np.array_equal(bits(out), bits(f32(g["weighted.out"])))


def test_left_to_right_order_in_binary32(golden):
    g = golden("aggregate_hand_cases.txt")
    ups = [f32(g[f"rounding.U{j}"]) for j in range(3)]
    abc = oracle.aggregate(ups, ints(g["rounding.order_abc"]))
    bca = oracle.aggregate(ups, ints(g["rounding.order_bca"]))
    assert abc[0] == float(g["rounding.out_abc"][0])
    assert bca[0] == float(g["rounding.out_bca"][0])


def test_product_rounded_before_sum(golden):
    g = golden("aggregate_hand_cases.txt")
    ups = [f32(g["product.U0"]), f32(g["product.U1"])]
    out = oracle.aggregate(ups, ints(g["product.order"]), f32(g["product.weights"]))
    assert out[0] == 0.0  # a fused multiply-add would leave 2^-24


# ---- exact arithmetic: permutation invariance --------------------------------

def test_exact_data_matches_integer_sum_for_every_permutation():
    rng = np.random.default_rng(5)
    K, n = 4, 257
    q = rng.integers(-1024, 1025, size=(K, n))           # integers, |v| <= 2^10
    ups = [(q[j] * 2.0 ** -10).astype(np.float32) for j in range(K)]
    wnum = np.array([4, 2, 1, 2])                          # weights 1, 1/2, 1/4, 1/2
    weights = (wnum / 4.0).astype(np.float32)
    exact = (q * wnum[:, None]).sum(axis=0)                # int64, units of 2^-12
    expect = (exact * 2.0 ** -12).astype(np.float32)       # exactly representable
    assert np.array_equal(expect.astype(np.float64) * 4096, exact)
    for perm in itertools.permutations(range(K)):
        out = oracle.aggregate(ups, list(perm), weights)
        assert np.array_equal(bits(out), bits(expect)), perm


def test_unweighted_exact_sum_and_dropped_updates():
    rng = np.random.default_rng(6)
    K, n = 5, 64
    q = rng.integers(-1000, 1001, size=(K, n))
    ups = [q[j].astype(np.float32) for j in range(K)]
    order = [3, 0, 4]                                      # workers 1 and 2 dropped
    out = oracle.aggregate(ups, order)
    assert np.array_equal(out.astype(np.int64), q[order].sum(axis=0))


# ---- against binary64 within the recursive-summation bound -------------------

@pytest.mark.parametrize("cfg_name", ["cfg1", "cfg2", "cfg4"])
def test_within_summation_bound_of_binary64(cfg_name):
    cfg = W.scaled(W.CONFIGS[cfg_name], n=4099)
    d = W.dense_inputs(cfg, "cpu")
    ups = [W.to_host(u) for u in d["updates"]]
    out = oracle.aggregate(ups, d["order"], d["weights"])
    if cfg.dtype == "bf16":
        wide = [torch.from_numpy(u.view(np.int16)).view(torch.bfloat16).double().numpy()
                for u in ups]
    else:
        wide = [u.astype(np.float64) for u in ups]
    terms = np.stack([np.float64(d["weights"][j]) * wide[j] for j in d["order"]])
    ref = terms.sum(axis=0)
    M = len(d["order"])
    bound = M * 2.0 ** -24 * np.abs(terms).sum(axis=0) * 1.01 + 1e-45
    assert np.all(np.abs(out.astype(np.float64) - ref) <= bound)
    # and it is a mean of K draws: the scale must be right
    assert abs(out.std() / (ref.std()) - 1) < 1e-4


# ---- special cases -----------------------------------------------------------

def test_single_update_without_weights_is_a_bit_copy():
    special = np.array([0.0, -0.0, 1e-45, -1e-40, np.inf, -np.inf, 3.0, 1.17549435e-38],
                       dtype=np.float32)
    junk = np.full_like(special, 7.0)
    out = oracle.aggregate([junk, special], [1])
    assert np.array_equal(bits(out), bits(special))
    nan_in = np.array([np.nan], dtype=np.float32)
    assert np.isnan(oracle.aggregate([nan_in], [0]))[0]


def test_empty_order_gives_positive_zero():
    out = oracle.aggregate([np.ones(5, dtype=np.float32)], [])
    assert np.array_equal(bits(out), np.zeros(5, dtype=np.uint32))


def test_weights_are_indexed_by_worker_not_by_position():
    ups = [np.full(3, 1.0, np.float32), np.full(3, 10.0, np.float32)]
    out = oracle.aggregate(ups, [1, 0], np.array([2.0, 0.5], np.float32))
    assert np.array_equal(out, np.full(3, 7.0, np.float32))   # 0.5*10 + 2*1


def test_denormals_are_kept():
    tiny = np.array([1e-45, 2e-45], dtype=np.float32)          # subnormal
    out = oracle.aggregate([tiny, tiny], [0, 1])
    assert np.array_equal(bits(out), bits(tiny) * 2)
    out = oracle.aggregate([np.array([2.0 ** -126], np.float32)], [0],
                           np.array([0.5], np.float32))
    assert out[0] == np.float32(2.0 ** -127)


# ---- bf16 widening: all 65,536 patterns against torch's conversion -----------

def test_bf16_widening_all_patterns():
    patt = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    out = oracle.aggregate([patt], [0])
    ref = torch.from_numpy(patt.view(np.int16)).view(torch.bfloat16).float().numpy()
    assert np.array_equal(bits(out), bits(ref))
    assert oracle.widen_bf16(0x3F80) == 1.0 and oracle.widen_bf16(0xC000) == -2.0


# ---- a library doing the same separate fp32 operations -----------------------

def test_matches_sequential_torch_float32_ops():
    cfg = W.scaled(W.CONFIGS["cfg2"], n=10007)
    d = W.dense_inputs(cfg, "cpu")
    acc = None
    for j in d["order"]:
        term = d["updates"][j] * torch.tensor(d["weights"][j])
        acc = term if acc is None else acc + term
    out = oracle.aggregate([W.to_host(u) for u in d["updates"]], d["order"], d["weights"])
    assert np.array_equal(bits(out), bits(acc.numpy()))


def test_thread_slices_do_not_change_bits():
    cfg = W.scaled(W.CONFIGS["cfg1"], n=100003)
    d = W.dense_inputs(cfg, "cpu")
    ups = [W.to_host(u) for u in d["updates"]]
    a = oracle.aggregate(ups, d["order"], d["weights"], threads=1)
    b = oracle.aggregate(ups, d["order"], d["weights"], threads=5)
    assert np.array_equal(bits(a), bits(b))


def test_rejects_bad_order():
    u = [np.zeros(2, np.float32)] * 2
    with pytest.raises(ValueError):
        oracle.aggregate(u, [0, 0])
    with pytest.raises(ValueError):
        oracle.aggregate(u, [2])
