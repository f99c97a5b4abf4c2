"""Pins for the oracle's server update (Eq. 2 of the paper, folded over the
scheduler's sequence) and for aggregate-then-apply (Sec. 5.4).  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W


def arr(*v):
    return np.array(v, dtype=np.float32)


def bits(a):
    return np.asarray(a, dtype=np.float32).view(np.uint32)


# ---- the paper's printed two-update forms ------------------------------------

def test_paper_two_update_values(golden):
    g = {k: float(v[0]) for k, v in golden("apply_two_updates.txt").items()}
    ups = [arr(g["g1"]), arr(g["g2"])]
    for order, tag in (([0, 1], "order12"), ([1, 0], "order21")):
        w, h = arr(g["w0"]), arr(g["h0"])
        oracle.apply_ordered(w, h, ups, order, g["lr"], g["gamma"])
        assert w[0] == g[f"w2_{tag}"] and h[0] == g[f"h2_{tag}"]
    assert g["w2_order12"] - g["w2_order21"] == g["divergence"]


def test_paper_closed_forms_in_exact_arithmetic():
    """w2 - w0 = (g + g^2) h0 + (1 + g) u1 + u2 ; h2 = g^2 h0 + g u1 + u2 ;
    swapping the two updates moves the model by g (u1 - u2)  (Sec. 3.3).
    Dyadic inputs, so binary32 is exact and must equal the rational value."""
    rng = np.random.default_rng(11)
    n = 8
    gamma, lr = Fraction(1, 2), Fraction(1, 4)
    w0 = rng.integers(-64, 65, n)
    h0 = rng.integers(-64, 65, n)
    g1 = rng.integers(-64, 65, n)
    g2 = rng.integers(-64, 65, n)
    ups = [g1.astype(np.float32), g2.astype(np.float32)]
    w_s, h_s = w0.astype(np.float32), h0.astype(np.float32)
    oracle.apply_ordered(w_s, h_s, ups, [0, 1], float(lr), float(gamma))
    w_r, h_r = w0.astype(np.float32), h0.astype(np.float32)
    oracle.apply_ordered(w_r, h_r, ups, [1, 0], float(lr), float(gamma))
    for i in range(n):
        u1, u2 = -lr * int(g1[i]), -lr * int(g2[i])
        lead = (gamma + gamma ** 2) * int(h0[i]) + (1 + gamma) * u1 + u2
        assert Fraction(float(w_s[i])) == int(w0[i]) + lead
        assert Fraction(float(h_s[i])) == gamma ** 2 * int(h0[i]) + gamma * u1 + u2
        assert Fraction(float(w_s[i])) - Fraction(float(w_r[i])) == gamma * (u1 - u2)


# ---- closed form for any M, in binary64 ---------------------------------------

@pytest.mark.parametrize("M,mu", [(1, 0.9), (5, 0.9), (32, 0.9), (7, 0.0), (16, 0.5)])
def test_closed_form_any_length(M, mu):
    """Unrolling Eq. 2:  h_M = mu^M h0 - lr sum_t mu^(M-t) g_t  (t = 1..M),
    w_M = w0 + sum_{s=1..M} h_s."""
    rng = np.random.default_rng(100 + M)
    n, lr = 513, 0.01
    ups = [rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(M)]
    order = rng.permutation(M).astype(np.int32)
    w0 = rng.normal(0, 1, n).astype(np.float32)
    h0 = rng.normal(0, 1e-4, n).astype(np.float32)
    w, h = w0.copy(), h0.copy()
    oracle.apply_ordered(w, h, ups, order, lr, mu)
    lr64, mu64 = np.float64(np.float32(lr)), np.float64(np.float32(mu))
    G = np.stack([ups[j].astype(np.float64) for j in order])       # g_1..g_M
    hs = []
    for s in range(1, M + 1):
        coeff = mu64 ** (s - np.arange(1, s + 1))                  # mu^(s-t)
        hs.append(mu64 ** s * h0 - lr64 * (coeff[:, None] * G[:s]).sum(axis=0))
    w_ref = w0.astype(np.float64) + np.sum(hs, axis=0)
    assert np.allclose(h, hs[-1], rtol=0, atol=4 * M * 2.0 ** -24 * np.abs(hs).max())
    assert np.all(np.abs(w - w_ref) <= M * 2.0 ** -23 * np.maximum(np.abs(w_ref), 1e-3))


# ---- special cases --------------------------------------------------------------

def test_single_update_no_momentum_is_plain_sgd():
    rng = np.random.default_rng(3)
    n = 1000
    g = rng.normal(0, 1, n).astype(np.float32)
    w0 = rng.normal(0, 1, n).astype(np.float32)
    lr = np.float32(0.01)
    expect = w0 - lr * g                    # numpy binary32: product, then difference
    w = w0.copy()
    oracle.apply_ordered(w, None, [g], [0], 0.01, 0.9)   # mu ignored without a buffer
    assert np.array_equal(bits(w), bits(expect))
    w2, h2 = w0.copy(), np.zeros(n, np.float32)
    oracle.apply_ordered(w2, h2, [g], [0], 0.01, 0.0)
    assert np.array_equal(bits(w2), bits(expect))
    assert np.array_equal(bits(h2), bits(-(lr * g)))


def test_momentum_from_zero_history_first_step():
    # h0 = 0: first step is plain SGD whatever mu is, and h1 = -lr g.
    g, w = arr(2.0, -4.0), arr(1.0, 1.0)
    h = np.zeros(2, np.float32)
    oracle.apply_ordered(w, h, [g], [0], 0.25, 0.9)
    assert np.array_equal(w, arr(0.5, 2.0)) and np.array_equal(h, arr(-0.5, 1.0))


def test_hand_case_three_updates():
    # gamma = 1/2, lr = 1, w0 = 0, h0 = 4, g = (1, 2, -3) applied as (g2, g0, g1)
    # h: 4 -> 2+3 = 5 -> 2.5-1 = 1.5 -> 0.75-2 = -1.25 ; w: 0 -> 5 -> 6.5 -> 5.25
    ups = [arr(1.0), arr(2.0), arr(-3.0)]
    w, h = arr(0.0), arr(4.0)
    oracle.apply_ordered(w, h, ups, [2, 0, 1], 1.0, 0.5)
    assert w[0] == 5.25 and h[0] == -1.25
    # a dropped update (order shorter than K) is simply not applied
    w, h = arr(0.0), arr(4.0)
    oracle.apply_ordered(w, h, ups, [2, 0], 1.0, 0.5)
    assert w[0] == 6.5 and h[0] == 1.5


def test_empty_order_is_a_no_op():
    w, h = arr(1.5), arr(-2.0)
    oracle.apply_ordered(w, h, [arr(9.0)], [], 0.1, 0.9)
    assert w[0] == 1.5 and h[0] == -2.0


def test_products_are_rounded_separately():
    # mu = h = 1 + 2^-12: mu*h = 1 + 2^-11 + 2^-24 rounds to 1 + 2^-11 = lr*g,
    # so h' = 0 and w is unchanged.  A fused mu*h - q would leave 2^-24.
    x = 1.0 + 2.0 ** -12
    w, h = arr(3.0), arr(x)
    oracle.apply_ordered(w, h, [arr(1.0 + 2.0 ** -11)], [0], 1.0, x)
    assert h[0] == 0.0 and w[0] == 3.0
    # same for lr*g in the plain-SGD branch
    w = arr(1.0 + 2.0 ** -11)
    oracle.apply_ordered(w, None, [arr(x)], [0], x, 0.0)
    assert w[0] == 0.0


def test_bf16_updates_are_widened_exactly():
    rng = np.random.default_rng(8)
    n, K = 300, 3
    patt = [rng.integers(0, 65536, n).astype(np.uint16) & np.uint16(0xBF7F) for _ in range(K)]
    wide = [(p.astype(np.uint32) << 16).view(np.float32) for p in patt]
    assert all(np.isfinite(x).all() for x in wide)
    w0 = rng.normal(0, 1, n).astype(np.float32)
    wa, ha = w0.copy(), np.zeros(n, np.float32)
    wb, hb = w0.copy(), np.zeros(n, np.float32)
    with np.errstate(all="ignore"):
        oracle.apply_ordered(wa, ha, patt, [1, 2, 0], 1e-3, 0.9)
        oracle.apply_ordered(wb, hb, wide, [1, 2, 0], 1e-3, 0.9)
    assert np.array_equal(bits(wa), bits(wb)) and np.array_equal(bits(ha), bits(hb))


def test_thread_slices_do_not_change_bits():
    cfg = W.scaled(W.CONFIGS["cfg3"], n=50021, K=6)
    d = W.dense_inputs(cfg, "cpu", momentum_init="random")
    ups = [W.to_host(u) for u in d["updates"]]
    res = []
    for th in (1, 7):
        w, h = W.to_host(d["model"]), W.to_host(d["momentum"])
        oracle.apply_ordered(w, h, ups, d["order"], d["lr"], d["mu"], threads=th)
        res.append((w, h))
    assert np.array_equal(bits(res[0][0]), bits(res[1][0]))
    assert np.array_equal(bits(res[0][1]), bits(res[1][1]))


# ---- aggregate + apply (synchronous iteration, Sec. 5.4) ------------------------

@pytest.mark.parametrize("cfg_name", ["cfg1", "cfg2", "cfg4"])
def test_aggregate_apply_is_aggregate_then_one_step(cfg_name):
    cfg = W.scaled(W.CONFIGS[cfg_name], n=4099)
    d = W.dense_inputs(cfg, "cpu", momentum_init="random")
    ups = [W.to_host(u) for u in d["updates"]]
    w1 = W.to_host(d["model"])
    h1 = W.to_host(d["momentum"]) if d["momentum"] is not None else None
    out = oracle.aggregate_apply(w1, h1, ups, d["order"], d["weights"], d["lr"], d["mu"],
                                 want_out=True)
    a = oracle.aggregate(ups, d["order"], d["weights"])
    w2 = W.to_host(d["model"])
    h2 = W.to_host(d["momentum"]) if d["momentum"] is not None else None
    oracle.apply_ordered(w2, h2, [a], [0], d["lr"], d["mu"])
    assert np.array_equal(bits(out), bits(a))
    assert np.array_equal(bits(w1), bits(w2))
    if h1 is not None:
        assert np.array_equal(bits(h1), bits(h2))


def test_aggregation_commutes_with_the_server_rule_only_without_momentum():
    """Sec. 5.2 says the model after in-network aggregation is consistent with
    no aggregation.  With Eq. 2 that holds for gamma = 0 only; with momentum the
    two differ by the gamma terms of the two-update expansion."""
    rng = np.random.default_rng(21)
    n, K = 64, 4
    ups = [rng.integers(-512, 513, n).astype(np.float32) for _ in range(K)]
    w0 = rng.integers(-512, 513, n).astype(np.float32)
    wt, lr = 0.25, 0.5
    weights = np.full(K, wt, np.float32)
    order = [2, 0, 3, 1]
    # gamma = 0, exact data: aggregate+apply == one-by-one with lr * weight
    wa = w0.copy()
    oracle.aggregate_apply(wa, None, ups, order, weights, lr, 0.0)
    wb = w0.copy()
    oracle.apply_ordered(wb, None, ups, order, lr * wt, 0.0)
    assert np.array_equal(bits(wa), bits(wb))
    expect = w0.astype(np.float64) - lr * wt * np.sum([u.astype(np.float64) for u in ups], axis=0)
    assert np.array_equal(wa.astype(np.float64), expect)
    # gamma = 1/2: they must differ, by exactly the momentum carried between steps
    wa, ha = w0.copy(), np.zeros(n, np.float32)
    oracle.aggregate_apply(wa, ha, ups, order, weights, lr, 0.5)
    wb, hb = w0.copy(), np.zeros(n, np.float32)
    oracle.apply_ordered(wb, hb, ups, order, lr * wt, 0.5)
    assert not np.array_equal(wa, wb)
    # one step on the sum from h0 = 0 is plain SGD on the sum
    assert np.array_equal(wa.astype(np.float64), expect)


def test_aggregate_apply_with_empty_order_takes_a_zero_gradient_step():
    w, h = arr(1.0), arr(0.5)
    out = oracle.aggregate_apply(w, h, [arr(3.0)], [], None, 0.1, 0.5, want_out=True)
    assert out[0] == 0.0 and h[0] == 0.25 and w[0] == 1.25


# ---- one scheduled batch: direct prefix + aggregated groups (Sec. 5.2) ----------

def test_grouped_hand_case_from_the_four_worker_example():
    """Sec. 3.2: g1 and g2 reach the server directly, g3 and g4 are summed at an
    aggregator and arrive as r = g3 + g4.  With gamma = 1/2, lr = 1, w0 = 0, h0 = 0:
      g1 = 1:  h = -1        w = -1
      g2 = 2:  h = -2.5      w = -3.5
      r = 4 + 8 = 12:  h = -1.25 - 12 = -13.25   w = -16.75"""
    ups = [arr(1.0), arr(2.0), arr(4.0), arr(8.0)]
    w, h = arr(0.0), arr(0.0)
    oracle.apply_grouped(w, h, ups, [0, 1, 2, 3], None, [1, 1, 2], 1.0, 0.5)
    assert w[0] == -16.75 and h[0] == -13.25


def test_grouped_in_exact_arithmetic():
    """Three arrivals u1, u2, r = (a3 g3 + a4 g4): unrolling Eq. 2 gives
    h3 = g^3 h0 + g^2 u1 + g u2 + ur and w3 = w0 + h1 + h2 + h3, checked as rationals."""
    rng = np.random.default_rng(31)
    n = 16
    gamma, lr = Fraction(1, 2), Fraction(1, 4)
    vals = {k: rng.integers(-32, 33, n) for k in ("w0", "h0", "g1", "g2", "g3", "g4")}
    ups = [vals[k].astype(np.float32) for k in ("g1", "g2", "g3", "g4")]
    weights = np.array([1.0, 1.0, 0.5, 0.25], np.float32)
    w, h = vals["w0"].astype(np.float32), vals["h0"].astype(np.float32)
    oracle.apply_grouped(w, h, ups, [1, 0, 3, 2], weights, [1, 1, 2], float(lr), float(gamma))
    for i in range(n):
        u_first = -lr * int(vals["g2"][i])                      # order starts with worker 1
        u_second = -lr * int(vals["g1"][i])
        u_r = -lr * (Fraction(1, 4) * int(vals["g4"][i]) + Fraction(1, 2) * int(vals["g3"][i]))
        h1 = gamma * int(vals["h0"][i]) + u_first
        h2 = gamma * h1 + u_second
        h3 = gamma * h2 + u_r
        assert Fraction(float(h[i])) == h3
        assert Fraction(float(w[i])) == int(vals["w0"][i]) + h1 + h2 + h3


@pytest.mark.parametrize("cfg_name", ["cfg2", "cfg4"])
def test_grouped_reduces_to_the_other_calls(cfg_name):
    cfg = W.scaled(W.CONFIGS[cfg_name], n=2053)
    d = W.dense_inputs(cfg, "cpu", momentum_init="random")
    ups = [W.to_host(u) for u in d["updates"]]
    M = len(d["order"])

    def fresh():
        return W.to_host(d["model"]), W.to_host(d["momentum"])

    # all groups of length 1, no weights  ==  apply_ordered
    w1, h1 = fresh()
    oracle.apply_grouped(w1, h1, ups, d["order"], None, [1] * M, d["lr"], d["mu"])
    w2, h2 = fresh()
    oracle.apply_ordered(w2, h2, ups, d["order"], d["lr"], d["mu"])
    assert np.array_equal(bits(w1), bits(w2)) and np.array_equal(bits(h1), bits(h2))
    # one group  ==  aggregate_apply
    w1, h1 = fresh()
    oracle.apply_grouped(w1, h1, ups, d["order"], d["weights"], [M], d["lr"], d["mu"])
    w2, h2 = fresh()
    oracle.aggregate_apply(w2, h2, ups, d["order"], d["weights"], d["lr"], d["mu"])
    assert np.array_equal(bits(w1), bits(w2)) and np.array_equal(bits(h1), bits(h2))
    # a direct prefix and two aggregated groups == aggregates computed apart, then applied
    lens = [1, 1, 3, M - 5]
    w1, h1 = fresh()
    oracle.apply_grouped(w1, h1, ups, d["order"], d["weights"], lens, d["lr"], d["mu"])
    arrivals, first = [], 0
    for ln in lens:
        arrivals.append(oracle.aggregate(ups, d["order"][first:first + ln], d["weights"]))
        first += ln
    w2, h2 = fresh()
    oracle.apply_ordered(w2, h2, arrivals, list(range(len(lens))), d["lr"], d["mu"])
    assert np.array_equal(bits(w1), bits(w2)) and np.array_equal(bits(h1), bits(h2))


def test_grouped_rejects_bad_lengths():
    ups = [arr(1.0), arr(2.0)]
    for lens in ([1], [1, 2], [0, 2], [2, 0]):
        with pytest.raises(ValueError):
            oracle.apply_grouped(arr(0.0), arr(0.0), ups, [0, 1], None, lens, 1.0, 0.5)
