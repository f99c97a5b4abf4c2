"""Pins for the oracle's LDA count-delta scatter-add (Sec. 6 of the paper: a
worker's update is a numerical update to the word-topic matrix).  CPU only."""
import numpy as np
import pytest

import oracle
import workloads as W


def small_cfg(**kw):
    base = dict(V=301, T=17, K=3, m=5000)
    base.update(kw)
    return W.scaled(W.CONFIGS["cfg5"], **base)


def host_inputs(cfg, **kw):
    d = W.sparse_inputs(cfg, "cpu", **kw)
    return (W.to_host(d["counts"]), W.to_host(d["totals"]),
            [W.to_host(t) for t in d["triples"]])


def test_hand_case(golden):
    g = {k: np.array([int(x) for x in v], dtype=np.int32)
         for k, v in golden("scatter_tiny.txt").items()}
    V, T = int(g["V"][0]), int(g["T"][0])
    counts, totals = g["counts0"].copy(), g["totals0"].copy()
    tr = [g["triples0"].reshape(-1, 3).copy(), g["triples1"].reshape(-1, 3).copy()]
    rej = oracle.scatter_add(counts, totals, V, T, tr)
    assert np.array_equal(counts, g["counts"])
    assert np.array_equal(totals, g["totals"])
    assert rej == int(g["rejected"][0])


@pytest.mark.parametrize("init", ["zeros", "random"])
def test_equals_numpy_add_at_and_bincount(init):
    cfg = small_cfg()
    counts, totals, tr = host_inputs(cfg, init=init)
    c0, t0 = counts.copy(), totals.copy()
    rej = oracle.scatter_add(counts, totals, cfg.V, cfg.T, tr)
    allt = np.concatenate(tr).astype(np.int64)
    flat = allt[:, 0] * cfg.T + allt[:, 1]
    ref = c0.astype(np.int64)
    np.add.at(ref, flat, allt[:, 2])
    assert rej == 0 and np.array_equal(counts, ref)
    hist = np.bincount(flat, weights=allt[:, 2], minlength=cfg.V * cfg.T)
    assert np.array_equal(counts - c0, hist.astype(np.int64))
    tref = t0 + np.bincount(allt[:, 1], weights=allt[:, 2], minlength=cfg.T).astype(np.int64)
    assert np.array_equal(totals, tref)


def test_mass_is_conserved_and_totals_are_column_sums():
    cfg = small_cfg()
    counts, totals, tr = host_inputs(cfg, init="random", n_invalid=9)
    c0, t0 = counts.copy(), totals.copy()
    rej = oracle.scatter_add(counts, totals, cfg.V, cfg.T, tr)
    assert rej == 9 * cfg.K
    allt = np.concatenate(tr).astype(np.int64)
    ok = (allt[:, 0] >= 0) & (allt[:, 0] < cfg.V) & (allt[:, 1] >= 0) & (allt[:, 1] < cfg.T)
    assert counts.astype(np.int64).sum() - c0.astype(np.int64).sum() == allt[ok, 2].sum()
    assert np.array_equal(totals - t0, (counts - c0).reshape(cfg.V, cfg.T).sum(axis=0))
    assert np.array_equal(totals, counts.reshape(cfg.V, cfg.T).sum(axis=0))


def test_negated_deltas_restore_the_state():
    cfg = small_cfg()
    counts, totals, tr = host_inputs(cfg, init="random")
    c0, t0 = counts.copy(), totals.copy()
    oracle.scatter_add(counts, totals, cfg.V, cfg.T, tr)
    assert not np.array_equal(counts, c0)
    neg = [t * np.array([1, 1, -1], dtype=np.int32) for t in tr]
    oracle.scatter_add(counts, totals, cfg.V, cfg.T, neg)
    assert np.array_equal(counts, c0) and np.array_equal(totals, t0)


def test_result_does_not_depend_on_order_or_split():
    cfg = small_cfg()
    counts, totals, tr = host_inputs(cfg)
    oracle.scatter_add(counts, totals, cfg.V, cfg.T, tr)
    allt = np.concatenate(tr)
    rng = np.random.default_rng(1)
    shuffled = allt[rng.permutation(len(allt))]
    parts = [np.ascontiguousarray(p) for p in np.array_split(shuffled, [10, 4000, 4001])]
    c2 = np.zeros_like(counts)
    t2 = np.zeros_like(totals)
    oracle.scatter_add(c2, t2, cfg.V, cfg.T, parts)
    assert np.array_equal(counts, c2) and np.array_equal(totals, t2)


def test_additions_wrap_modulo_2_32():
    counts = np.array([2 ** 31 - 1, -2 ** 31], dtype=np.int32)
    totals = np.array([2 ** 31 - 1], dtype=np.int32)
    tr = [np.array([[0, 0, 1], [1, 0, -1]], dtype=np.int32)]
    oracle.scatter_add(counts, totals, 2, 1, tr)
    assert counts.tolist() == [-2 ** 31, 2 ** 31 - 1]
    assert totals.tolist() == [2 ** 31 - 1]


def test_totals_are_optional_and_empty_input_is_fine():
    counts = np.zeros(6, dtype=np.int32)
    tr = [np.array([[1, 1, 5]], dtype=np.int32), np.zeros((0, 3), dtype=np.int32)]
    assert oracle.scatter_add(counts, None, 3, 2, tr) == 0
    assert counts.tolist() == [0, 0, 0, 5, 0, 0]
    assert oracle.scatter_add(counts, None, 3, 2, []) == 0


def test_thread_partition_gives_the_same_state():
    cfg = small_cfg(m=20000)
    counts, totals, tr = host_inputs(cfg, init="random", n_invalid=3)
    c1, t1 = counts.copy(), totals.copy()
    r1 = oracle.scatter_add(c1, t1, cfg.V, cfg.T, tr, threads=1)
    c2, t2 = counts.copy(), totals.copy()
    r2 = oracle.scatter_add(c2, t2, cfg.V, cfg.T, tr, threads=6)
    assert r1 == r2 and np.array_equal(c1, c2) and np.array_equal(t1, t2)


def test_generator_follows_the_truncated_zipf_law():
    cfg = small_cfg(V=1000, T=10, K=1, m=400000)
    tr = W.to_host(W.sparse_triples(cfg, 0, "cpu"))
    assert tr[:, 0].min() >= 0 and tr[:, 0].max() < cfg.V
    assert set(np.unique(tr[:, 2]).tolist()) == {-1, 1}
    freq = np.bincount(tr[:, 0], minlength=cfg.V) / cfg.m
    pmf = np.arange(1, cfg.V + 1) ** -1.1
    pmf /= pmf.sum()
    assert abs(freq[0] - pmf[0]) < 0.01 and abs(freq[:10].sum() - pmf[:10].sum()) < 0.01
    assert abs(tr[:, 2].mean()) < 0.01


# ---- the same update exchanged as dense delta matrices (Sec. 6) ------------------

def dense_deltas(cfg, triples):
    """One V x T delta matrix per worker, built from its triples with numpy."""
    mats = []
    for t in triples:
        t = t.astype(np.int64)
        ok = (t[:, 0] >= 0) & (t[:, 0] < cfg.V) & (t[:, 1] >= 0) & (t[:, 1] < cfg.T)
        m = np.zeros(cfg.V * cfg.T, dtype=np.int64)
        np.add.at(m, t[ok, 0] * cfg.T + t[ok, 1], t[ok, 2])
        mats.append(m.astype(np.int32))
    return mats


def test_dense_delta_sum_equals_the_triple_scatter():
    cfg = small_cfg(m=20000)
    counts, totals, tr = host_inputs(cfg, init="random", n_invalid=4)
    c1, t1 = counts.copy(), totals.copy()
    oracle.scatter_add(c1, t1, cfg.V, cfg.T, tr)
    c2, t2 = counts.copy(), totals.copy()
    oracle.counts_add_dense(c2, t2, cfg.V, cfg.T, dense_deltas(cfg, tr))
    assert np.array_equal(c1, c2) and np.array_equal(t1, t2)
    c3, t3 = counts.copy(), totals.copy()
    oracle.counts_add_dense(c3, t3, cfg.V, cfg.T, dense_deltas(cfg, tr), threads=5)
    assert np.array_equal(c1, c3) and np.array_equal(t1, t3)


def test_dense_delta_sum_against_numpy_and_wraparound():
    rng = np.random.default_rng(12)
    V, T, K = 37, 11, 5
    mats = [rng.integers(-2 ** 31, 2 ** 31, V * T, dtype=np.int64).astype(np.int32) for _ in range(K)]
    counts = rng.integers(-2 ** 31, 2 ** 31, V * T, dtype=np.int64).astype(np.int32)
    totals = rng.integers(-2 ** 31, 2 ** 31, T, dtype=np.int64).astype(np.int32)
    total = np.sum([m.astype(np.int64) for m in mats], axis=0)
    ref_c = ((counts.astype(np.int64) + total) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
    ref_t = ((totals.astype(np.int64) + total.reshape(V, T).sum(axis=0)) & 0xFFFFFFFF
             ).astype(np.uint32).view(np.int32)
    oracle.counts_add_dense(counts, totals, V, T, mats)
    assert np.array_equal(counts, ref_c) and np.array_equal(totals, ref_t)
    c = np.array([1, 2], dtype=np.int32)
    oracle.counts_add_dense(c, None, 2, 1, [])             # no workers, no totals
    assert c.tolist() == [1, 2]


def test_touched_cells_counts_distinct_valid_cells():
    """Pinned by numpy.unique on the flat indices of the valid triples; deltas that
    cancel and triples that repeat a cell must not change the count."""
    rng = np.random.default_rng(5)
    V, T = 37, 11
    tr = np.stack([rng.integers(-2, V + 2, 4000), rng.integers(-1, T + 1, 4000),
                   rng.choice([-1, 1], 4000)], axis=1).astype(np.int32)
    valid = (tr[:, 0] >= 0) & (tr[:, 0] < V) & (tr[:, 1] >= 0) & (tr[:, 1] < T)
    want = np.unique(tr[valid, 0].astype(np.int64) * T + tr[valid, 1]).size
    halves = [tr[:1500].copy(), tr[1500:].copy()]
    assert oracle.touched_cells(V, T, halves) == want
    assert oracle.touched_cells(V, T, halves, threads=4) == want
    cancel = np.array([[3, 2, 1], [3, 2, -1], [3, 2, 5]], dtype=np.int32)
    assert oracle.touched_cells(V, T, [cancel]) == 1
    assert oracle.touched_cells(V, T, []) == 0
