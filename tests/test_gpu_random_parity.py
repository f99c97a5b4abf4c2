"""Seeded random sweep over the dense calls: K, n, order length, weights,
momentum, data type, group shapes and pointer misalignment are all drawn at
random (fixed seeds, so every run checks the same cases), each compared with
the oracle bit for bit."""
import numpy as np
import pytest
import torch

import workloads as W
from parity import run_dense

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = np.random.default_rng(seed)
    K = int(rng.choice([1, 2, 3, 4, 7, 8, 15, 16, 17, 31, 32, 40, 64]))
    n = int(rng.choice([1, 2, 5, 63, 64, 65, 127, 129, 511, 513, 1000, 4097, 20_011, 131_075]))
    dtype = str(rng.choice(["f32", "bf16"]))
    base = str(rng.choice(["cfg1", "cfg2", "cfg3", "cfg4"]))
    cfg = W.scaled(W.CONFIGS[base], n=n + 3, K=K, dtype=dtype, momentum=bool(rng.random() < 0.7),
                   lr=float(rng.choice([0.1, 0.01, 1.0, 3e-4])), mu=float(rng.choice([0.0, 0.5, 0.9, 0.99])))
    d = W.dense_inputs(cfg, "cuda", momentum_init="random", n_dropped=int(rng.integers(0, K)))
    # views into the padded tensors: offsets 0..3 elements break 16-byte alignment
    def view(t, off):
        return t[off:off + n]
    offs = rng.integers(0, 4, size=K + 2) * int(rng.random() < 0.4)
    d["updates"] = [view(u, int(offs[j])) for j, u in enumerate(d["updates"])]
    d["model"] = view(d["model"], int(offs[K]))
    if d["momentum"] is not None:
        d["momentum"] = view(d["momentum"], int(offs[K + 1]))
    kind = rng.integers(0, 3)
    if kind == 0:
        d["weights"] = None
    elif kind == 1:
        d["weights"] = rng.uniform(-2.0, 2.0, K).astype(np.float32)
    else:
        d["weights"] = np.full(K, 1.0 / K, np.float32)
    M = len(d["order"])
    lens, left = [], M
    while left > 0:
        ln = int(rng.integers(1, left + 1)) if rng.random() < 0.5 else 1
        lens.append(ln)
        left -= ln
    d["group_len"] = lens
    return d


@pytest.mark.parametrize("block", range(8))
def test_random_dense_cases(block):
    for seed in range(block * 12, block * 12 + 12):
        d = random_case(1907_00434 + seed)
        for call in ("aggregate", "apply_ordered", "aggregate_apply", "apply_grouped"):
            try:
                run_dense(call, d, want_out=bool(seed % 2), threads=4)
            except AssertionError as e:
                raise AssertionError(f"seed {seed}, call {call}: {e}") from e
    torch.cuda.synchronize()


def random_sparse_case(seed):
    """Shape, skew, number and raggedness of the buffers, delta range (both
    record formats), invalid triples and word-id permutation drawn at random;
    sizes on both sides of the point where the binned path takes over."""
    rng = np.random.default_rng(seed)
    V = int(rng.choice([1, 7, 300, 5_003, 40_000, 250_000]))
    T = int(rng.choice([1, 3, 64, 1_000, 4_097]))
    while V * T > 100_000_000:
        V //= 2
    K = int(rng.choice([1, 2, 5, 9, 64]))
    total = int(rng.choice([50_000, 300_000, 700_000, 1_500_000]))
    cfg = W.scaled(W.CONFIGS["cfg5"], V=V, T=T, K=K, m=max(total // K, 1),
                   zipf_s=float(rng.choice([0.0, 0.8, 1.1, 2.0])), index=int(seed % 100_000))
    d = W.sparse_inputs(cfg, "cuda", init=str(rng.choice(["zeros", "random"])),
                        permute_ids=bool(rng.random() < 0.5), n_invalid=int(rng.integers(0, 9)))
    # ragged buffers: cut each at a random length (some empty)
    d["triples"] = [t[: int(rng.integers(0, t.shape[0] + 1))] if rng.random() < 0.4 else t
                    for t in d["triples"]]
    mode = rng.integers(0, 3)
    if mode == 1:      # a few large deltas: the call switches to 8-byte records
        for t in d["triples"]:
            if t.shape[0] > 10:
                t[3::1013, 2] = int(rng.integers(-2 ** 31, 2 ** 31))
    elif mode == 2:    # every delta small but not +-1
        for t in d["triples"]:
            t[:, 2] *= int(rng.integers(1, 1023))
    return cfg, d


@pytest.mark.parametrize("block", range(4))
def test_random_sparse_cases(block):
    from parity import run_sparse
    for seed in range(block * 6, block * 6 + 6):
        cfg, d = random_sparse_case(1907_00434 + 1000 + seed)
        for use_workspace in (False, True):
            try:
                run_sparse(cfg, d, use_workspace, threads=4)
            except AssertionError as e:
                raise AssertionError(f"seed {seed}, workspace {use_workspace}: {e}") from e
    torch.cuda.synchronize()
