"""The C-ABI library loads, exports every symbol the header declares, and its
host-side argument checks answer without touching a GPU (every call below
returns before anything is enqueued)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1907_00434_amd as mlf
from paper_1907_00434_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mlfabric.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mlf_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"mlf_aggregate", "mlf_apply_ordered", "mlf_aggregate_apply", "mlf_apply_grouped",
            "mlf_sparse_scatter_add", "mlf_sparse_workspace_bytes", "mlf_aggregate_norm",
            "mlf_apply_grouped_norms", "mlf_norms_workspace_bytes", "mlf_divergence", "mlf_divergence_static",
            "mlf_counts_add_dense", "mlf_aggregate_update_norms", "mlf_apply_grouped_update_norms",
            "mlf_update_norms_workspace_bytes", "mlf_divergence_bound",
            "mlf_status_string"} <= set(names)
    lib = ctypes.CDLL(mlf.library_path())
    for name in names:
        assert hasattr(lib, name), name


def test_header_is_plain_c():
    """The boundary is a C header: it must compile as C99 on its own."""
    import subprocess
    hdr = os.path.join(ROOT, "include", "mlfabric.h")
    res = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                          "-fsyntax-only", "-x", "c", hdr], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def test_status_strings():
    for code in (0, -1, -2, -3, -4):
        assert mlf.mlf_status_string(code).startswith("MLF_")
    assert "unknown" in mlf.mlf_status_string(-99)


FAKE = 0x10000000   # stands for a 16-byte aligned device address; never dereferenced


def tab(*ptrs):
    t = (ctypes.c_void_p * len(ptrs))(*ptrs)
    return t


def order(*idx):
    a = (ctypes.c_int32 * max(len(idx), 1))(*idx)
    return a, len(idx)


def agg(ptrs, K, n, dtype, idx, out, weights=None):
    o, m = order(*idx)
    return B.raw().mlf_aggregate(tab(*ptrs), K, n, dtype, o, m, weights, out, None)


def test_aggregate_argument_checks():
    u0, u1, out = FAKE, FAKE + 0x100000, FAKE + 0x200000
    assert agg([u0, u1], 2, 0, B.MLF_F32, [0, 1], out) == B.MLF_OK          # n = 0
    assert agg([u0, u1], 0, 8, B.MLF_F32, [], out) == B.MLF_EINVAL          # K < 1
    assert agg([u0, u1], 2, -1, B.MLF_F32, [0], out) == B.MLF_EINVAL
    assert agg([u0, u1], 2, 8, B.MLF_F32, [0, 0], out) == B.MLF_EINVAL      # listed twice
    assert agg([u0, u1], 2, 8, B.MLF_F32, [2], out) == B.MLF_EINVAL         # out of range
    assert agg([u0, u1], 2, 8, B.MLF_F32, [-1], out) == B.MLF_EINVAL
    assert agg([u0, u1], 2, 8, B.MLF_F32, [0, 1, 0], out) == B.MLF_EINVAL   # n_order > K
    assert agg([u0, None], 2, 8, B.MLF_F32, [1], out) == B.MLF_EINVAL       # listed but NULL
    assert agg([u0, u1], 2, 8, B.MLF_F32, [0], None) == B.MLF_EINVAL        # NULL out
    assert agg([u0, u1], 2, 8, 7, [0], out) == B.MLF_EINVAL                 # dtype
    assert agg([u0 + 2, u1], 2, 8, B.MLF_F32, [0], out) == B.MLF_EALIGN
    assert agg([u0 + 1, u1], 2, 8, B.MLF_BF16, [0], out) == B.MLF_EALIGN
    assert agg([u0, u1], 2, 8, B.MLF_F32, [0], out + 2) == B.MLF_EALIGN
    assert agg([u0, u1], 2, 8, B.MLF_F32, [1], u1 + 16) == B.MLF_EINVAL     # out overlaps update
    assert agg([u0] * 65, 65, 8, B.MLF_F32, [0], out) == B.MLF_EUNSUPPORTED


def test_apply_argument_checks():
    lib = B.raw()
    u0, w, h = FAKE, FAKE + 0x100000, FAKE + 0x200000
    o, m = order(0)
    assert lib.mlf_apply_ordered(None, h, tab(u0), 1, 8, 0, o, m, 0.1, 0.9, None) == B.MLF_EINVAL
    assert lib.mlf_apply_ordered(w, w + 16, tab(u0), 1, 8, 0, o, m, 0.1, 0.9, None) == B.MLF_EINVAL
    assert lib.mlf_apply_ordered(w, h, tab(w), 1, 8, 0, o, m, 0.1, 0.9, None) == B.MLF_EINVAL
    assert lib.mlf_apply_ordered(w, h, tab(u0), 1, 0, 0, o, m, 0.1, 0.9, None) == B.MLF_OK
    e, _ = order()
    assert lib.mlf_apply_ordered(w, h, tab(u0), 1, 8, 0, e, 0, 0.1, 0.9, None) == B.MLF_OK
    assert lib.mlf_aggregate_apply(w, h, w + 4, tab(u0), 1, 8, 0, o, m, None, 0.1, 0.9,
                                   None) == B.MLF_EINVAL
    assert lib.mlf_aggregate_apply(None, h, None, tab(u0), 1, 8, 0, o, m, None, 0.1, 0.9,
                                   None) == B.MLF_EINVAL


def test_grouped_argument_checks():
    lib = B.raw()
    u0, u1, w, h = FAKE, FAKE + 0x100000, FAKE + 0x200000, FAKE + 0x300000
    o, m = order(0, 1)

    def call(lens, n=8):
        g = (ctypes.c_int32 * max(len(lens), 1))(*lens)
        return lib.mlf_apply_grouped(w, h, tab(u0, u1), 2, n, 0, o, m, None, g, len(lens),
                                     0.1, 0.9, None)

    assert call([1, 1], n=0) == B.MLF_OK
    assert call([1]) == B.MLF_EINVAL             # does not cover the order
    assert call([1, 2]) == B.MLF_EINVAL          # overshoots
    assert call([2, 0]) == B.MLF_EINVAL          # empty group
    assert call([0, 2]) == B.MLF_EINVAL
    assert call([]) == B.MLF_EINVAL
    assert lib.mlf_apply_grouped(None, h, tab(u0, u1), 2, 8, 0, o, m, None,
                                 (ctypes.c_int32 * 1)(2), 1, 0.1, 0.9, None) == B.MLF_EINVAL


def test_sparse_argument_checks():
    lib = B.raw()
    counts, buf = FAKE, FAKE + 0x100000
    n1 = (ctypes.c_int64 * 1)(5)
    n0 = (ctypes.c_int64 * 1)(0)
    neg = (ctypes.c_int64 * 1)(-1)

    def call(c, V, T, ptrs, cnt, K):
        return lib.mlf_sparse_scatter_add(c, None, V, T, ptrs, cnt, K, None, 0, None, None)

    assert call(None, 3, 2, tab(buf), n1, 1) == B.MLF_EINVAL
    assert call(counts, 0, 2, tab(buf), n1, 1) == B.MLF_EINVAL
    assert call(counts, 3, 0, tab(buf), n1, 1) == B.MLF_EINVAL
    assert call(counts, 3, 2, tab(buf), neg, 1) == B.MLF_EINVAL
    assert call(counts, 3, 2, tab(None), n1, 1) == B.MLF_EINVAL
    assert call(counts, 3, 2, tab(buf + 2), n1, 1) == B.MLF_EALIGN
    assert call(counts, 3, 2, tab(buf), n0, 1) == B.MLF_OK
    assert call(counts, 3, 2, None, None, 0) == B.MLF_OK
    many = (ctypes.c_int64 * 65)(*([1] * 65))
    assert call(counts, 3, 2, tab(*([buf] * 65)), many, 65) == B.MLF_EUNSUPPORTED
    assert mlf.mlf_sparse_workspace_bytes(100000, 1000, 0) >= 0


def test_sparse_scratch_size_and_path_selection():
    """Host logic of the sparse call's scratch query: 0 where the direct path
    serves (small batches, matrices past 2^30 cells), else 8 to 14 bytes per
    triple, growing with the batch, a multiple of the 256-byte alignment."""
    ws = mlf.mlf_sparse_workspace_bytes
    tile = 32_768                                              # cells per tile
    for V, T in ((100_000, 1_000), (1, 1), (3, 40_000), (1_000_000, 1_000)):
        tiles = (V * T + tile - 1) // tile
        least = 262_144 + 600 * tiles
        assert ws(V, T, least - 1) == 0
        assert ws(V, T, 0) == 0 and ws(V, T, -5) == 0
        a, b = ws(V, T, least), ws(V, T, 4 * least)
        assert 0 < a < b and a % 256 == 0 and b % 256 == 0
        assert 8 * least <= a <= 14 * least + 64 * tiles * 4 + (1 << 20)
    assert ws(32_768, 32_768, 10 ** 9) > 0                     # exactly 2^30 cells
    assert ws(32_769, 32_768, 10 ** 9) == 0                    # one row more
    assert ws(0, 5, 10 ** 6) == 0 and ws(5, 0, 10 ** 6) == 0
    assert ws(100_000, 1_000, 2 ** 31) == 0                    # more triples than a 32-bit index


def test_norms_scratch_size():
    ws = mlf.mlf_norms_workspace_bytes
    assert ws(-1) == 0
    sizes = [ws(n) for n in (0, 1, 511, 512, 513, 10 ** 6, 10 ** 9)]
    assert all(x > 0 and x % 16 == 0 for x in sizes)
    assert sizes == sorted(sizes)
    assert ws(10 ** 9) <= 70 * 10 ** 6                         # 16 bytes per 256 elements, about


def test_dense_delta_argument_checks():
    lib = B.raw()
    counts, d0 = FAKE, FAKE + 0x100000
    assert lib.mlf_counts_add_dense(counts, None, 3, 2, tab(d0), 0, None) == B.MLF_OK
    assert lib.mlf_counts_add_dense(None, None, 3, 2, tab(d0), 1, None) == B.MLF_EINVAL
    assert lib.mlf_counts_add_dense(counts, None, 0, 2, tab(d0), 1, None) == B.MLF_EINVAL
    assert lib.mlf_counts_add_dense(counts, None, 3, 2, tab(None), 1, None) == B.MLF_EINVAL
    assert lib.mlf_counts_add_dense(counts, None, 3, 2, tab(d0 + 2), 1, None) == B.MLF_EALIGN
    assert lib.mlf_counts_add_dense(counts, None, 3, 2, tab(counts + 8), 1, None) == B.MLF_EINVAL
    assert lib.mlf_counts_add_dense(counts, None, 3, 2, tab(*([d0] * 65)), 65, None) == B.MLF_EUNSUPPORTED


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        mlf.mlf_aggregate([torch.zeros(4)], [0], None, torch.zeros(4))


def test_divergence_static_argument_checks():
    """The entry point without a workspace rejects sizes beyond its scratch array
    (and the other bad arguments) before it touches the device."""
    lib = B.raw()
    a, b, out = FAKE, FAKE + 0x100000, FAKE + 0x200000
    assert lib.mlf_divergence_static(a, b, B.MLF_STATIC_MAX_N + 1, out, None) == B.MLF_EUNSUPPORTED
    assert "MLF_STATIC_MAX_N" in mlf.mlf_status_string(B.MLF_EUNSUPPORTED)
    assert lib.mlf_divergence_static(None, b, 8, out, None) == B.MLF_EINVAL
    assert lib.mlf_divergence_static(a, None, 8, out, None) == B.MLF_EINVAL
    assert lib.mlf_divergence_static(a, b, 8, None, None) == B.MLF_EINVAL
    assert lib.mlf_divergence_static(a, b, -1, out, None) == B.MLF_EINVAL
    assert lib.mlf_divergence_static(a + 2, b, 8, out, None) == B.MLF_EALIGN
    assert lib.mlf_divergence_static(a, b, 8, out + 4, None) == B.MLF_EALIGN
    text = open(os.path.join(ROOT, "include", "mlfabric.h")).read()
    assert re.search(r"#define MLF_STATIC_MAX_N \(1ll << 28\)", text) and B.MLF_STATIC_MAX_N == 1 << 28


def test_update_norms_argument_checks():
    lib = B.raw()
    u0, u1, w, h, out = FAKE, FAKE + 0x100000, FAKE + 0x200000, FAKE + 0x300000, FAKE + 0x400000
    norms, per_update, ws = FAKE + 0x500000, FAKE + 0x500100, FAKE + 0x600000
    need = mlf.mlf_update_norms_workspace_bytes(8)
    assert need > 0 and need == mlf.mlf_update_norms_workspace_bytes(10 ** 9) and need < 8 << 20
    assert mlf.mlf_update_norms_workspace_bytes(-1) == 0
    o, m = order(0, 1)
    g = (ctypes.c_int32 * 2)(1, 1)

    def agg_call(out=out, norms=norms, per_update=per_update, ws=ws, nbytes=need, n=0):
        return lib.mlf_aggregate_update_norms(tab(u0, u1), 2, n, 0, o, m, None, out, norms, per_update,
                                              ws, nbytes, None)

    assert agg_call(per_update=None) == B.MLF_EINVAL
    assert agg_call(norms=None) == B.MLF_EINVAL
    assert agg_call(out=None) == B.MLF_EINVAL
    assert agg_call(ws=None) == B.MLF_EINVAL
    assert agg_call(nbytes=need - 1) == B.MLF_EINVAL
    assert agg_call(per_update=per_update + 4) == B.MLF_EALIGN
    assert agg_call(ws=ws + 8) == B.MLF_EALIGN

    def grouped_call(model=w, norms=norms, per_update=per_update, ws=ws, nbytes=need, lens=g, n_groups=2):
        return lib.mlf_apply_grouped_update_norms(model, h, tab(u0, u1), 2, 8, 0, o, m, None, lens, n_groups,
                                                  0.1, 0.9, norms, per_update, ws, nbytes, None)

    assert grouped_call(per_update=None) == B.MLF_EINVAL
    assert grouped_call(model=None) == B.MLF_EINVAL
    assert grouped_call(nbytes=16) == B.MLF_EINVAL
    assert grouped_call(n_groups=1) == B.MLF_EINVAL            # does not cover the order
    assert grouped_call(norms=norms + 4) == B.MLF_EALIGN


def test_divergence_bound_against_the_oracle_and_its_argument_checks():
    import math

    import oracle
    rng = np.random.default_rng(31)
    for trial in range(50):
        K = int(rng.integers(1, 20))
        M = int(rng.integers(0, K + 1))
        order_ = [int(i) for i in rng.permutation(K)[:M]]
        groups, left = [], M
        while left > 0:
            ln = int(rng.integers(1, left + 1))
            groups.append(ln)
            left -= ln
        weights = rng.uniform(-2, 2, K).astype(np.float32) if trial % 3 else None
        lr, mu = float(np.float32(rng.uniform(0.001, 0.5))), float(np.float32(rng.uniform(0, 0.99)))
        h_sq = float(rng.uniform(0, 10))
        u_sq = rng.uniform(0, 100, M)
        got = mlf.mlf_divergence_bound(h_sq, u_sq, order_, K, weights, groups, lr, mu)
        in_sequence = weights[order_] if weights is not None else None
        want = oracle.divergence_bound(math.sqrt(h_sq), np.sqrt(u_sq), in_sequence, groups, lr, mu)
        assert abs(got - want) <= 1e-13 * max(abs(want), 1e-300), (trial, got, want)
    # the two-update case of Sec. 3.3 with dyadic numbers: (g + g^2) ||h0|| + (1 + g) ||u1|| + ||u2||
    assert mlf.mlf_divergence_bound(9.0, [25.0, 49.0], [1, 0], 2, None, [1, 1], 0.25, 0.5) == \
        0.75 * 3 + 1.5 * 0.25 * 5 + 0.25 * 7
    lib = B.raw()
    out = ctypes.c_double()
    o, m = order(0, 1)
    u = (ctypes.c_double * 2)(1.0, 2.0)
    g = (ctypes.c_int32 * 2)(1, 1)

    def call(h=1.0, u=u, o=o, m=m, K=2, g=g, n_groups=2, out=ctypes.byref(out)):
        return lib.mlf_divergence_bound(h, u, o, m, K, None, g, n_groups, 0.1, 0.9, out)

    assert call() == B.MLF_OK
    assert call(out=None) == B.MLF_EINVAL
    assert call(h=-1.0) == B.MLF_EINVAL and call(h=float("nan")) == B.MLF_EINVAL
    assert call(u=(ctypes.c_double * 2)(1.0, -2.0)) == B.MLF_EINVAL
    assert call(u=None) == B.MLF_EINVAL
    assert call(n_groups=1) == B.MLF_EINVAL
    assert call(g=(ctypes.c_int32 * 2)(2, 0)) == B.MLF_EINVAL
    assert call(o=order(0, 5)[0]) == B.MLF_EINVAL
    assert call(K=65) == B.MLF_EUNSUPPORTED
    assert call(m=0, n_groups=0) == B.MLF_OK and out.value == 0.0
