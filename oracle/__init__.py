"""ctypes front end of the CPU oracle (``mlf_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library and its Python binding never
import this package, and this package never imports them.

All arguments are host numpy arrays.  Dense updates are ``float32`` arrays, or
``uint16`` arrays holding bfloat16 bit patterns.  ``threads`` only splits the
element range (dense) or the row / topic ranges (sparse) into independent
slices that run the same C loops; it changes no result.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mlf_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

# One rounding per written operation: no contraction, no fast-math.
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-Wall",
          "-Wextra", "-fPIC", "-shared"]


def build(force: bool = True) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or (
            os.path.getmtime(_LIB) < os.path.getmtime(_SRC)):
        subprocess.run(["gcc", *CFLAGS, "-o", _LIB, _SRC], check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    c = ctypes
    pp = c.POINTER(c.c_void_p)
    i32p = c.POINTER(c.c_int32)
    f32p = c.POINTER(c.c_float)
    for dt in ("f32", "bf16"):
        f = getattr(lib, f"orc_aggregate_{dt}")
        f.argtypes = [pp, c.c_int, c.c_int64, i32p, c.c_int, f32p, c.c_void_p]
        f.restype = None
        f = getattr(lib, f"orc_apply_ordered_{dt}")
        f.argtypes = [c.c_void_p, c.c_void_p, pp, c.c_int, c.c_int64, i32p,
                      c.c_int, c.c_float, c.c_float]
        f.restype = None
        f = getattr(lib, f"orc_aggregate_apply_{dt}")
        f.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, pp, c.c_int,
                      c.c_int64, i32p, c.c_int, f32p, c.c_float, c.c_float]
        f.restype = None
        f = getattr(lib, f"orc_apply_grouped_{dt}")
        f.argtypes = [c.c_void_p, c.c_void_p, pp, c.c_int, c.c_int64, i32p, c.c_int,
                      f32p, i32p, c.c_int, c.c_float, c.c_float]
        f.restype = None
    lib.orc_counts_add_dense.argtypes = [c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, pp,
                                         c.c_int, c.c_int32, c.c_int32, c.c_int32, c.c_int32]
    lib.orc_counts_add_dense.restype = None
    lib.orc_sum_sq_f32.argtypes = [c.c_void_p, c.c_int64]
    lib.orc_sum_sq_f32.restype = c.c_double
    lib.orc_sum_sq_diff_f32.argtypes = [c.c_void_p, c.c_void_p, c.c_int64]
    lib.orc_sum_sq_diff_f32.restype = c.c_double
    lib.orc_sum_sq_bf16.argtypes = [c.c_void_p, c.c_int64]
    lib.orc_sum_sq_bf16.restype = c.c_double
    lib.orc_divergence_bound.argtypes = [c.c_double, c.POINTER(c.c_double), f32p, i32p, c.c_int,
                                         c.c_double, c.c_double]
    lib.orc_divergence_bound.restype = c.c_double
    lib.orc_scatter_add.argtypes = [c.c_void_p, c.c_void_p, c.c_int32,
                                    c.c_int32, pp, c.POINTER(c.c_int64),
                                    c.c_int, c.c_int32, c.c_int32, c.c_int32,
                                    c.c_int32, c.c_int]
    lib.orc_scatter_add.restype = c.c_int64
    lib.orc_widen_bf16.argtypes = [c.c_uint16]
    lib.orc_widen_bf16.restype = c.c_float
    _lib = lib
    return lib


def _dense_kind(updates):
    if len(updates) == 0:
        raise ValueError("need at least one update")
    dt = updates[0].dtype
    if dt == np.float32:
        kind, size = "f32", 4
    elif dt == np.uint16:
        kind, size = "bf16", 2
    else:
        raise TypeError("updates must be float32 or uint16 (bfloat16 bits)")
    n = updates[0].shape[0]
    for u in updates:
        if u.dtype != dt or u.ndim != 1 or u.shape[0] != n or (
                not u.flags.c_contiguous):
            raise ValueError("updates must be equal-length contiguous vectors")
    return kind, size, n


def _order_array(order, K):
    o = np.ascontiguousarray(np.asarray(order, dtype=np.int32))
    if o.ndim != 1 or len(o) > K:
        raise ValueError("order must list at most K indices")
    if len(o) and (o.min() < 0 or o.max() >= K or len(set(o.tolist())) != len(o)):
        raise ValueError("order must hold distinct indices in [0, K)")
    return o


def _weights_array(weights, K):
    if weights is None:
        return None
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.float32))
    if w.shape != (K,):
        raise ValueError("weights must have K entries")
    return w


def _slices(n, threads):
    threads = max(1, min(int(threads), max(1, n)))
    edges = [n * j // threads for j in range(threads + 1)]
    return [(edges[j], edges[j + 1]) for j in range(threads)
            if edges[j + 1] > edges[j]]


def _run(jobs, threads):
    if len(jobs) <= 1 or threads <= 1:
        return [j() for j in jobs]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda j: j(), jobs))


def _ptr_table(arrays, byte_offset):
    tab = (ctypes.c_void_p * len(arrays))()
    for j, a in enumerate(arrays):
        tab[j] = a.ctypes.data + byte_offset
    return tab


def _f32_inplace(a, name, n):
    if a.dtype != np.float32 or a.shape != (n,) or not a.flags.c_contiguous or (
            not a.flags.writeable):
        raise ValueError(f"{name} must be a writeable contiguous float32[n]")


def widen_bf16(bits: int) -> float:
    return float(_load().orc_widen_bf16(int(bits)))


def aggregate(updates, order, weights=None, threads=1):
    """Ordered weighted sum of the listed updates; returns float32[n]."""
    lib = _load()
    kind, size, n = _dense_kind(updates)
    K = len(updates)
    o = _order_array(order, K)
    w = _weights_array(weights, K)
    out = np.empty(n, dtype=np.float32)
    fn = getattr(lib, f"orc_aggregate_{kind}")
    op = o.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    wp = w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)) if w is not None else None

    def job(lo, hi):
        tab = _ptr_table(updates, lo * size)
        return lambda: fn(tab, K, hi - lo, op, len(o), wp, out.ctypes.data + 4 * lo)

    _run([job(lo, hi) for lo, hi in _slices(n, threads)], threads)
    return out


def apply_ordered(model, momentum, updates, order, lr, mu, threads=1):
    """Fold the server update rule over the listed updates, in place."""
    lib = _load()
    kind, size, n = _dense_kind(updates)
    K = len(updates)
    o = _order_array(order, K)
    _f32_inplace(model, "model", n)
    if momentum is not None:
        _f32_inplace(momentum, "momentum", n)
    fn = getattr(lib, f"orc_apply_ordered_{kind}")
    op = o.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))

    def job(lo, hi):
        tab = _ptr_table(updates, lo * size)
        hp = momentum.ctypes.data + 4 * lo if momentum is not None else None
        return lambda: fn(model.ctypes.data + 4 * lo, hp, tab, K, hi - lo, op,
                          len(o), float(lr), float(mu))

    _run([job(lo, hi) for lo, hi in _slices(n, threads)], threads)


def aggregate_apply(model, momentum, updates, order, weights, lr, mu,
                    want_out=False, threads=1):
    """Aggregate, then one server step with the aggregate; in place.

    Returns the aggregate (float32[n]) when ``want_out`` is set, else None."""
    lib = _load()
    kind, size, n = _dense_kind(updates)
    K = len(updates)
    o = _order_array(order, K)
    w = _weights_array(weights, K)
    _f32_inplace(model, "model", n)
    if momentum is not None:
        _f32_inplace(momentum, "momentum", n)
    out = np.empty(n, dtype=np.float32) if want_out else None
    fn = getattr(lib, f"orc_aggregate_apply_{kind}")
    op = o.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    wp = w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)) if w is not None else None

    def job(lo, hi):
        tab = _ptr_table(updates, lo * size)
        hp = momentum.ctypes.data + 4 * lo if momentum is not None else None
        outp = out.ctypes.data + 4 * lo if out is not None else None
        return lambda: fn(model.ctypes.data + 4 * lo, hp, outp, tab, K, hi - lo,
                          op, len(o), wp, float(lr), float(mu))

    _run([job(lo, hi) for lo, hi in _slices(n, threads)], threads)
    return out


def apply_grouped(model, momentum, updates, order, weights, group_len, lr, mu, threads=1):
    """One scheduled batch: consecutive groups of the order, each summed (ordered,
    weighted) and applied as one server step; in place."""
    lib = _load()
    kind, size, n = _dense_kind(updates)
    K = len(updates)
    o = _order_array(order, K)
    w = _weights_array(weights, K)
    g = np.ascontiguousarray(np.asarray(group_len, dtype=np.int32))
    if g.ndim != 1 or (len(g) and g.min() < 1) or int(g.sum()) != len(o):
        raise ValueError("group lengths must be positive and add up to len(order)")
    _f32_inplace(model, "model", n)
    if momentum is not None:
        _f32_inplace(momentum, "momentum", n)
    fn = getattr(lib, f"orc_apply_grouped_{kind}")
    op = o.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    gp = g.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    wp = w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)) if w is not None else None

    def job(lo, hi):
        tab = _ptr_table(updates, lo * size)
        hp = momentum.ctypes.data + 4 * lo if momentum is not None else None
        return lambda: fn(model.ctypes.data + 4 * lo, hp, tab, K, hi - lo, op, len(o), wp,
                          gp, len(g), float(lr), float(mu))

    _run([job(lo, hi) for lo, hi in _slices(n, threads)], threads)


def sum_sq(x, threads=1):
    """||x||_2^2 of a float32 vector, or of a bfloat16 one given as uint16 bit
    patterns (widened exactly first): correctly rounded to binary64 with one
    thread; with several, each slice's exact sum is rounded before the slices are
    combined (exactly), so the result is within a few units in the last place."""
    import math
    lib = _load()
    if x.dtype == np.uint16:
        assert x.flags["C_CONTIGUOUS"], "x must be contiguous"
        jobs = [(lambda lo=lo, hi=hi: lib.orc_sum_sq_bf16(x.ctypes.data + 2 * lo, hi - lo))
                for lo, hi in _slices(x.shape[0], threads)]
        return math.fsum(_run(jobs, threads))
    _f32_inplace(x, "x", x.shape[0])
    jobs = [(lambda lo=lo, hi=hi: lib.orc_sum_sq_f32(x.ctypes.data + 4 * lo, hi - lo))
            for lo, hi in _slices(x.shape[0], threads)]
    return math.fsum(_run(jobs, threads))


def divergence_bound(h_norm, g_norms, weights, group_len, lr, mu):
    """Upper bound of ||w_after - w_before||_2 for a batch applied as
    len(group_len) server steps, from ||h0|| and the norms ||g|| of the committed
    updates in sequence (weights: one per committed update in sequence, or None)."""
    lib = _load()
    g = np.ascontiguousarray(g_norms, dtype=np.float64)
    gl = np.ascontiguousarray(group_len, dtype=np.int32)
    assert int(gl.sum()) == g.shape[0] and (gl >= 1).all(), "the groups must tile the sequence"
    wt = None
    if weights is not None:
        wt = np.ascontiguousarray(weights, dtype=np.float32)
        assert wt.shape[0] == g.shape[0]
    return lib.orc_divergence_bound(
        float(h_norm), g.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        wt.ctypes.data_as(ctypes.POINTER(ctypes.c_float)) if wt is not None else None,
        gl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), int(gl.shape[0]), float(lr), float(mu))


def sum_sq_diff(a, b, threads=1):
    """||a - b||_2^2 of two float32 vectors, the differences taken exactly."""
    import math
    lib = _load()
    _f32_inplace(a, "a", a.shape[0])
    _f32_inplace(b, "b", a.shape[0])
    jobs = [(lambda lo=lo, hi=hi: lib.orc_sum_sq_diff_f32(a.ctypes.data + 4 * lo,
                                                          b.ctypes.data + 4 * lo, hi - lo))
            for lo, hi in _slices(a.shape[0], threads)]
    return math.fsum(_run(jobs, threads))


def scatter_add(counts, totals, V, T, triples, threads=1):
    """Add (word, topic, delta) triples into counts[V*T] (and totals[T]), in
    place.  ``triples`` is a list of int32 arrays of shape (m, 3).  Returns the
    number of out-of-range triples that were skipped."""
    lib = _load()
    if counts.dtype != np.int32 or counts.size != V * T or (
            not counts.flags.c_contiguous):
        raise ValueError("counts must be contiguous int32 with V*T entries")
    if totals is not None and (totals.dtype != np.int32 or totals.shape != (T,)
                               or not totals.flags.c_contiguous):
        raise ValueError("totals must be contiguous int32[T]")
    for t in triples:
        if t.dtype != np.int32 or t.ndim != 2 or t.shape[1] != 3 or (
                not t.flags.c_contiguous):
            raise ValueError("each triple buffer must be contiguous int32[m,3]")
    K = len(triples)
    tab = _ptr_table(triples, 0) if K else (ctypes.c_void_p * 1)()
    nt = (ctypes.c_int64 * max(K, 1))(*[t.shape[0] for t in triples])
    tp = totals.ctypes.data if totals is not None else None
    threads = max(1, int(threads))
    rows = _slices(V, threads) or [(0, V)]
    cols = _slices(T, len(rows)) or [(0, T)]
    jobs = []
    for j, (lo, hi) in enumerate(rows):
        tlo, thi = cols[j] if j < len(cols) else (0, 0)
        jobs.append(lambda lo=lo, hi=hi, tlo=tlo, thi=thi, j=j: lib.orc_scatter_add(
            counts.ctypes.data, tp, V, T, tab, nt, K, lo, hi, tlo, thi,
            1 if j == 0 else 0))
    return int(sum(_run(jobs, threads)))


def touched_cells(V, T, triples, threads=1):
    """Number of distinct cells of the V x T matrix that the valid triples hit:
    scatter_add of the same triples with every delta replaced by 1 into a zero
    matrix, then the non-zero cells are counted.  (A measurement for the
    benchmark's byte count, not part of the method.)"""
    ones = []
    for t in triples:
        u = np.ascontiguousarray(t).copy()
        u[:, 2] = 1
        ones.append(u)
    counts = np.zeros(V * T, dtype=np.int32)
    scatter_add(counts, None, V, T, ones, threads=threads)
    return int(np.count_nonzero(counts))


def counts_add_dense(counts, totals, V, T, deltas, threads=1):
    """counts += sum of the workers' dense int32 V x T delta matrices, totals +=
    its column sums; in place.  ``deltas`` is a list of int32 arrays of V*T."""
    lib = _load()
    if counts.dtype != np.int32 or counts.size != V * T or not counts.flags.c_contiguous:
        raise ValueError("counts must be contiguous int32 with V*T entries")
    for dm in deltas:
        if dm.dtype != np.int32 or dm.size != V * T or not dm.flags.c_contiguous:
            raise ValueError("each delta matrix must be contiguous int32 with V*T entries")
    K = len(deltas)
    tab = _ptr_table(deltas, 0) if K else (ctypes.c_void_p * 1)()
    tp = totals.ctypes.data if totals is not None else None
    rows = _slices(V, max(1, int(threads))) or [(0, V)]
    cols = _slices(T, len(rows)) or [(0, T)]
    jobs = []
    for j, (lo, hi) in enumerate(rows):
        tlo, thi = cols[j] if j < len(cols) else (0, 0)
        jobs.append(lambda lo=lo, hi=hi, tlo=tlo, thi=thi: lib.orc_counts_add_dense(
            counts.ctypes.data, tp, V, T, tab, K, lo, hi, tlo, thi))
    _run(jobs, threads)
