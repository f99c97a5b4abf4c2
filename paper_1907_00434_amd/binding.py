"""ctypes binding of libmlfabric_hip.so: same names as the C ABI, argument
marshalling only.  torch is used for device memory and the current stream.

There is no fallback: if the HIP library cannot be loaded the calls raise.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

from . import build as _build

MLF_MAX_K = 64
MLF_STATIC_MAX_N = 1 << 28
MLF_OK, MLF_EINVAL, MLF_EALIGN, MLF_EUNSUPPORTED, MLF_EHIP = 0, -1, -2, -3, -4
MLF_F32, MLF_BF16 = 0, 1

_c = ctypes
_lib = None


class MlfError(RuntimeError):
    def __init__(self, status: int):
        self.status = int(status)
        super().__init__(mlf_status_string(status))


def library_path() -> str:
    return _build.LIB


def raw():
    """The loaded ctypes library (built first if no built copy is there)."""
    global _lib
    if _lib is not None:
        return _lib
    if not _build.is_built():
        _build.build()
    lib = _c.CDLL(_build.LIB)
    vpp = _c.POINTER(_c.c_void_p)
    i32p = _c.POINTER(_c.c_int32)
    f32p = _c.POINTER(_c.c_float)
    lib.mlf_aggregate.argtypes = [vpp, _c.c_int, _c.c_int64, _c.c_int, i32p, _c.c_int,
                                  f32p, _c.c_void_p, _c.c_void_p]
    lib.mlf_aggregate.restype = _c.c_int
    lib.mlf_apply_ordered.argtypes = [_c.c_void_p, _c.c_void_p, vpp, _c.c_int, _c.c_int64,
                                      _c.c_int, i32p, _c.c_int, _c.c_float, _c.c_float,
                                      _c.c_void_p]
    lib.mlf_apply_ordered.restype = _c.c_int
    lib.mlf_aggregate_apply.argtypes = [_c.c_void_p, _c.c_void_p, _c.c_void_p, vpp, _c.c_int,
                                        _c.c_int64, _c.c_int, i32p, _c.c_int, f32p,
                                        _c.c_float, _c.c_float, _c.c_void_p]
    lib.mlf_aggregate_apply.restype = _c.c_int
    lib.mlf_apply_grouped.argtypes = [_c.c_void_p, _c.c_void_p, vpp, _c.c_int, _c.c_int64,
                                      _c.c_int, i32p, _c.c_int, f32p, i32p, _c.c_int,
                                      _c.c_float, _c.c_float, _c.c_void_p]
    lib.mlf_apply_grouped.restype = _c.c_int
    lib.mlf_norms_workspace_bytes.argtypes = [_c.c_int64]
    lib.mlf_norms_workspace_bytes.restype = _c.c_size_t
    lib.mlf_aggregate_norm.argtypes = [vpp, _c.c_int, _c.c_int64, _c.c_int, i32p, _c.c_int,
                                       f32p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                       _c.c_size_t, _c.c_void_p]
    lib.mlf_aggregate_norm.restype = _c.c_int
    lib.mlf_apply_grouped_norms.argtypes = [_c.c_void_p, _c.c_void_p, vpp, _c.c_int, _c.c_int64,
                                            _c.c_int, i32p, _c.c_int, f32p, i32p, _c.c_int,
                                            _c.c_float, _c.c_float, _c.c_void_p, _c.c_void_p,
                                            _c.c_size_t, _c.c_void_p]
    lib.mlf_apply_grouped_norms.restype = _c.c_int
    lib.mlf_update_norms_workspace_bytes.argtypes = [_c.c_int64]
    lib.mlf_update_norms_workspace_bytes.restype = _c.c_size_t
    lib.mlf_aggregate_update_norms.argtypes = [vpp, _c.c_int, _c.c_int64, _c.c_int, i32p, _c.c_int,
                                               f32p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                               _c.c_void_p, _c.c_size_t, _c.c_void_p]
    lib.mlf_aggregate_update_norms.restype = _c.c_int
    lib.mlf_apply_grouped_update_norms.argtypes = [_c.c_void_p, _c.c_void_p, vpp, _c.c_int,
                                                   _c.c_int64, _c.c_int, i32p, _c.c_int, f32p,
                                                   i32p, _c.c_int, _c.c_float, _c.c_float,
                                                   _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                                   _c.c_size_t, _c.c_void_p]
    lib.mlf_apply_grouped_update_norms.restype = _c.c_int
    lib.mlf_divergence_bound.argtypes = [_c.c_double, _c.POINTER(_c.c_double), i32p, _c.c_int,
                                         _c.c_int, f32p, i32p, _c.c_int, _c.c_float, _c.c_float,
                                         _c.POINTER(_c.c_double)]
    lib.mlf_divergence_bound.restype = _c.c_int
    lib.mlf_divergence.argtypes = [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p,
                                   _c.c_void_p, _c.c_size_t, _c.c_void_p]
    lib.mlf_divergence.restype = _c.c_int
    lib.mlf_divergence_static.argtypes = [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p,
                                          _c.c_void_p]
    lib.mlf_divergence_static.restype = _c.c_int
    lib.mlf_sparse_scatter_add.argtypes = [_c.c_void_p, _c.c_void_p, _c.c_int32, _c.c_int32,
                                           vpp, _c.POINTER(_c.c_int64), _c.c_int,
                                           _c.c_void_p, _c.c_size_t, _c.c_void_p,
                                           _c.c_void_p]
    lib.mlf_sparse_scatter_add.restype = _c.c_int
    lib.mlf_counts_add_dense.argtypes = [_c.c_void_p, _c.c_void_p, _c.c_int32, _c.c_int32, vpp,
                                         _c.c_int, _c.c_void_p]
    lib.mlf_counts_add_dense.restype = _c.c_int
    lib.mlf_sparse_workspace_bytes.argtypes = [_c.c_int32, _c.c_int32, _c.c_int64]
    lib.mlf_sparse_workspace_bytes.restype = _c.c_size_t
    lib.mlf_status_string.argtypes = [_c.c_int]
    lib.mlf_status_string.restype = _c.c_char_p
    _lib = lib
    return lib


def mlf_status_string(status: int) -> str:
    return raw().mlf_status_string(int(status)).decode()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensors expected")
    return t.data_ptr()


def _dense_tables(updates, order, weights, n):
    K = len(updates)
    kind = None
    tab = (_c.c_void_p * max(K, 1))()
    for j, u in enumerate(updates):
        if u is None:
            tab[j] = None
            continue
        if u.dtype == torch.float32:
            k = MLF_F32
        elif u.dtype == torch.bfloat16:
            k = MLF_BF16
        else:
            raise TypeError("updates must be float32 or bfloat16")
        if kind is not None and k != kind:
            raise TypeError("all updates of a call share one dtype")
        kind = k
        if u.dim() != 1 or not u.is_contiguous() or u.numel() < n:
            raise ValueError("updates must be contiguous vectors of at least n elements")
        tab[j] = _ptr(u)
    if kind is None:
        kind = MLF_F32
    o = np.ascontiguousarray(np.asarray(order, dtype=np.int32).reshape(-1))
    op = o.ctypes.data_as(_c.POINTER(_c.c_int32))
    w = wp = None
    if weights is not None:
        w = np.ascontiguousarray(np.asarray(weights, dtype=np.float32).reshape(-1))
        if w.shape[0] != K:
            raise ValueError("weights must have one entry per worker")
        wp = w.ctypes.data_as(_c.POINTER(_c.c_float))
    return tab, K, kind, o, op, w, wp


def _state(t, n, name):
    if t is None:
        return
    if t.dtype != torch.float32 or t.dim() != 1 or not t.is_contiguous() or t.numel() < n:
        raise ValueError(f"{name} must be a contiguous float32 vector of at least n elements")


def _done(status, check):
    if check and status != MLF_OK:
        raise MlfError(status)
    return status


def mlf_aggregate(updates, order, weights, out, n=None, stream=None, check=True):
    """out[i] = sum_t weights[order[t]] * updates[order[t]][i], left to right."""
    n = out.numel() if n is None else int(n)
    _state(out, n, "out")
    tab, K, kind, o, op, w, wp = _dense_tables(updates, order, weights, n)
    st = raw().mlf_aggregate(tab, K, n, kind, op, len(o), wp, _ptr(out), _stream(stream))
    return _done(st, check)


def mlf_apply_ordered(model, momentum, updates, order, lr, mu, n=None, stream=None,
                      check=True):
    """Fold h <- mu h - lr g ; w <- w + h over the listed updates, in one pass."""
    n = model.numel() if n is None else int(n)
    _state(model, n, "model")
    _state(momentum, n, "momentum")
    tab, K, kind, o, op, _, _ = _dense_tables(updates, order, None, n)
    st = raw().mlf_apply_ordered(_ptr(model), _ptr(momentum), tab, K, n, kind, op, len(o),
                                 float(lr), float(mu), _stream(stream))
    return _done(st, check)


def mlf_aggregate_apply(model, momentum, out, updates, order, weights, lr, mu, n=None,
                        stream=None, check=True):
    """The ordered weighted sum, then one server step with it, fused."""
    n = model.numel() if n is None else int(n)
    _state(model, n, "model")
    _state(momentum, n, "momentum")
    _state(out, n, "out")
    tab, K, kind, o, op, w, wp = _dense_tables(updates, order, weights, n)
    st = raw().mlf_aggregate_apply(_ptr(model), _ptr(momentum), _ptr(out), tab, K, n, kind,
                                   op, len(o), wp, float(lr), float(mu), _stream(stream))
    return _done(st, check)


def mlf_apply_grouped(model, momentum, updates, order, weights, group_len, lr, mu, n=None,
                      stream=None, check=True):
    """Consecutive groups of the order, each summed and applied as one server
    step, in one pass (a directly forwarded update is a group of length 1)."""
    n = model.numel() if n is None else int(n)
    _state(model, n, "model")
    _state(momentum, n, "momentum")
    tab, K, kind, o, op, w, wp = _dense_tables(updates, order, weights, n)
    g = np.ascontiguousarray(np.asarray(group_len, dtype=np.int32).reshape(-1))
    gp = g.ctypes.data_as(_c.POINTER(_c.c_int32))
    st = raw().mlf_apply_grouped(_ptr(model), _ptr(momentum), tab, K, n, kind, op, len(o), wp,
                                 gp, len(g), float(lr), float(mu), _stream(stream))
    return _done(st, check)


def mlf_norms_workspace_bytes(n) -> int:
    return int(raw().mlf_norms_workspace_bytes(int(n)))


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def mlf_aggregate_norm(updates, order, weights, out, norm_sq, workspace, n=None, stream=None,
                       check=True):
    """mlf_aggregate, plus norm_sq[0] = sum of out^2 (float64 device tensor)."""
    n = out.numel() if n is None else int(n)
    _state(out, n, "out")
    if norm_sq.dtype != torch.float64 or norm_sq.numel() < 1:
        raise ValueError("norm_sq must be a float64 device tensor")
    tab, K, kind, o, op, w, wp = _dense_tables(updates, order, weights, n)
    st = raw().mlf_aggregate_norm(tab, K, n, kind, op, len(o), wp, _ptr(out), _ptr(norm_sq),
                                  _ptr(workspace), _nbytes(workspace), _stream(stream))
    return _done(st, check)


def mlf_apply_grouped_norms(model, momentum, updates, order, weights, group_len, lr, mu,
                            norms_sq, workspace, n=None, stream=None, check=True):
    """mlf_apply_grouped, plus norms_sq = [sum h_after^2, sum (w_after - w_before)^2]."""
    n = model.numel() if n is None else int(n)
    _state(model, n, "model")
    _state(momentum, n, "momentum")
    if norms_sq.dtype != torch.float64 or norms_sq.numel() < 2:
        raise ValueError("norms_sq must be a float64 device tensor of 2 elements")
    tab, K, kind, o, op, w, wp = _dense_tables(updates, order, weights, n)
    g = np.ascontiguousarray(np.asarray(group_len, dtype=np.int32).reshape(-1))
    gp = g.ctypes.data_as(_c.POINTER(_c.c_int32))
    st = raw().mlf_apply_grouped_norms(_ptr(model), _ptr(momentum), tab, K, n, kind, op, len(o),
                                       wp, gp, len(g), float(lr), float(mu), _ptr(norms_sq),
                                       _ptr(workspace), _nbytes(workspace), _stream(stream))
    return _done(st, check)


def mlf_update_norms_workspace_bytes(n) -> int:
    return int(raw().mlf_update_norms_workspace_bytes(int(n)))


def _update_norms_out(t, n_order):
    if t.dtype != torch.float64 or t.numel() < n_order:
        raise ValueError("update_norm_sq must be a float64 device tensor of len(order) elements")


def mlf_aggregate_update_norms(updates, order, weights, out, norm_sq, update_norm_sq, workspace,
                               n=None, stream=None, check=True):
    """mlf_aggregate_norm, plus update_norm_sq[t] = sum of updates[order[t]]^2."""
    n = out.numel() if n is None else int(n)
    _state(out, n, "out")
    if norm_sq.dtype != torch.float64 or norm_sq.numel() < 1:
        raise ValueError("norm_sq must be a float64 device tensor")
    tab, K, kind, o, op, w, wp = _dense_tables(updates, order, weights, n)
    _update_norms_out(update_norm_sq, len(o))
    st = raw().mlf_aggregate_update_norms(tab, K, n, kind, op, len(o), wp, _ptr(out), _ptr(norm_sq),
                                          _ptr(update_norm_sq), _ptr(workspace), _nbytes(workspace),
                                          _stream(stream))
    return _done(st, check)


def mlf_apply_grouped_update_norms(model, momentum, updates, order, weights, group_len, lr, mu,
                                   norms_sq, update_norm_sq, workspace, n=None, stream=None,
                                   check=True):
    """mlf_apply_grouped_norms, plus update_norm_sq[t] = sum of updates[order[t]]^2."""
    n = model.numel() if n is None else int(n)
    _state(model, n, "model")
    _state(momentum, n, "momentum")
    if norms_sq.dtype != torch.float64 or norms_sq.numel() < 2:
        raise ValueError("norms_sq must be a float64 device tensor of 2 elements")
    tab, K, kind, o, op, w, wp = _dense_tables(updates, order, weights, n)
    _update_norms_out(update_norm_sq, len(o))
    g = np.ascontiguousarray(np.asarray(group_len, dtype=np.int32).reshape(-1))
    gp = g.ctypes.data_as(_c.POINTER(_c.c_int32))
    st = raw().mlf_apply_grouped_update_norms(_ptr(model), _ptr(momentum), tab, K, n, kind, op,
                                              len(o), wp, gp, len(g), float(lr), float(mu),
                                              _ptr(norms_sq), _ptr(update_norm_sq), _ptr(workspace),
                                              _nbytes(workspace), _stream(stream))
    return _done(st, check)


def mlf_divergence_bound(h_norm_sq, update_norm_sq, order, K, weights, group_len, lr, mu,
                         check=True):
    """Upper bound of ||w_after - w_before||_2 for a batch (host arithmetic).  The
    norms are host values: update_norm_sq[t] belongs to updates[order[t]]."""
    u = np.ascontiguousarray(np.asarray(update_norm_sq, dtype=np.float64).reshape(-1))
    o = np.ascontiguousarray(np.asarray(order, dtype=np.int32).reshape(-1))
    g = np.ascontiguousarray(np.asarray(group_len, dtype=np.int32).reshape(-1))
    w = wp = None
    if weights is not None:
        w = np.ascontiguousarray(np.asarray(weights, dtype=np.float32).reshape(-1))
        if w.shape[0] != K:
            raise ValueError("weights must have one entry per worker")
        wp = w.ctypes.data_as(_c.POINTER(_c.c_float))
    if u.shape[0] != o.shape[0]:
        raise ValueError("one norm per committed update")
    out = _c.c_double(0.0)
    st = raw().mlf_divergence_bound(float(h_norm_sq), u.ctypes.data_as(_c.POINTER(_c.c_double)),
                                    o.ctypes.data_as(_c.POINTER(_c.c_int32)), len(o), int(K), wp,
                                    g.ctypes.data_as(_c.POINTER(_c.c_int32)), len(g), float(lr),
                                    float(mu), _c.byref(out))
    _done(st, check)
    return out.value if st == MLF_OK else None


def mlf_divergence(w_server, w_replica, dist_sq, workspace, n=None, stream=None, check=True):
    """dist_sq[0] = sum (w_server - w_replica)^2 (float64 device tensor)."""
    n = w_server.numel() if n is None else int(n)
    _state(w_server, n, "w_server")
    _state(w_replica, n, "w_replica")
    if dist_sq.dtype != torch.float64 or dist_sq.numel() < 1:
        raise ValueError("dist_sq must be a float64 device tensor")
    st = raw().mlf_divergence(_ptr(w_server), _ptr(w_replica), n, _ptr(dist_sq), _ptr(workspace),
                              _nbytes(workspace), _stream(stream))
    return _done(st, check)


def mlf_divergence_static(w_server, w_replica, dist_sq, n=None, stream=None, check=True):
    """mlf_divergence without a workspace (the library's own scratch array)."""
    n = w_server.numel() if n is None else int(n)
    _state(w_server, n, "w_server")
    _state(w_replica, n, "w_replica")
    if dist_sq.dtype != torch.float64 or dist_sq.numel() < 1:
        raise ValueError("dist_sq must be a float64 device tensor")
    st = raw().mlf_divergence_static(_ptr(w_server), _ptr(w_replica), n, _ptr(dist_sq),
                                     _stream(stream))
    return _done(st, check)


def mlf_sparse_workspace_bytes(V, T, total_triples) -> int:
    return int(raw().mlf_sparse_workspace_bytes(int(V), int(T), int(total_triples)))


def mlf_sparse_scatter_add(counts, totals, V, T, triples, workspace=None, n_rejected=None,
                           stream=None, check=True):
    """counts[word*T+topic] += delta and totals[topic] += delta for every
    (word, topic, delta) row of every int32 [m, 3] buffer in ``triples``."""
    if counts.dtype != torch.int32 or not counts.is_contiguous() or counts.numel() < V * T:
        raise ValueError("counts must be contiguous int32 with V*T entries")
    if totals is not None and (totals.dtype != torch.int32 or not totals.is_contiguous()
                               or totals.numel() < T):
        raise ValueError("totals must be contiguous int32 with T entries")
    K = len(triples)
    tab = (_c.c_void_p * max(K, 1))()
    cnt = (_c.c_int64 * max(K, 1))()
    for k, t in enumerate(triples):
        if t.dtype != torch.int32 or not t.is_contiguous() or t.numel() % 3 != 0:
            raise ValueError("each triple buffer must be contiguous int32 [m, 3]")
        tab[k] = _ptr(t)
        cnt[k] = t.numel() // 3
    ws_bytes = 0
    if workspace is not None:
        ws_bytes = workspace.numel() * workspace.element_size()
    st = raw().mlf_sparse_scatter_add(_ptr(counts), _ptr(totals), int(V), int(T), tab, cnt, K,
                                      _ptr(workspace), ws_bytes, _ptr(n_rejected),
                                      _stream(stream))
    return _done(st, check)


def mlf_counts_add_dense(counts, totals, V, T, deltas, stream=None, check=True):
    """counts += the sum of the workers' dense int32 V x T delta matrices and
    totals += its column sums."""
    if counts.dtype != torch.int32 or not counts.is_contiguous() or counts.numel() < V * T:
        raise ValueError("counts must be contiguous int32 with V*T entries")
    K = len(deltas)
    tab = (_c.c_void_p * max(K, 1))()
    for k, dm in enumerate(deltas):
        if dm.dtype != torch.int32 or not dm.is_contiguous() or dm.numel() < V * T:
            raise ValueError("each delta matrix must be contiguous int32 with V*T entries")
        tab[k] = _ptr(dm)
    st = raw().mlf_counts_add_dense(_ptr(counts), _ptr(totals), int(V), int(T), tab, K,
                                    _stream(stream))
    return _done(st, check)
