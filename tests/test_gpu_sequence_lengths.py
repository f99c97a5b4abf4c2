"""Every dense call on streamed state (model + momentum above 256 MiB) for EVERY
number of committed updates from 1 to 40, binary32 updates, against the oracle
bit for bit.

Why every length: the kernels consume the sequence in double-buffered blocks of
8 updates and a halving remainder (4, 2, 1), so the code a launch runs through
is chosen by the parity of the number of whole blocks and by the three bits of
the remainder; from 8 (4 for the plain aggregate, 16 for the update-norm
variants) committed updates on, the binary32 kernels also change to their narrow
launch shape, which is a separate set of instantiations, and the number of
workgroups per compute unit they are launched with changes at 8, 9, 16, 17 and
24.  16 .. 31 covers every combination of block parity and remainder, 32 .. 40
repeats the loop, 1 .. 15 does the same across the change of shape.  The
compiler has produced wrong code for other instantiations of this template (a
register still holding loaded data reused as a temporary, under an occupancy
attribute the library no longer uses), always on every tile of the launch: a
test per path is what guards the instantiations that ship.

The norms variants share the data path: their model / momentum / output must be
the same bits, their norms within 1e-12 of the oracle's exactly rounded sums."""
import numpy as np
import pytest
import torch

import oracle
import paper_1907_00434_amd as mlf
import workloads as W
from parity import assert_same_bits

pytestmark = pytest.mark.gpu

K = 40
N = 33_554_432 + 1_005          # model + momentum = 256 MiB + 8 KB: streamed; ragged tail
N_BIG = 67_108_864 + 1_005      # a model alone above 256 MiB: streamed without momentum
THREADS = 16
RTOL = 1e-12


def close(got, ref):
    return abs(got - ref) <= RTOL * max(abs(ref), 1e-300)


def group_lengths(M):
    """A directly forwarded prefix, then groups whose ends fall inside and across
    the blocks of 8."""
    lens = []
    for ln in (1, 1, 1, 5, 7, 2, 9):
        if sum(lens) + ln > M:
            break
        lens.append(ln)
    if sum(lens) < M:
        lens.append(M - sum(lens))
    return lens


@pytest.fixture(scope="module")
def batch():
    cfg = W.scaled(W.CONFIGS["cfg3"], n=N, K=K)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    d["ups_h"] = [W.to_host(u) for u in d["updates"]]
    d["w_h"], d["h_h"] = W.to_host(d["model"]), W.to_host(d["momentum"])
    d["weights"] = np.random.default_rng(40).uniform(0.25, 1.5, K).astype(np.float32)
    d["update_sq"] = [oracle.sum_sq(u, threads=THREADS) for u in d["ups_h"]]
    d["norms_ws"] = torch.empty(mlf.mlf_norms_workspace_bytes(N), dtype=torch.uint8, device="cuda")
    d["update_norms_ws"] = torch.empty(mlf.mlf_update_norms_workspace_bytes(N), dtype=torch.uint8,
                                       device="cuda")
    yield d
    del d
    torch.cuda.empty_cache()


@pytest.mark.parametrize("M", range(1, K + 1))
def test_apply_ordered_every_length(batch, M):
    d, order = batch, batch["order"][:M]
    w, h = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_ordered(w, h, d["updates"], order, d["lr"], d["mu"])
    w_h, h_h = d["w_h"].copy(), d["h_h"].copy()
    oracle.apply_ordered(w_h, h_h, d["ups_h"], order, d["lr"], d["mu"], threads=THREADS)
    assert_same_bits(w, w_h, "model")
    assert_same_bits(h, h_h, "momentum")


@pytest.mark.parametrize("M", range(1, K + 1))
def test_grouped_apply_and_its_norms_every_length(batch, M):
    d, order, lens = batch, batch["order"][:M], group_lengths(M)
    w_h, h_h = d["w_h"].copy(), d["h_h"].copy()
    oracle.apply_grouped(w_h, h_h, d["ups_h"], order, d["weights"], lens, d["lr"], d["mu"],
                         threads=THREADS)
    h_sq = oracle.sum_sq(h_h, threads=THREADS)
    dw_sq = oracle.sum_sq_diff(w_h, d["w_h"], threads=THREADS)

    w, h = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_grouped(w, h, d["updates"], order, d["weights"], lens, d["lr"], d["mu"])
    assert_same_bits(w, w_h, "grouped: model")
    assert_same_bits(h, h_h, "grouped: momentum")

    norms = torch.full((2,), -1.0, dtype=torch.float64, device="cuda")
    w.copy_(d["model"]); h.copy_(d["momentum"])
    mlf.mlf_apply_grouped_norms(w, h, d["updates"], order, d["weights"], lens, d["lr"], d["mu"], norms,
                                d["norms_ws"])
    assert_same_bits(w, w_h, "grouped + norms: model")
    assert_same_bits(h, h_h, "grouped + norms: momentum")
    got = norms.cpu().numpy()
    assert close(got[0], h_sq) and close(got[1], dw_sq), (got, h_sq, dw_sq)

    norms.fill_(-1.0)
    per_update = torch.full((M,), -1.0, dtype=torch.float64, device="cuda")
    w.copy_(d["model"]); h.copy_(d["momentum"])
    mlf.mlf_apply_grouped_update_norms(w, h, d["updates"], order, d["weights"], lens, d["lr"], d["mu"],
                                       norms, per_update, d["update_norms_ws"])
    assert_same_bits(w, w_h, "grouped + update norms: model")
    assert_same_bits(h, h_h, "grouped + update norms: momentum")
    got, got_updates = norms.cpu().numpy(), per_update.cpu().numpy()
    assert close(got[0], h_sq) and close(got[1], dw_sq), (got, h_sq, dw_sq)
    for t, j in enumerate(order):
        assert close(got_updates[t], d["update_sq"][int(j)]), (t, got_updates[t], d["update_sq"][int(j)])


@pytest.mark.parametrize("M", range(1, K + 1))
def test_aggregate_calls_every_length(batch, M):
    d, order = batch, batch["order"][:M]
    w_h, h_h = d["w_h"].copy(), d["h_h"].copy()
    ref = oracle.aggregate_apply(w_h, h_h, d["ups_h"], order, d["weights"], d["lr"], d["mu"],
                                 want_out=True, threads=THREADS)
    ref_sq = oracle.sum_sq(ref, threads=THREADS)

    # with momentum, and (model + output above 256 MiB) without
    w, h = d["model"].clone(), d["momentum"].clone()
    out = torch.empty(N, device="cuda")
    mlf.mlf_aggregate_apply(w, h, out, d["updates"], order, d["weights"], d["lr"], d["mu"])
    assert_same_bits(out, ref, "aggregate+apply: aggregate")
    assert_same_bits(w, w_h, "aggregate+apply: model")
    assert_same_bits(h, h_h, "aggregate+apply: momentum")
    del h
    w.copy_(d["model"]); out.fill_(-1.0)
    mlf.mlf_aggregate_apply(w, None, out, d["updates"], order, d["weights"], d["lr"], 0.0)
    w_plain = d["w_h"].copy()
    oracle.aggregate_apply(w_plain, None, d["ups_h"], order, d["weights"], d["lr"], 0.0, threads=THREADS)
    assert_same_bits(out, ref, "aggregate+apply without momentum: aggregate")
    assert_same_bits(w, w_plain, "aggregate+apply without momentum: model")
    del w

    out.fill_(-1.0)
    mlf.mlf_aggregate(d["updates"], order, d["weights"], out)
    assert_same_bits(out, ref, "aggregate")

    norm = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    out.fill_(-1.0)
    mlf.mlf_aggregate_norm(d["updates"], order, d["weights"], out, norm, d["norms_ws"])
    assert_same_bits(out, ref, "aggregate + norm")
    assert close(norm.item(), ref_sq), (norm.item(), ref_sq)

    norm.fill_(-1.0)
    per_update = torch.full((M,), -1.0, dtype=torch.float64, device="cuda")
    out.fill_(-1.0)
    mlf.mlf_aggregate_update_norms(d["updates"], order, d["weights"], out, norm, per_update,
                                   d["update_norms_ws"])
    assert_same_bits(out, ref, "aggregate + update norms")
    assert close(norm.item(), ref_sq), (norm.item(), ref_sq)
    got_updates = per_update.cpu().numpy()
    for t, j in enumerate(order):
        assert close(got_updates[t], d["update_sq"][int(j)]), (t, got_updates[t], d["update_sq"][int(j)])


@pytest.fixture(scope="module")
def big_batch():
    cfg = W.scaled(W.CONFIGS["cfg3"], n=N_BIG, K=32)
    d = W.dense_inputs(cfg, "cuda")
    d["ups_h"] = [W.to_host(u) for u in d["updates"]]
    d["w_h"] = W.to_host(d["model"])
    d["weights"] = np.random.default_rng(41).uniform(0.25, 1.5, 32).astype(np.float32)
    yield d
    del d
    torch.cuda.empty_cache()


@pytest.mark.parametrize("M", range(16, 32))
def test_plain_sgd_streamed_every_path(big_batch, M):
    """No momentum vector: the other half of the apply instantiations.  The state
    is the model alone, so it takes 64 Mi elements to be streamed."""
    d, order, lens = big_batch, big_batch["order"][:M], group_lengths(M)
    w = d["model"].clone()
    mlf.mlf_apply_ordered(w, None, d["updates"], order, d["lr"], 0.0)
    w_h = d["w_h"].copy()
    oracle.apply_ordered(w_h, None, d["ups_h"], order, d["lr"], 0.0, threads=THREADS)
    assert_same_bits(w, w_h, "ordered apply: model")
    w.copy_(d["model"])
    mlf.mlf_apply_grouped(w, None, d["updates"], order, d["weights"], lens, d["lr"], 0.0)
    w_h = d["w_h"].copy()
    oracle.apply_grouped(w_h, None, d["ups_h"], order, d["weights"], lens, d["lr"], 0.0, threads=THREADS)
    assert_same_bits(w, w_h, "grouped apply: model")
