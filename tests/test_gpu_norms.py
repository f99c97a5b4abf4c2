"""GPU parity of the norms fused into the aggregate / grouped-apply passes.

The data outputs (out, model, momentum) must equal the oracle's bit for bit, as
for the plain calls.  The norms are binary64 sums of exact squares taken in a
fixed tree order on the GPU, against the oracle's exactly rounded sums: each
lane adds at most a few hundred terms and the trees have about 30 levels, so
the two differ by well under 400 x 2^-53 ~ 5e-14 relative; the tests allow
1e-12.  The GPU's sums must also repeat bit for bit from run to run."""
import numpy as np
import pytest
import torch

import oracle
import paper_1907_00434_amd as mlf
import workloads as W
from parity import assert_same_bits

pytestmark = pytest.mark.gpu
RTOL = 1e-12


def close(got, ref):
    return abs(got - ref) <= RTOL * max(abs(ref), 1e-300)


def workspace(n):
    return torch.empty(mlf.mlf_norms_workspace_bytes(n), dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [1, 7, 257, 4099, 700_003])
def test_aggregate_norm(dtype, n):
    cfg = W.scaled(W.CONFIGS["cfg2"], n=n, K=5, dtype=dtype)
    d = W.dense_inputs(cfg, "cuda")
    ups_h = [W.to_host(u) for u in d["updates"]]
    out = torch.empty(n, device="cuda")
    norm = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    ws = workspace(n)
    mlf.mlf_aggregate_norm(d["updates"], d["order"], d["weights"], out, norm, ws)
    ref = oracle.aggregate(ups_h, d["order"], d["weights"])
    assert_same_bits(out, ref, "aggregate_norm out")
    first = norm.item()
    assert close(first, oracle.sum_sq(ref)), (first, oracle.sum_sq(ref))
    mlf.mlf_aggregate_norm(d["updates"], d["order"], d["weights"], out, norm, ws)
    assert norm.item() == first                     # reproducible bit for bit


def groups_for(M, seed):
    rng = np.random.default_rng(seed)
    lens, left = [1] * int(rng.integers(0, M)), 0
    left = M - len(lens)
    while left > 0:
        ln = int(rng.integers(1, left + 1))
        lens.append(ln)
        left -= ln
    return lens


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,K", [(1, 1), (9, 3), (4099, 8), (300_001, 16), (70_001, 33)])
def test_apply_grouped_norms(dtype, n, K):
    cfg = W.scaled(W.CONFIGS["cfg2"], n=n, K=K, dtype=dtype)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    d["weights"] = np.random.default_rng(K).uniform(0.1, 2.0, K).astype(np.float32)
    lens = groups_for(len(d["order"]), K * 7 + n)
    ups_h = [W.to_host(u) for u in d["updates"]]
    w0 = W.to_host(d["model"])
    w_h, h_h = w0.copy(), W.to_host(d["momentum"])
    oracle.apply_grouped(w_h, h_h, ups_h, d["order"], d["weights"], lens, d["lr"], d["mu"])
    norms = torch.full((2,), -1.0, dtype=torch.float64, device="cuda")
    model, momentum = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_grouped_norms(model, momentum, d["updates"], d["order"], d["weights"], lens,
                                d["lr"], d["mu"], norms, workspace(n))
    assert_same_bits(model, w_h, "model")
    assert_same_bits(momentum, h_h, "momentum")
    got = norms.cpu().numpy()
    assert close(got[0], oracle.sum_sq(h_h)), (got[0], oracle.sum_sq(h_h))
    assert close(got[1], oracle.sum_sq_diff(w_h, w0)), (got[1], oracle.sum_sq_diff(w_h, w0))


def test_norms_without_momentum_misaligned_and_empty():
    n = 50_001
    cfg = W.scaled(W.CONFIGS["cfg1"], n=n + 1, K=4)
    d = W.dense_inputs(cfg, "cuda")
    model = d["model"][1:].clone()[:n]            # aligned copy for the reference
    ups = [u[1:] for u in d["updates"]]           # misaligned views: element-wise path
    assert ups[0].data_ptr() % 16 != 0
    ups_h = [W.to_host(u) for u in ups]
    w0 = W.to_host(model)
    w_h = w0.copy()
    oracle.apply_grouped(w_h, None, ups_h, d["order"], d["weights"], [1, 3], d["lr"], 0.0)
    norms = torch.zeros(2, dtype=torch.float64, device="cuda")
    mlf.mlf_apply_grouped_norms(model, None, ups, d["order"], d["weights"], [1, 3], d["lr"], 0.0,
                                norms, workspace(n))
    assert_same_bits(model, w_h, "model")
    got = norms.cpu().numpy()
    assert got[0] == 0.0 and close(got[1], oracle.sum_sq_diff(w_h, w0))
    # nothing committed: model untouched, norms describe the state as it is
    h = torch.randn(n, device="cuda")
    before = model.clone()
    mlf.mlf_apply_grouped_norms(model, h, ups, [], None, [], 0.1, 0.9, norms, workspace(n))
    assert torch.equal(model, before)
    got = norms.cpu().numpy()
    assert close(got[0], oracle.sum_sq(W.to_host(h))) and got[1] == 0.0
    # n = 0: zeros
    norms.fill_(5.0)
    mlf.mlf_apply_grouped_norms(model, h, ups, d["order"], None, [4], 0.1, 0.9, norms,
                                workspace(0), n=0)
    assert norms.cpu().numpy().tolist() == [0.0, 0.0]


def test_norms_argument_checks():
    n = 100
    u = torch.ones(n, device="cuda")
    out = torch.empty(n, device="cuda")
    norm = torch.zeros(2, dtype=torch.float64, device="cuda")
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    assert mlf.mlf_aggregate_norm([u], [0], None, out, norm, small, check=False) == -1
    assert mlf.mlf_aggregate_norm([u], [0], None, out, norm, None, check=False) == -1
    assert mlf.mlf_apply_grouped_norms(out, None, [u], [0], None, [2], 0.1, 0.9, norm,
                                       workspace(n), check=False) == -1


def test_norms_at_full_size_resnet_batch():
    """cfg2 as a scheduled batch with the norms: data bit-exact, norms to 1e-12."""
    cfg = W.CONFIGS["cfg2"]
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    lens = [1] * 4 + [4, 8]
    ups_h = [W.to_host(u) for u in d["updates"]]
    w0 = W.to_host(d["model"])
    w_h, h_h = w0.copy(), W.to_host(d["momentum"])
    oracle.apply_grouped(w_h, h_h, ups_h, d["order"], d["weights"], lens, d["lr"], d["mu"], threads=16)
    norms = torch.zeros(2, dtype=torch.float64, device="cuda")
    mlf.mlf_apply_grouped_norms(d["model"], d["momentum"], d["updates"], d["order"], d["weights"],
                                lens, d["lr"], d["mu"], norms, workspace(cfg.n))
    assert_same_bits(d["model"], w_h, "model")
    assert_same_bits(d["momentum"], h_h, "momentum")
    got = norms.cpu().numpy()
    assert close(got[0], oracle.sum_sq(h_h, threads=16))
    assert close(got[1], oracle.sum_sq_diff(w_h, w0, threads=16))


# ---- exact server-replica divergence and replica catch-up -----------------------

@pytest.mark.parametrize("n", [1, 5, 1023, 1024, 1025, 70_001, 3_000_003])
def test_divergence(n):
    g = torch.Generator(device="cuda")
    g.manual_seed(n)
    a = torch.randn(n + 1, generator=g, device="cuda")
    b = a + torch.randn(n + 1, generator=g, device="cuda") * 1e-3
    dist = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    for off in (0, 1):                               # aligned, then element-wise path
        x, y = a[off:off + n], b[off:off + n]
        mlf.mlf_divergence(x, y, dist, workspace(n))
        ref = oracle.sum_sq_diff(W.to_host(x), W.to_host(y), threads=8)
        first = dist.item()
        assert close(first, ref), (off, first, ref)
        mlf.mlf_divergence(x, y, dist, workspace(n))
        assert dist.item() == first
    mlf.mlf_divergence(a, a, dist, workspace(n + 1))
    assert dist.item() == 0.0


def test_replica_lags_then_catches_up():
    """Sec. 3.3: the server is two updates ahead of the replica; the divergence
    is ||(g + g^2) h0 + (1 + g) u1 + u2||.  Replaying the same updates in the same
    order on the replica brings it to the identical model; replaying them swapped
    leaves gamma (u1 - u2)."""
    cfg = W.scaled(W.CONFIGS["cfg3"], n=200_003, K=2)
    d = W.dense_inputs(cfg, "cuda", momentum_init="random")
    ws = workspace(cfg.n)
    dist = torch.zeros(1, dtype=torch.float64, device="cuda")
    w_s, h_s = d["model"].clone(), d["momentum"].clone()
    w_r, h_r = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_ordered(w_s, h_s, d["updates"], [0, 1], d["lr"], d["mu"])
    mlf.mlf_divergence(w_s, w_r, dist, ws)
    g, lr = np.float64(np.float32(d["mu"])), np.float64(np.float32(d["lr"]))
    h0 = W.to_host(d["momentum"]).astype(np.float64)
    u1 = -lr * W.to_host(d["updates"][0]).astype(np.float64)
    u2 = -lr * W.to_host(d["updates"][1]).astype(np.float64)
    lead = (g + g * g) * h0 + (1 + g) * u1 + u2
    assert abs(dist.item() / float(np.sum(lead ** 2)) - 1) < 1e-4      # binary32 model rounding
    assert close(dist.item(), oracle.sum_sq_diff(W.to_host(w_s), W.to_host(w_r)))
    mlf.mlf_apply_ordered(w_r, h_r, d["updates"], [0, 1], d["lr"], d["mu"])   # catch up
    mlf.mlf_divergence(w_s, w_r, dist, ws)
    assert dist.item() == 0.0 and torch.equal(h_s, h_r)
    w_x, h_x = d["model"].clone(), d["momentum"].clone()
    mlf.mlf_apply_ordered(w_x, h_x, d["updates"], [1, 0], d["lr"], d["mu"])   # wrong order
    mlf.mlf_divergence(w_s, w_x, dist, ws)
    swapped = float(np.sum((g * (u1 - u2)) ** 2))
    assert dist.item() > 0 and abs(dist.item() / swapped - 1) < 1e-2


# ---- sizes above the small-input paths --------------------------------------------------

def test_divergence_several_tiles_per_workgroup():
    """17,000,005 elements: 16,602 tiles for the 8,192 workgroups of the 128-bit
    region, so workgroups take two or three tiles each, plus the ragged tail; the
    same path the benchmark times on 61 M elements."""
    n = 17_000_005
    g = torch.Generator(device="cuda")
    g.manual_seed(4242)
    a = torch.randn(n, generator=g, device="cuda")
    b = a + torch.randn(n, generator=g, device="cuda") * 1e-3
    dist = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    ws = workspace(n)
    mlf.mlf_divergence(a, b, dist, ws)
    first = dist.item()
    ref = oracle.sum_sq_diff(W.to_host(a), W.to_host(b), threads=16)
    assert close(first, ref), (first, ref)
    ws.fill_(0xff)                                    # the scratch's old contents do not matter
    mlf.mlf_divergence(a, b, dist, ws)
    assert dist.item() == first


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_aggregate_norm_two_stage_reduction(dtype):
    # (partial sums are reduced in two launches from 16,384 pairs on)
    n = 17_000_005                                    # 33,204 partial pairs
    cfg = W.scaled(W.CONFIGS["cfg2"], n=n, K=3, dtype=dtype)
    d = W.dense_inputs(cfg, "cuda")
    ups_h = [W.to_host(u) for u in d["updates"]]
    out = torch.empty(n, device="cuda")
    norm = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    ws = workspace(n)
    mlf.mlf_aggregate_norm(d["updates"], d["order"], d["weights"], out, norm, ws)
    ref = oracle.aggregate(ups_h, d["order"], d["weights"], threads=16)
    assert_same_bits(out, ref, "aggregate_norm out")
    first = norm.item()
    assert close(first, oracle.sum_sq(ref, threads=16)), (first, oracle.sum_sq(ref, threads=16))
    ws.fill_(0xff)
    mlf.mlf_aggregate_norm(d["updates"], d["order"], d["weights"], out, norm, ws)
    assert norm.item() == first
