"""GPU parity: the LDA count-delta scatter-add against the CPU oracle; integer
work, so the bar is exact equality of every count and total."""
import numpy as np
import pytest
import torch

import paper_1907_00434_amd as mlf
import workloads as W
from parity import run_sparse

pytestmark = pytest.mark.gpu


def recipe(**kw):
    return W.scaled(W.CONFIGS["cfg5"], **kw)


@pytest.mark.parametrize("use_workspace", [False, True])
@pytest.mark.parametrize("init", ["zeros", "random"])
def test_scaled_lda_recipe(use_workspace, init):
    cfg = recipe(V=5003, T=1000, K=4, m=300_007)
    assert mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m) > 0
    d = W.sparse_inputs(cfg, "cuda", init=init, n_invalid=11)
    counts, totals = run_sparse(cfg, d, use_workspace)
    # totals stay the column sums of counts (they started consistent)
    col = counts.view(cfg.V, cfg.T).sum(dim=0, dtype=torch.int64).to(torch.int32)
    assert torch.equal(col, totals)


@pytest.mark.parametrize("use_workspace", [False, True])
def test_permuted_word_ids(use_workspace):
    cfg = recipe(V=20_011, T=257, K=3, m=200_001)
    assert mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m) > 0
    d = W.sparse_inputs(cfg, "cuda", init="random", permute_ids=True)
    run_sparse(cfg, d, use_workspace)


@pytest.mark.parametrize("use_workspace", [False, True])
@pytest.mark.parametrize("V,T,K,m", [(1, 1, 1, 1), (3, 2, 2, 5), (7, 1, 1, 1000), (2, 4099, 3, 777),
                                     (100, 3, 64, 129), (50_000, 17, 2, 65_536),
                                     (50_000, 17, 2, 400_000)])
def test_odd_shapes(use_workspace, V, T, K, m):
    cfg = recipe(V=V, T=T, K=K, m=m)
    d = W.sparse_inputs(cfg, "cuda", init="random", n_invalid=min(m, 5))
    run_sparse(cfg, d, use_workspace)


@pytest.mark.parametrize("V,T,K,m", [(1, 1, 1, 300_000), (3, 2, 2, 150_000), (32_769, 1, 1, 290_000),
                                     (1, 32_768, 2, 140_000), (7, 9_363, 3, 100_011),
                                     (4_099, 8, 1, 300_000), (2_100_000, 1, 2, 160_000),
                                     (16_385, 2_048, 2, 450_000), (5, 7, 2, 400_000)])
def test_binned_path_edge_shapes(V, T, K, m):
    """Shapes chosen around the binned path's geometry: one tile shared by
    several workgroups, a matrix that ends just past a tile boundary, many coarse
    ranges, and batches just above the size where the binned path starts."""
    cfg = recipe(V=V, T=T, K=K, m=m)
    d = W.sparse_inputs(cfg, "cuda", init="random", n_invalid=7)
    assert mlf.mlf_sparse_workspace_bytes(V, T, K * m) > 0
    run_sparse(cfg, d, True)


def test_shapes_the_binned_path_declines():
    # more than 2^30 cells: no scratch is asked for and the direct path serves
    assert mlf.mlf_sparse_workspace_bytes(140_000, 8_000, 100_000_000) == 0
    assert mlf.mlf_sparse_workspace_bytes(70_000, 8_000, 1_000_000) == 0     # batch too small for 17,090 tiles
    assert mlf.mlf_sparse_workspace_bytes(100, 100, 100) == 0        # tiny batch
    # small batches on a large matrix: the fixed cost per tile would dominate
    assert mlf.mlf_sparse_workspace_bytes(100_000, 1_000, 1_000_000) == 0
    assert mlf.mlf_sparse_workspace_bytes(100_000, 1_000, 4_000_000) > 0
    cfg = recipe(V=70_000, T=8_000, K=1, m=100_000)
    d = W.sparse_inputs(cfg, "cuda", init="zeros")
    run_sparse(cfg, d, True)


def test_matrix_of_more_than_16384_tiles():
    """2.4 GB of counts (18,311 tiles): the first pass keeps its histogram in a
    static LDS array, and the hot-tile bitmap is used beyond its first half."""
    cfg = recipe(V=600_000, T=1_000, K=6, m=2_000_000)
    assert mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m) > 0
    d = W.sparse_inputs(cfg, "cuda", init="zeros", permute_ids=True, n_invalid=5)
    run_sparse(cfg, d, True)
    del d
    torch.cuda.empty_cache()


@pytest.mark.parametrize("V,T", [(1_000_000, 1_000), (1_048_576, 1_024)])
def test_matrices_at_the_binned_paths_upper_limit(V, T):
    """30,518 tiles (4 GB of counts) and exactly 32,768 tiles = 2^30 cells, the
    most the binned path serves: histogram, plan tables and hot-tile bitmap at
    their full size.  Zero initial counts, permuted word ids, every cell compared."""
    cfg = recipe(V=V, T=T, K=8, m=2_600_000)
    assert mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m) > 0
    d = W.sparse_inputs(cfg, "cuda", init="zeros", permute_ids=True, n_invalid=5)
    run_sparse(cfg, d, True)
    del d
    torch.cuda.empty_cache()


def _misleading_batch(V, T, K, m, sampled_word_hi, other_word_lo, other_word_hi, seed):
    """Triples whose sampled blocks (every p-th block of 256, p as the header
    states) hit words below `sampled_word_hi` only, while all other blocks hit
    words in [other_word_lo, other_word_hi): the plan made from the sample is
    wrong about the rest of the batch."""
    tiles = (V * T + 32767) // 32768
    period = max(1, min(64, (K * m) // (256 * tiles)))
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    out = []
    for _ in range(K):
        block = torch.arange(m, device="cuda") // 256
        sampled = (block % period) == 0
        lo = torch.where(sampled, 0, other_word_lo)
        hi = torch.where(sampled, sampled_word_hi, other_word_hi)
        word = lo + (torch.rand(m, generator=g, device="cuda") * (hi - lo)).long().clamp_(max=V - 1)
        topic = torch.randint(0, T, (m,), generator=g, device="cuda")
        delta = torch.randint(0, 2, (m,), generator=g, device="cuda") * 2 - 1
        out.append(torch.stack([word, topic, delta], dim=1).to(torch.int32).contiguous())
    return out


@pytest.mark.parametrize("case", ["sample concentrated, bulk spread", "sample spread, bulk concentrated"])
def test_plan_made_from_a_misleading_sample(case):
    """The groups' room comes from a sample; records that find their group full
    are added to counts[] directly.  Here the sample is as wrong as it can be, at
    the coarse level (first case) and at both levels (second case: the bulk goes
    to a few tiles of one coarse range that the sample saw as lightly used), and
    the result must still equal the oracle's in every cell."""
    V, T, K, m = 160_000, 257, 2, 1_500_000               # 1,255 tiles, 10 coarse ranges
    cfg = recipe(V=V, T=T, K=K, m=m)
    assert mlf.mlf_sparse_workspace_bytes(V, T, K * m) > 0
    if case.startswith("sample concentrated"):
        triples = _misleading_batch(V, T, K, m, 100, 0, V, seed=1)
    else:
        triples = _misleading_batch(V, T, K, m, V, 40_000, 40_300, seed=2)
    d = W.sparse_inputs(recipe(V=V, T=T, K=1, m=8), "cuda", init="random")
    d["triples"] = triples
    run_sparse(cfg, d, True)


@pytest.mark.parametrize("use_workspace", [False, True])
def test_hand_case_ragged_buffers_and_optional_arguments(use_workspace, golden):
    g = {k: np.array([int(x) for x in v], dtype=np.int32)
         for k, v in golden("scatter_tiny.txt").items()}
    V, T = int(g["V"][0]), int(g["T"][0])
    counts = torch.from_numpy(g["counts0"].copy()).cuda()
    totals = torch.from_numpy(g["totals0"].copy()).cuda()
    tr = [torch.from_numpy(g["triples0"].reshape(-1, 3).copy()).cuda(),
          torch.zeros((0, 3), dtype=torch.int32, device="cuda"),          # an empty buffer
          torch.from_numpy(g["triples1"].reshape(-1, 3).copy()).cuda()]
    rej = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda") if use_workspace else None
    mlf.mlf_sparse_scatter_add(counts, totals, V, T, tr, workspace=ws, n_rejected=rej)
    assert counts.cpu().numpy().tolist() == g["counts"].tolist()
    assert totals.cpu().numpy().tolist() == g["totals"].tolist()
    assert rej.item() == int(g["rejected"][0])
    # totals and the reject counter are optional
    counts2 = torch.from_numpy(g["counts0"].copy()).cuda()
    mlf.mlf_sparse_scatter_add(counts2, None, V, T, tr, workspace=ws)
    assert torch.equal(counts, counts2)
    mlf.mlf_sparse_scatter_add(counts2, None, V, T, [])                   # nothing to do
    assert torch.equal(counts, counts2)


@pytest.mark.parametrize("use_workspace", [False, True])
def test_wraps_modulo_2_32_and_large_deltas(use_workspace):
    V, T = 4, 3
    counts = torch.tensor([2 ** 31 - 1] + [0] * (V * T - 1), dtype=torch.int32, device="cuda")
    totals = torch.tensor([2 ** 31 - 1, 0, 0], dtype=torch.int32, device="cuda")
    tr = torch.tensor([[0, 0, 1], [1, 1, -2 ** 31], [1, 1, -2 ** 31], [2, 2, 123456789],
                       [2, 2, 2 ** 31 - 1]], dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda") if use_workspace else None
    mlf.mlf_sparse_scatter_add(counts, totals, V, T, [tr], workspace=ws)
    c = counts.cpu().numpy()
    assert c[0] == -2 ** 31 and c[1 * T + 1] == 0
    assert c[2 * T + 2] == np.int32((123456789 + 2 ** 31 - 1) - 2 ** 32)
    assert totals.cpu().numpy().tolist() == [-2 ** 31, 0, int(c[2 * T + 2])]


@pytest.mark.parametrize("use_workspace", [False, True])
def test_many_topics_fall_back_to_global_totals(use_workspace):
    cfg = recipe(V=11, T=20_000, K=2, m=140_000)
    d = W.sparse_inputs(cfg, "cuda", init="zeros")
    assert mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m) > 0
    run_sparse(cfg, d, use_workspace)


# ---- the LDA update as dense delta matrices ---------------------------------------

def delta_matrices(V, T, K, seed, density=0.05):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    mats = []
    for _ in range(K):
        vals = torch.randint(-5, 6, (V * T,), generator=g, device="cuda", dtype=torch.int32)
        keep = torch.rand(V * T, generator=g, device="cuda") < density
        mats.append(torch.where(keep, vals, torch.zeros_like(vals)).contiguous())
    return mats


def run_dense_delta(V, T, mats, counts, totals, threads=16):
    import oracle
    c_h = W.to_host(counts)
    t_h = W.to_host(totals) if totals is not None else None
    oracle.counts_add_dense(c_h, t_h, V, T, [W.to_host(m) for m in mats], threads=threads)
    mlf.mlf_counts_add_dense(counts, totals, V, T, mats)
    assert np.array_equal(counts.cpu().numpy(), c_h), "counts differ"
    if totals is not None:
        assert np.array_equal(totals.cpu().numpy(), t_h), "totals differ"


@pytest.mark.parametrize("V,T,K", [(1, 1, 1), (3, 2, 2), (7, 5, 3), (301, 17, 8), (1000, 1000, 9),
                                   (4099, 257, 17), (50, 20_000, 2), (257, 129, 64)])
def test_dense_delta_matrices(V, T, K):
    g = torch.Generator(device="cuda")
    g.manual_seed(V * T + K)
    counts = torch.randint(0, 50, (V * T,), generator=g, device="cuda", dtype=torch.int32)
    totals = counts.view(V, T).sum(dim=0, dtype=torch.int64).to(torch.int32)
    run_dense_delta(V, T, delta_matrices(V, T, K, seed=K), counts, totals)
    col = counts.view(V, T).sum(dim=0, dtype=torch.int64).to(torch.int32)
    assert torch.equal(col, totals)


def test_dense_delta_misaligned_no_totals_and_wraparound():
    V, T, K = 123, 45, 3
    mats = delta_matrices(V, T + 1, K, seed=5, density=0.5)
    views = [m[1:1 + V * T] for m in mats]                      # 4-byte aligned only
    assert views[0].data_ptr() % 16 != 0
    counts = torch.full((V * T,), 2 ** 31 - 3, dtype=torch.int32, device="cuda")
    run_dense_delta(V, T, views, counts, None)
    mlf.mlf_counts_add_dense(counts, None, V, T, [])            # no workers: nothing happens


def test_dense_delta_equals_triple_scatter_on_the_gpu():
    cfg = recipe(V=2003, T=300, K=4, m=100_000)
    d = W.sparse_inputs(cfg, "cuda", init="random")
    mats = []
    for tr in d["triples"]:
        m = torch.zeros(cfg.V * cfg.T, dtype=torch.int32, device="cuda")
        m.index_put_((tr[:, 0].long() * cfg.T + tr[:, 1].long(),), tr[:, 2], accumulate=True)
        mats.append(m)
    c1, t1 = d["counts"].clone(), d["totals"].clone()
    mlf.mlf_sparse_scatter_add(c1, t1, cfg.V, cfg.T, d["triples"])
    c2, t2 = d["counts"].clone(), d["totals"].clone()
    mlf.mlf_counts_add_dense(c2, t2, cfg.V, cfg.T, mats)
    assert torch.equal(c1, c2) and torch.equal(t1, t2)


def test_dense_delta_full_matrix_size():
    """The LDA matrix of the sparse configuration (100,000 x 1,000), 8 workers."""
    cfg = W.CONFIGS["cfg5"]
    counts = torch.zeros(cfg.V * cfg.T, dtype=torch.int32, device="cuda")
    totals = torch.zeros(cfg.T, dtype=torch.int32, device="cuda")
    run_dense_delta(cfg.V, cfg.T, delta_matrices(cfg.V, cfg.T, 8, seed=11, density=0.02), counts, totals)
    torch.cuda.empty_cache()


@pytest.mark.parametrize("V,T,K", [(8193, 8192, 1), (8193, 8192, 3), (8193, 8192, 9), (16389, 4099, 17),
                                   (3400, 20_000, 2)])
def test_dense_delta_matrix_larger_than_the_cache(V, T, K):
    """More than 256 MiB of counts: the kernel takes its other shape (one-wavefront
    workgroups, every group written back, no-reuse hints), with one and with
    several blocks of 8 matrices, totals in LDS and (20,000 topics) in memory,
    a cell count that is not a multiple of 4, non-zero counts to start from."""
    assert 4 * V * T > 256 << 20
    g = torch.Generator(device="cuda")
    g.manual_seed(V + T + K)
    counts = torch.randint(-50, 50, (V * T,), generator=g, device="cuda", dtype=torch.int32)
    totals = torch.randint(0, 1000, (T,), generator=g, device="cuda", dtype=torch.int32)
    run_dense_delta(V, T, delta_matrices(V, T, K, seed=K, density=0.03), counts, totals)
    torch.cuda.empty_cache()


def test_dense_delta_larger_than_the_cache_misaligned_and_without_totals():
    V, T, K = 8193, 8192, 2
    mats = delta_matrices(V, T + 1, K, seed=6, density=0.2)
    views = [m[1:1 + V * T] for m in mats]                      # 4-byte aligned only: cell-wise region
    assert views[0].data_ptr() % 16 != 0
    counts = torch.full((V * T,), 2 ** 31 - 2, dtype=torch.int32, device="cuda")
    run_dense_delta(V, T, views, counts, None)
    torch.cuda.empty_cache()


@pytest.mark.parametrize("big", [511, -512, 512, -513, 1023, 2 ** 30, -2 ** 31])
def test_binned_path_record_formats(big):
    """Deltas in [-512, 512) travel as 4-byte records through the scratch, any
    other delta switches the whole call to 8-byte records: both sides of the
    boundary, and extreme values."""
    cfg = recipe(V=3001, T=500, K=3, m=100_000)
    assert mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m) > 0
    d = W.sparse_inputs(cfg, "cuda", init="random", n_invalid=3)
    for k, tr in enumerate(d["triples"]):
        tr[7 + k::997, 2] = big
        tr[11 + k::1499, 2] = -big if big != -2 ** 31 else 2 ** 31 - 1
    run_sparse(cfg, d, True)


@pytest.mark.parametrize("use_workspace", [False, True])
def test_counts_aligned_to_four_bytes_only(use_workspace):
    """counts (and totals) that are not 16-byte aligned: the merge of the tile
    images falls back to single cells."""
    cfg = recipe(V=700, T=333, K=2, m=140_000)
    assert mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m) > 0
    d = W.sparse_inputs(cfg, "cuda", init="random")
    big_c = torch.zeros(cfg.V * cfg.T + 3, dtype=torch.int32, device="cuda")
    big_t = torch.zeros(cfg.T + 3, dtype=torch.int32, device="cuda")
    big_c[1:1 + cfg.V * cfg.T] = d["counts"]
    big_t[3:3 + cfg.T] = d["totals"]
    d["counts"], d["totals"] = big_c[1:1 + cfg.V * cfg.T], big_t[3:3 + cfg.T]
    assert d["counts"].data_ptr() % 16 == 4
    counts_h, totals_h = W.to_host(d["counts"]), W.to_host(d["totals"])
    tr_h = [W.to_host(t) for t in d["triples"]]
    import oracle
    oracle.scatter_add(counts_h, totals_h, cfg.V, cfg.T, tr_h)
    ws = None
    if use_workspace:
        ws = torch.empty(mlf.mlf_sparse_workspace_bytes(cfg.V, cfg.T, cfg.K * cfg.m),
                         dtype=torch.uint8, device="cuda")
    mlf.mlf_sparse_scatter_add(d["counts"], d["totals"], cfg.V, cfg.T, d["triples"], workspace=ws)
    assert np.array_equal(d["counts"].cpu().numpy(), counts_h)
    assert np.array_equal(d["totals"].cpu().numpy(), totals_h)
    assert big_c[0].item() == 0 and big_c[-2:].abs().sum().item() == 0     # nothing outside
