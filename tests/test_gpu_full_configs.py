"""GPU parity at the full sizes of the five benchmark configurations, in the
launch configuration the benchmark times.  The threaded oracle is fast enough
to check EVERY output element, so nothing is sampled."""
import pytest
import torch

import workloads as W
from parity import run_dense, run_sparse

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4"])
def test_dense_config_full_size(name):
    cfg = W.CONFIGS[name]
    d = W.dense_inputs(cfg, "cuda")
    run_dense(cfg.call, d, want_out=False)
    del d
    torch.cuda.empty_cache()


@pytest.mark.parametrize("use_workspace", [True, False])
def test_sparse_config_full_size(use_workspace):
    cfg = W.CONFIGS["cfg5"]
    d = W.sparse_inputs(cfg, "cuda")
    counts, totals = run_sparse(cfg, d, use_workspace)
    col = counts.view(cfg.V, cfg.T).sum(dim=0, dtype=torch.int64).to(torch.int32)
    assert torch.equal(col, totals)
    del d
    torch.cuda.empty_cache()


def test_sparse_config_full_size_permuted_ids():
    cfg = W.CONFIGS["cfg5"]
    d = W.sparse_inputs(cfg, "cuda", permute_ids=True)
    run_sparse(cfg, d, True)
