"""mlf_divergence_static -- the entry point for callers that cannot allocate --
called through the raw C ABI and checked against mlf_divergence (with a
workspace) on the same inputs: two calls in a row, the second on a smaller
input, so that what the first left in the library's scratch array cannot leak
into the second.  The results must be equal bit for bit (same kernels, same
order of the partial sums), and both are checked against the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1907_00434_amd as mlf
import workloads as W
from paper_1907_00434_amd import binding as B

pytestmark = pytest.mark.gpu


def _pair(n, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    a = torch.randn(n, generator=g, device="cuda")
    b = a + torch.randn(n, generator=g, device="cuda") * 1e-3
    return a, b


def _both(a, b, n):
    """(static, with workspace) squared distances through the C ABI."""
    lib = B.raw()
    stream = torch.cuda.current_stream().cuda_stream
    got = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    want = torch.full((1,), -2.0, dtype=torch.float64, device="cuda")
    st = lib.mlf_divergence_static(a.data_ptr(), b.data_ptr(), n, got.data_ptr(), stream)
    assert st == B.MLF_OK, mlf.mlf_status_string(st)
    ws = torch.empty(lib.mlf_norms_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    st = lib.mlf_divergence(a.data_ptr(), b.data_ptr(), n, want.data_ptr(), ws.data_ptr(),
                            ws.numel(), stream)
    assert st == B.MLF_OK, mlf.mlf_status_string(st)
    torch.cuda.synchronize()
    return got.item(), want.item()


def test_two_calls_in_a_row_second_smaller():
    # 17,000,005 elements: several tiles per workgroup, ragged tail; then 70,001
    # elements: one tile per workgroup, partial sums over a prefix of the same scratch.
    for n, seed in ((17_000_005, 11), (70_001, 12), (3, 13), (1_050_000, 14)):
        a, b = _pair(n, seed)
        got, want = _both(a, b, n)
        assert got == want, (n, got, want)
        ref = oracle.sum_sq_diff(W.to_host(a), W.to_host(b), threads=8)
        assert abs(got - ref) <= 1e-12 * abs(ref), (n, got, ref)
        del a, b


def test_unaligned_and_identical_vectors():
    a, b = _pair(300_002, 21)
    got, want = _both(a[1:], b[1:], 300_001)        # element-wise path
    assert got == want
    got, want = _both(a, a, 300_002)
    assert got == 0.0 and want == 0.0


def test_largest_accepted_size():
    """MLF_STATIC_MAX_N elements (2^28: 32 tiles per workgroup of the 128-bit region)."""
    n = B.MLF_STATIC_MAX_N
    a, b = _pair(n, 41)
    got, want = _both(a, b, n)
    assert got == want, (got, want)
    ref = oracle.sum_sq_diff(W.to_host(a), W.to_host(b), threads=16)
    assert abs(got - ref) <= 1e-12 * abs(ref), (got, ref)
    del a, b
    torch.cuda.empty_cache()


def test_size_limit_and_errors():
    lib = B.raw()
    a, b = _pair(16, 31)
    out = torch.zeros(1, dtype=torch.float64, device="cuda")
    big = B.MLF_STATIC_MAX_N + 1                     # rejected before anything is read
    assert lib.mlf_divergence_static(a.data_ptr(), b.data_ptr(), big, out.data_ptr(), None) == B.MLF_EUNSUPPORTED
    assert lib.mlf_divergence_static(None, b.data_ptr(), 16, out.data_ptr(), None) == B.MLF_EINVAL
    assert lib.mlf_divergence_static(a.data_ptr(), b.data_ptr(), -1, out.data_ptr(), None) == B.MLF_EINVAL
    assert lib.mlf_divergence_static(a.data_ptr() + 2, b.data_ptr(), 8, out.data_ptr(), None) == B.MLF_EALIGN
    assert lib.mlf_divergence_static(a.data_ptr(), b.data_ptr(), 0, out.data_ptr(), None) == B.MLF_OK
    torch.cuda.synchronize()
    assert out.item() == 0.0
