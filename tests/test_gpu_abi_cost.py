"""The library called from a plain C program (no binding, no Python): the call
works through the C ABI alone, and its host cost per call is measured where it
matters, on the smallest configuration.  The program is built beforehand
(paper_1907_00434_amd.build.build_c_caller, part of the build entry point)."""
import json
import os
import subprocess

import pytest

from paper_1907_00434_amd import build as B

pytestmark = pytest.mark.gpu


def test_c_caller_runs_and_reports_its_host_cost():
    if not os.path.exists(B.C_CALLER):
        pytest.skip("tests/native/abi_call_cost was not built (run the build entry point first)")
    res = subprocess.run([B.C_CALLER], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    rec = json.loads(res.stdout.strip().splitlines()[-1])
    print("bare C ABI on cfg1:", rec)
    # generous ceilings: a call is argument checks plus one kernel launch
    assert 0 < rec["checks_only_us_per_call"] < 5
    assert 0 < rec["host_us_per_call"] < 60
    assert rec["us_per_call_until_done"] < 60
