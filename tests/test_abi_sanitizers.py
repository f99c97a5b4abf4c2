"""Host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer:
the library's host code is built with both (device code untouched) and linked
to a C driver (tests/native/abi_sanitize_main.c) that makes the argument checks
and scratch-size queries with invalid and extreme arguments.  Those return
before anything is enqueued, so no GPU is needed."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


@pytest.mark.skipif(not os.path.exists(HIPCC) or shutil.which("gcc") is None, reason="needs hipcc and gcc")
def test_host_code_of_the_library_is_clean_under_asan_and_ubsan(tmp_path):
    include = os.path.join(ROOT, "include")
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=all"]
    objects = []
    jobs = []
    for name in ("dense", "sparse"):
        obj = str(tmp_path / f"{name}.o")
        objects.append(obj)
        jobs.append(subprocess.Popen(
            [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san, "-I", include,
             "-c", os.path.join(ROOT, "paper_1907_00434_amd", "csrc", f"{name}.hip"), "-o", obj],
            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    main_obj = str(tmp_path / "main.o")
    gcc = subprocess.run(
        ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-I", include, "-c", os.path.join(ROOT, "tests", "native", "abi_sanitize_main.c"), "-o", main_obj],
        capture_output=True, text=True)
    assert gcc.returncode == 0, gcc.stderr
    for job in jobs:
        out, _ = job.communicate(timeout=900)
        assert job.returncode == 0, out
    exe = str(tmp_path / "abi_sanitize")
    link = subprocess.run(
        [HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
         *objects, main_obj, "-o", exe], capture_output=True, text=True)
    assert link.returncode == 0, link.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "abi sanitizer run: ok" in run.stdout
