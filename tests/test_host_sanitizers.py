"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Two stand-alone drivers under tests/native/ are compiled and run here:

* san_oracle.c  -- the CPU oracle on exactly sized heap buffers (gcc);
* san_api.cpp   -- the host side of the C ABI: every argument check, handle lifetime,
                   the no-device error path, and the job partitioner on seeded ragged
                   populations against the invariants the kernel's indexing relies on
                   (hipcc; only the host pass is instrumented, kernels are stubbed out).

* tsan_api.cpp  -- contexts created, used and destroyed from four threads at once under
                   ThreadSanitizer (the registry of live handles is the shared state).

GPU code is not instrumented and no kernel is launched.
"""
from __future__ import annotations

import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
NATIVE = os.path.join(HERE, "native")

SAN_ENV = dict(os.environ,
               ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(exe):
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         env=SAN_ENV, timeout=300)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "ERROR: AddressSanitizer" not in res.stdout, res.stdout[-4000:]
    assert "runtime error" not in res.stdout, res.stdout[-4000:]
    return res.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "san_oracle")
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-g", "-ffp-contract=off",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-o", exe, os.path.join(NATIVE, "san_oracle.c"), "-lm"])
    assert "san_oracle: ok" in _run(exe)


def test_c_abi_host_side_under_sanitizers(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else shutil.which("hipcc")
    if not hipcc:
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "san_api")
    cmd = [hipcc, "-x", "hip", "--offload-arch=gfx950", "-std=c++17", "-O1", "-g",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2510_03760_amd", "csrc"),
           "-o", exe, os.path.join(NATIVE, "san_api.cpp")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "san_api: ok" in _run(exe)


def test_c_abi_handles_from_several_threads_under_tsan(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else shutil.which("hipcc")
    if not hipcc:
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "tsan_api")
    cmd = [hipcc, "-x", "hip", "--offload-arch=gfx950", "-std=c++17", "-O1", "-g",
           "-Xarch_host", "-fsanitize=thread",
           "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2510_03760_amd", "csrc"),
           "-o", exe, os.path.join(NATIVE, "tsan_api.cpp"), "-lpthread"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "ThreadSanitizer" not in run.stdout, run.stdout[-4000:]
    assert "tsan_api: ok" in run.stdout
