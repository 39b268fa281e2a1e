"""The host side of the library (planner, session pool) under AddressSanitizer and UBSan: the two
drivers in tests/native/ push random inputs through the C++ code compiled by g++ with the
sanitizers on, and check coverage / consistency properties on the way.  No GPU, no HIP runtime
(only its headers, for the types the internal header names)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_21889_amd", "csrc")
NATIVE = os.path.join(ROOT, "tests", "native")
FLAGS = ["-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]


def _build_and_run(tmp_path, name, sources, extra):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("g++ not available")
    exe = str(tmp_path / name)
    cmd = [gxx] + FLAGS + extra + ["-I", os.path.join(ROOT, "include"), "-I", CSRC] + sources + ["-o", exe, "-lpthread"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)   # the sanitizer runtime has to come first in the link order
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    return run.stdout


def test_planner_under_sanitizers(tmp_path):
    hip_include = "/opt/rocm/include"
    if not os.path.exists(os.path.join(hip_include, "hip", "hip_runtime.h")):
        pytest.skip("HIP headers not available")
    out = _build_and_run(tmp_path, "fuzz_planner",
                         [os.path.join(NATIVE, "fuzz_planner.cpp"), os.path.join(CSRC, "planner.cpp")],
                         ["-D__HIP_PLATFORM_AMD__", "-I", hip_include])
    assert "planner ok" in out


def test_session_pool_under_sanitizers(tmp_path):
    out = _build_and_run(tmp_path, "fuzz_pool",
                         [os.path.join(NATIVE, "fuzz_pool.cpp"), os.path.join(CSRC, "session_pool.cpp")], [])
    assert "session pool ok" in out
