"""Builds libefim.so (HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB_DIR = os.path.join(PKG, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libefim.so")
SOURCES = ["api.hip", "planner.cpp", "session_pool.cpp", "rope_append.hip", "extend_attention.hip"]
# measured-ceiling kernels of the benchmark: a library of their own, never part of libefim.so
CEILINGS_PATH = os.path.join(LIB_DIR, "libefim_ceilings.so")
CEILINGS_SOURCES = ["ceilings.hip"]


def hipcc_path():
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: libefim needs the ROCm toolchain to build")


def source_digest():
    """SHA-256 over every file the library is built from; compiled into the library so that a
    binary left over from older sources can be told from a current one."""
    import hashlib
    h = hashlib.sha256()
    names = [os.path.join(ROOT, "include", n) for n in sorted(os.listdir(os.path.join(ROOT, "include")))]
    names += [os.path.join(CSRC, n) for n in sorted(os.listdir(CSRC)) if n not in CEILINGS_SOURCES]
    for path in names:
        if os.path.isfile(path):
            h.update(os.path.basename(path).encode() + b"\0")
            with open(path, "rb") as fh:
                h.update(fh.read())
    return h.hexdigest()


def build_library(verbose=False, extra_flags=()):
    """Compile every source of the library for gfx950 and link libefim.so."""
    os.makedirs(LIB_DIR, exist_ok=True)
    cmd = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wno-unused-command-line-argument",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        '-DEFIM_SOURCE_DIGEST="%s"' % source_digest(),
    ]
    cmd += list(extra_flags)
    for s in SOURCES:
        if s.endswith(".cpp"):
            cmd += ["-x", "hip", os.path.join(CSRC, s)]
        else:
            cmd += [os.path.join(CSRC, s)]
    cmd += ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB_PATH


def build_ceilings(verbose=False):
    """Compile the benchmark's measured-ceiling kernels (libefim_ceilings.so)."""
    os.makedirs(LIB_DIR, exist_ok=True)
    cmd = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wno-unused-command-line-argument",
    ]
    cmd += [os.path.join(CSRC, s) for s in CEILINGS_SOURCES] + ["-o", CEILINGS_PATH]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return CEILINGS_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_ceilings(verbose=True))
