"""Compile libshm355.so -- and the application-kernel example that uses its device header -- for
gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
REPO_DIR = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libshm355.so")
SOURCES = [os.path.join(PKG_DIR, "csrc", "shm_api.hip")]
# the same library with release/acquire atomics on the signalling path: the signalling tests are run
# against it as a cross-check of the default build's relaxed atomics (tests/test_parity_full_release.py)
FULL_RELEASE_LIB_PATH = os.path.join(PKG_DIR, "libshm355_full_release.so")
EXAMPLE_LIB_PATH = os.path.join(PKG_DIR, "libshm355_user_example.so")
EXAMPLE_SOURCES = [os.path.join(PKG_DIR, "csrc", "shm_user_example.hip")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False) -> str:
    """Always compiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(REPO_DIR, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
           *SOURCES, "-o", LIB_PATH, "-L/opt/rocm/lib", "-lhsa-runtime64"]
    if verbose:
        print(" ".join(cmd), flush=True)
    variant = [hipcc, *HIPCC_FLAGS, "-DSHM_SIGNAL_FULL_RELEASE", "-I", os.path.join(REPO_DIR, "include"),
               "-I", os.path.join(PKG_DIR, "csrc"), *SOURCES, "-o", FULL_RELEASE_LIB_PATH, "-L/opt/rocm/lib", "-lhsa-runtime64"]
    if verbose:
        print(" ".join(variant), flush=True)
    procs = [subprocess.Popen(c, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True) for c in (cmd, variant)]
    for proc in procs:
        out, err = proc.communicate()
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out + err)
        if verbose and err.strip():
            print(err)
    # the example is an application of its own: device header only, no link to the library
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(PKG_DIR, "csrc"), *EXAMPLE_SOURCES, "-o", EXAMPLE_LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    return LIB_PATH


def ensure_built() -> None:
    """Compile only if nothing has been built yet (tests, the smoke check and the benchmark load what
    is there; the build driver always compiles)."""
    if not (os.path.exists(LIB_PATH) and os.path.exists(EXAMPLE_LIB_PATH) and os.path.exists(FULL_RELEASE_LIB_PATH)):
        build()


if __name__ == "__main__":
    print(build(verbose=True))
