"""CPU test of the reverse-offload proxy thread (paper section "Synchronization with Host"): a small
C++ driver, built here with g++, plays the GPU senders on CPU threads against the real proxy class --
ring wrap-around, scrambled arrival of message quarters, blocking and fire-and-forget requests,
completion-word reuse, the host-side quiet (wait_idle), stop taking what is left in the ring, restart."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir(os.path.join(ROCM, "include", "hsa")),
                    reason="needs g++ and the HSA headers")
def test_proxy_thread_serves_the_ring_protocol(tmp_path):
    exe = tmp_path / "proxy_ring_driver"
    cmd = ["g++", "-O2", "-std=c++17", "-pthread", "-Wall", "-Wextra", "-Werror",
           f"-I{ROCM}/include", f"-I{ROOT}/paper_2409_20476_amd/csrc",
           f"{ROOT}/tests/native/proxy_ring_driver.cpp", "-o", str(exe),
           f"-L{ROCM}/lib", "-lhsa-runtime64", f"-Wl,-rpath,{ROCM}/lib"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    ran = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert ran.returncode == 0, ran.stdout + ran.stderr
    assert ran.stdout.strip().endswith("ok")
