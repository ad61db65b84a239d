"""The signalling path against its textbook form.

The library publishes a payload with write-through stores, a wait for their acknowledgement and
RELAXED agent-scope atomics on the arrival counters and the signal word (paper section "Proposed
Device APIs": put-with-signal orders the signal after its own payload only).  The same sources built
with -DSHM_SIGNAL_FULL_RELEASE use acquire-release / release atomics there instead.  This test runs
the put-with-signal, wait, ring and ping-pong parity tests in a child process that loads that
second library: both builds must agree with the oracle bit for bit.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_signalling_tests_pass_on_the_release_acquire_build():
    if os.environ.get("SHM355_LIBRARY_VARIANT"):
        pytest.skip("already running against a library variant")
    env = dict(os.environ, SHM355_LIBRARY_VARIANT="full_release")
    files = ["tests/test_parity_c1.py", "tests/test_parity_signal_amo.py", "tests/test_parity_ring_collectives.py",
             "tests/test_zz_no_alloc.py"]
    proc = subprocess.run([sys.executable, "-u", "-m", "pytest", "-x", "-q", "-m", "gpu", "--timeout", "120", "--timeout-method", "thread",
                           "-p", "no:cacheprovider", *files], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = "\n".join((proc.stdout + proc.stderr).splitlines()[-25:])
    assert proc.returncode == 0, tail
    assert " passed" in proc.stdout and "libshm355_full_release.so" in _loaded_libraries_note(env), tail


def _loaded_libraries_note(env):
    """Which library a process with that environment loads (asked of the binding, no GPU needed)."""
    code = ("import ctypes, os\n"
            "from paper_2409_20476_amd import shm\n"
            "lib = shm.load_library()\n"
            "print(lib._name)\n")
    return subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=120).stdout
