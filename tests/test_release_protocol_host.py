"""CPU test of the protocol by which the work-groups of an XCD share one agent-scope release
(csrc/shm_release_algo.hpp, the same source the device code instantiates; paper section "Proposed
Device APIs": quiet completes the caller's puts).  A small C++ driver, built here with g++, runs the
protocol on CPU threads with std::atomic and a logical clock and checks, for every call, that a
write-back begun after the call's arrival finished before its return; a planted mistake must be
noticed; a second build runs the same under the thread sanitizer."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build_and_run(tmp_path, name, extra):
    exe = tmp_path / name
    cmd = ["g++", "-std=c++17", "-pthread", "-Wall", "-Wextra", "-Werror", *extra, f"-I{ROOT}/paper_2409_20476_amd/csrc",
           f"{ROOT}/tests/native/release_algo_driver.cpp", "-o", str(exe)]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    ran = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert ran.returncode == 0, ran.stdout + ran.stderr
    assert ran.stdout.strip().endswith("ok") and "ThreadSanitizer" not in ran.stderr, ran.stdout + ran.stderr


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_every_caller_is_covered_by_a_write_back_begun_after_it_arrived(tmp_path):
    _build_and_run(tmp_path, "release_algo_driver", ["-O2"])


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_the_same_under_the_thread_sanitizer(tmp_path):
    _build_and_run(tmp_path, "release_algo_tsan", ["-O1", "-g", "-fsanitize=thread"])
