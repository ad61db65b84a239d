"""Host-side check of the compiled device code: the long-message copy kernels must keep the
nontemporal hint on every 16-byte load and store.

Why this is a test: the compiler once peeled the first tile of the tile walk and its copies of that
tile's first loads came out as ordinary loads.  Nothing was wrong with the bytes, but a transfer
repeated on the same buffers then found an eighth of its source in the memory-side cache and measured
3-5 points of the HBM roofline more than a transfer of fresh data.  The walk's first tile is now a
compile-time case of its own; this test reads the assembly hipcc makes from the sources and fails if a
load or store in those kernels loses the hint again."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2409_20476_amd", "csrc")


@pytest.fixture(scope="module")
def kernels(tmp_path_factory):
    from paper_2409_20476_amd.build import HIPCC_FLAGS
    out = tmp_path_factory.mktemp("asm") / "shm_api.s"
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), *flags, "-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, os.path.join(CSRC, "shm_api.hip"), "-o", str(out)]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr[-2000:]
    text = out.read_text()
    bodies = {}
    for m in re.finditer(r"^(_Z\w+):.*?^\.Lfunc_end\d+:", text, re.M | re.S):
        bodies[m.group(1)] = m.group(0)
    return bodies


def _find(kernels, fragment):
    names = [k for k in kernels if fragment in k]
    assert names, f"no kernel named like {fragment}"
    return names


@pytest.mark.parametrize("fragment", ["shmk_wg_rma_tiles", "shmk_wg_put_timedILi1E", "shmk_wg_put_timedILi2E", "shmk_fcollect_vec", "shmk_broadcast", "shmk_reduce_sum_f32_vecILb1E", "shmk_collect", "shmk_reduceIfLi2ELb1E"])
def test_long_copies_keep_the_nontemporal_hint(kernels, fragment):
    for name in _find(kernels, fragment):
        body = kernels[name]
        loads = re.findall(r"global_load_dwordx4 [^\n]*", body)
        stores = re.findall(r"global_store_dwordx4 [^\n]*", body)
        assert len(loads) >= 4 and len(stores) >= 4, f"{name}: {len(loads)} loads, {len(stores)} stores"
        # write-through stores (sc1: the policy of short puts, deliberate) are the one other form allowed
        plain = [l for l in loads + stores if not re.search(r"\bnt\b", l) and not (l.startswith("global_store") and re.search(r"\bsc1\b", l))]
        assert not plain, f"{name}: {len(plain)} of {len(loads) + len(stores)} 16-byte accesses lost the nontemporal hint, e.g. {plain[0]}"
