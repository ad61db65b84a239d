"""Shared plumbing for the GPU parity tests: one GPU context and one oracle fed the same bytes."""
import numpy as np

from oracle.shmem_oracle import ShmemOracle
from paper_2409_20476_amd import shm as S


def make_pair(npes, heap_bytes):
    """A GPU context on torch memory/streams and an oracle with the same usable heap size."""
    g = S.Shm.on_torch(npes, heap_bytes)
    o = ShmemOracle(npes, g.heap_bytes())
    return g, o


def fill_random(g, o, seed, upto=None):
    """Same random bytes into the first `upto` bytes of every PE's heap on both sides."""
    n = upto or o.heap_bytes
    rng = np.random.default_rng(seed)
    for p in range(o.npes):
        data = rng.integers(0, 256, n, dtype=np.uint8)
        o.heap[p][:n] = data
        g.write(p, 0, data)


def write_both(g, o, pe, off, data):
    g.write(pe, off, data)
    o.write(pe, off, data)


def assert_heaps_equal(g, o, upto=None, what=""):
    n = upto or o.heap_bytes
    for p in range(o.npes):
        got = g.read(p, 0, n)
        want = o.heap[p][:n]
        if not np.array_equal(got, want):
            bad = np.flatnonzero(got != want)
            raise AssertionError(f"{what}: PE {p} differs at {bad.size} bytes, first at offset {bad[0]} "
                                 f"(got {got[bad[0]]}, want {want[bad[0]]})")
