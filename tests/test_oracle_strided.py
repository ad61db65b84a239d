"""Pins for the oracle's strided put/get: a hand-worked example, numpy slicing, reduction to the
contiguous put, inverse pairs and argument errors."""
import os

import numpy as np
import pytest

from oracle.shmem_oracle import OracleError, ShmemOracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "strided_example.txt")


def test_golden_worked_example():
    want = np.array([l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")][0], dtype=np.uint16)
    o = ShmemOracle(2, 4096)
    o.write(0, 0, np.arange(10, 20, dtype=np.uint16).view(np.uint8))
    o.iput(0, 4, 2, 3, 2, 4, 2, 1)
    assert np.array_equal(o.read(1, 0, 28).view(np.uint16), want)
    assert not o.heap[1][28:].any()


@pytest.mark.parametrize("elem", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("dst_stride,src_stride,n", [(1, 1, 100), (3, 1, 57), (1, 5, 33), (7, 2, 41), (2, 2, 1), (4, 4, 0)])
def test_matches_numpy_slicing(elem, dst_stride, src_stride, n):
    rng = np.random.default_rng(elem * 100 + n)
    o = ShmemOracle(3, 1 << 15)
    for p in range(3):
        o.heap[p][:] = rng.integers(0, 256, 1 << 15, dtype=np.uint8)
    before = [h.copy() for h in o.heap]
    src, dst = 16 * 3, 8192 + 16
    o.iput(2, dst, src, dst_stride, src_stride, n, elem, 0)
    want = before[0].copy()
    rows_s = before[2][src:src + max(n * src_stride, 1) * elem].reshape(-1, elem)[::src_stride][:n]
    view = want[dst:dst + max(n * dst_stride, 1) * elem].reshape(-1, elem)
    view[::dst_stride][:n] = rows_s
    assert np.array_equal(o.heap[0], want)
    assert np.array_equal(o.heap[1], before[1]) and np.array_equal(o.heap[2], before[2])
    # the get moves the same elements the other way round
    o2 = ShmemOracle(3, 1 << 15)
    for p in range(3):
        o2.heap[p][:] = before[p]
    o2.iget(0, dst, src, dst_stride, src_stride, n, elem, 2)
    assert np.array_equal(o2.heap[0], want)


def test_unit_strides_are_the_contiguous_put_and_get():
    rng = np.random.default_rng(1)
    a, b = ShmemOracle(2, 8192), ShmemOracle(2, 8192)
    for p in range(2):
        data = rng.integers(0, 256, 8192, dtype=np.uint8)
        a.heap[p][:], b.heap[p][:] = data, data
    a.iput(0, 4096, 64, 1, 1, 100, 8, 1), b.putmem(0, 4096, 64, 800, 1)
    a.iget(1, 1024, 4096, 1, 1, 50, 4, 0), b.getmem(1, 1024, 4096, 200, 0)
    assert all(np.array_equal(x, y) for x, y in zip(a.heap, b.heap))


def test_scatter_then_gather_is_the_identity():
    rng = np.random.default_rng(2)
    o = ShmemOracle(2, 1 << 14)
    x = rng.integers(0, 256, 400, dtype=np.uint8)
    o.write(0, 0, x)
    o.iput(0, 4096, 0, 5, 1, 100, 4, 1)           # scatter with stride 5
    o.iget(0, 1024, 4096, 1, 5, 100, 4, 1)        # gather it back
    assert np.array_equal(o.read(0, 1024, 400), x)


def test_argument_errors():
    o = ShmemOracle(2, 4096)
    for bad in (lambda: o.iput(0, 0, 2048, 0, 1, 4, 4, 1), lambda: o.iput(0, 0, 2048, 1, -1, 4, 4, 1),
                lambda: o.iput(0, 0, 2048, 1, 1, 4, 3, 1), lambda: o.iput(0, 2, 2048, 1, 1, 4, 4, 1),
                lambda: o.iput(0, 0, 2048, 1, 200, 4, 4, 1), lambda: o.iput(0, 0, 2048, 400, 1, 4, 4, 1),
                lambda: o.iput(0, 0, 8, 4, 1, 4, 4, 0), lambda: o.iget(0, 0, 2048, 1, 1, 4, 4, 2)):
        with pytest.raises(OracleError):
            bad()
    o.iput(0, 0, 4096 - 4, 1, 1000, 1, 4, 1)      # one element: strides do not matter


def test_span_ends_at_the_last_element_not_a_stride_later():
    """A strided transfer occupies (nelems - 1) * stride + 1 elements: the last element may end
    exactly at the end of the heap, and on one PE the two spans may touch without overlapping."""
    o = ShmemOracle(2, 4096)
    o.write(0, 0, np.arange(40, dtype=np.uint8))
    o.iput(0, 4096 - 37 * 4, 0, 4, 1, 10, 4, 1)             # destination elements at 3948, 3964, ..., 4092
    assert np.array_equal(o.read(1, 4092, 4), np.arange(36, 40, dtype=np.uint8))
    o.iget(0, 4096 - 19 * 2, 0, 2, 3, 10, 2, 1)             # both spans end where they must: source 56 bytes, destination 38
    with pytest.raises(OracleError):
        o.iput(0, 4096 - 37 * 4 + 4, 0, 4, 1, 10, 4, 1)     # one element further leaves the heap
    # same PE: source span [0, 148), destination span starting right behind it
    o.iput(0, 148, 0, 3, 4, 10, 4, 0)
    with pytest.raises(OracleError):
        o.iput(0, 144, 0, 3, 4, 10, 4, 0)
