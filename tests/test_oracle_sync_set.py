"""Pins for the oracle's wait_until / test family (OpenSHMEM 1.5 point-to-point synchronisation):
a hand-worked example, brute force over every status mask and comparison on a tiny set, the signed
comparison, and the relations between the forms."""
import itertools

import numpy as np
import pytest

from oracle.shmem_oracle import CMP_EQ, CMP_GE, CMP_GT, CMP_LE, CMP_LT, CMP_NE, OracleError, ShmemOracle

PY = {CMP_EQ: lambda a, b: a == b, CMP_NE: lambda a, b: a != b, CMP_GT: lambda a, b: a > b, CMP_GE: lambda a, b: a >= b,
      CMP_LT: lambda a, b: a < b, CMP_LE: lambda a, b: a <= b}


def _with(values, pe=1, off=64):
    o = ShmemOracle(2, 256)
    o.write(pe, off, np.array(values, dtype=np.int64))
    return o


def test_hand_worked_example():
    """Variables 5, -1, 7, 0 on PE 1; status takes the third one out.  '> 0' holds for index 0 only,
    '>= 0' for 0 and 3, '< 0' for 1 (a signed comparison: -1 is not a huge unsigned number)."""
    o = _with([5, -1, 7, 0])
    status = [0, 0, 1, 0]
    assert o.test_some(1, 64, 4, status, CMP_GT, 0) == [0]
    assert o.test_some(1, 64, 4, status, CMP_GE, 0) == [0, 3]
    assert o.test_some(1, 64, 4, status, CMP_LT, 0) == [1]
    assert o.test_some(1, 64, 4, None, CMP_GT, 0) == [0, 2]
    assert not o.test_all(1, 64, 4, status, CMP_GE, 0) and o.test_all(1, 64, 4, [0, 1, 0, 0], CMP_GE, 0)
    assert o.test_all(1, 64, 4, [1, 1, 1, 1], CMP_EQ, 99) and o.test_any(1, 64, 4, [1, 1, 1, 1], CMP_NE, 99) == []
    assert o.wait_until(1, 80, CMP_GT, 3) == 7 and o.wait_until(1, 72, CMP_LE, 0) == -1          # the variable's value, not the threshold
    assert o.wait_until(1, 64, CMP_EQ, 5) == 5 and o.test(1, 72, CMP_EQ, -1) and not o.test(1, 72, CMP_GT, 0)
    assert o.wait_until_any(1, 64, 4, status, CMP_GE, 0) == [0, 3] and o.wait_until_some(1, 64, 4, None, CMP_LE, 0) == [1, 3]
    o.wait_until_all(1, 64, 4, [0, 1, 0, 1], CMP_GE, 5)
    assert np.array_equal(o.read(1, 64, 32, np.int64), [5, -1, 7, 0])          # nothing here changes the heap
    assert o.heap[0].sum() == 0


def test_waits_that_cannot_end_raise_and_empty_sets_do_not_wait():
    o = _with([5, -1, 7, 0])
    for bad in (lambda: o.wait_until(1, 64, CMP_LT, 5), lambda: o.wait_until_all(1, 64, 4, None, CMP_GE, 0),
                lambda: o.wait_until_any(1, 64, 4, [0, 0, 1, 0], CMP_GT, 5), lambda: o.wait_until_some(1, 64, 4, None, CMP_EQ, 3)):
        with pytest.raises(OracleError):
            bad()
    assert o.wait_until_some(1, 64, 4, [1, 1, 1, 1], CMP_EQ, 3) == [] and o.wait_until_any(1, 64, 0, None, CMP_EQ, 3) == []
    o.wait_until_all(1, 64, 4, [1, 1, 1, 1], CMP_EQ, 3)
    for bad in (lambda: o.test_some(1, 60, 1, None, CMP_EQ, 0), lambda: o.test_some(1, 64, 100, None, CMP_EQ, 0),
                lambda: o.test_some(2, 64, 1, None, CMP_EQ, 0), lambda: o.test_some(1, 64, 2, [0], CMP_EQ, 0), lambda: o.test(1, 64, 9, 0)):
        with pytest.raises(OracleError):
            bad()


def test_brute_force_every_mask_comparison_and_threshold():
    values = [3, -4, 0, 3, 2 ** 63 - 1, -2 ** 63]
    o = _with(values, pe=0, off=8)
    for mask in itertools.product([0, 1], repeat=len(values)):
        for cmp, f in PY.items():
            for t in (-2 ** 63, -4, 0, 3, 4, 2 ** 63 - 1):
                want = [i for i, v in enumerate(values) if not mask[i] and f(v, t)]
                assert o.test_some(0, 8, len(values), list(mask), cmp, t) == want
                assert o.test_all(0, 8, len(values), list(mask), cmp, t) == (len(want) == mask.count(0))


def test_threshold_given_as_unsigned_bit_pattern_is_read_as_signed():
    o = _with([-1])
    assert o.test(1, 64, CMP_EQ, 2 ** 64 - 1) and o.test(1, 64, CMP_LT, 0)
    assert o.test(1, 64, CMP_GT, 2 ** 63) and not o.test(1, 64, CMP_GT, 2 ** 63 - 1)      # 2^63 is the most negative value
