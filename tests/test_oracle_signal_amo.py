"""Pins for the oracle's signalling and atomic model (CPU only)."""
import numpy as np
import pytest

from oracle.shmem_oracle import (CMP_EQ, CMP_GE, CMP_GT, CMP_LE, CMP_LT, CMP_NE, SIGNAL_ADD, SIGNAL_SET,
                                 OracleError, ShmemOracle)

I64_MAX = 2 ** 63 - 1
I64_MIN = -2 ** 63


def test_put_signal_payload_lands_before_signal():
    """Record the destination at the moment the signal word is written."""
    seen = {}

    class Spy(ShmemOracle):
        def _store_u64(self, pe, off, v):
            seen["dst"] = self.heap[pe][64:64 + 40].copy()
            super()._store_u64(pe, off, v)

    o = Spy(2, 256)
    o.heap[0][8:48] = np.arange(1, 41, dtype=np.uint8)
    o.put_signal(0, 64, 8, 40, 128, 1, SIGNAL_SET, 1)
    assert (seen["dst"] == np.arange(1, 41)).all(), "signal written before its data"
    assert (o.heap[1][64:104] == np.arange(1, 41)).all()
    assert o.signal_fetch(1, 128) == 1
    assert o.signal_fetch(0, 128) == 0          # only the target's word changes


def test_signal_ops_set_add_wrap_and_zero_length():
    o = ShmemOracle(2, 128)
    o.put_signal(0, 0, 0, 0, 64, 5, SIGNAL_SET, 1)      # n = 0 still signals
    assert o.signal_fetch(1, 64) == 5
    o.put_signal(0, 0, 0, 0, 64, 7, SIGNAL_ADD, 1)
    assert o.signal_fetch(1, 64) == 12
    o.put_signal(0, 0, 0, 0, 64, 2 ** 64 - 1, SIGNAL_SET, 1)
    o.put_signal(0, 0, 0, 0, 64, 2, SIGNAL_ADD, 1)      # wraps modulo 2^64
    assert o.signal_fetch(1, 64) == 1
    assert bytes(o.heap[1][64:72]) == (1).to_bytes(8, "little")
    with pytest.raises(OracleError):
        o.put_signal(0, 0, 0, 0, 60, 1, SIGNAL_SET, 1)  # misaligned signal word
    with pytest.raises(OracleError):
        o.put_signal(0, 0, 0, 0, 64, 1, 9, 1)
    # OpenSHMEM 1.5, put-with-signal: the signal word may not overlap the destination; touching it is fine
    before = [h.copy() for h in o.heap]
    for dst, n in [(60, 8), (64, 1), (71, 3), (40, 30)]:
        with pytest.raises(OracleError):
            o.put_signal(0, dst, 0, n, 64, 1, SIGNAL_SET, 1)
    assert all(np.array_equal(a, b) for a, b in zip(before, o.heap)), "a refused operation changed the heap"
    o.put_signal(0, 56, 0, 8, 64, 1, SIGNAL_SET, 1)     # ends where the word begins
    o.put_signal(0, 72, 0, 8, 64, 1, SIGNAL_SET, 1)     # begins where the word ends
    o.put_signal(0, 64, 0, 0, 64, 1, SIGNAL_SET, 1)     # no payload, nothing to overlap


def test_wait_until_unsigned_compare_and_illegal_schedule():
    o = ShmemOracle(1, 64)
    o.put_signal(0, 0, 0, 0, 8, 2 ** 63, SIGNAL_SET, 0)   # would be negative if read signed
    assert o.signal_wait_until(0, 8, CMP_GT, 1) == 2 ** 63
    assert o.signal_wait_until(0, 8, CMP_GE, 2 ** 63) == 2 ** 63
    assert o.signal_wait_until(0, 8, CMP_NE, 0) == 2 ** 63
    with pytest.raises(OracleError):
        o.signal_wait_until(0, 8, CMP_LT, 1)
    o.put_signal(0, 0, 0, 0, 8, 3, SIGNAL_SET, 0)
    table = {CMP_EQ: [3], CMP_NE: [2, 4], CMP_GT: [2, 0], CMP_GE: [3, 2], CMP_LT: [4], CMP_LE: [3, 4]}
    bad = {CMP_EQ: [2, 4], CMP_NE: [3], CMP_GT: [3, 4], CMP_GE: [4], CMP_LT: [3, 2], CMP_LE: [2]}
    for c, vals in table.items():
        for v in vals:
            assert o.signal_wait_until(0, 8, c, v) == 3
    for c, vals in bad.items():
        for v in vals:
            with pytest.raises(OracleError):
                o.signal_wait_until(0, 8, c, v)


def test_ordering_ops_change_nothing_and_are_logged():
    o = ShmemOracle(2, 64)
    o.heap[0][:] = 3
    before = [h.copy() for h in o.heap]
    o.quiet(0), o.fence(1), o.barrier_all()
    assert all((a == b).all() for a, b in zip(before, o.heap))
    assert o.log == [("quiet", 0), ("fence", 1), ("barrier_all",)]


def test_fetch_add_returns_running_count_and_wraps():
    o = ShmemOracle(3, 64)
    got = [o.atomic_fetch_add(i % 3, 16, 1, 2) for i in range(50)]
    assert got == list(range(50))
    assert sum(got) == 50 * 49 // 2
    assert o.atomic_fetch(0, 16, 2) == 50
    assert o.atomic_fetch(0, 16, 1) == 0
    o.atomic_set(0, 24, I64_MAX, 1)
    assert o.atomic_fetch_add(0, 24, 1, 1) == I64_MAX
    assert o.atomic_fetch(0, 24, 1) == I64_MIN          # two's-complement wrap
    assert o.atomic_fetch_add(0, 24, -1, 1) == I64_MIN
    assert o.atomic_fetch(0, 24, 1) == I64_MAX
    with pytest.raises(OracleError):
        o.atomic_fetch_add(0, 20, 1, 1)
    with pytest.raises(OracleError):
        o.atomic_fetch_add(0, 64, 1, 1)


def test_compare_swap_swap_inc_semantics():
    o = ShmemOracle(2, 64)
    assert o.atomic_compare_swap(0, 8, 0, 11, 1) == 0       # matches: stored
    assert o.atomic_fetch(0, 8, 1) == 11
    assert o.atomic_compare_swap(0, 8, 0, 99, 1) == 11      # no match: unchanged
    assert o.atomic_fetch(0, 8, 1) == 11
    assert o.atomic_compare_swap(1, 8, -1, 5, 1) == 11
    o.atomic_set(0, 8, -1, 1)
    assert o.atomic_compare_swap(1, 8, 2 ** 64 - 1, 5, 1) == -1   # same 64-bit pattern as -1
    assert o.atomic_fetch(0, 8, 1) == 5
    assert o.atomic_swap(0, 8, -7, 1) == 5
    assert o.atomic_fetch(1, 8, 1) == -7
    assert o.atomic_fetch_inc(0, 8, 1) == -7
    o.atomic_inc(0, 8, 1), o.atomic_add(0, 8, 10, 1)
    assert o.atomic_fetch(0, 8, 1) == 5
    # textbook: an increment built from a compare-swap retry loop equals fetch-add
    for _ in range(20):
        while True:
            cur = o.atomic_fetch(0, 16, 0)
            if o.atomic_compare_swap(1, 16, cur, cur + 3, 0) == cur:
                break
    assert o.atomic_fetch(0, 16, 0) == 60


@pytest.mark.parametrize("npes,n_ctr,n_items,ops", [(2, 4, 10, 10), (3, 5, 12, 7), (1, 1, 4, 4), (4, 2, 8, 1)])
def test_amo_storm_vectorised_equals_loop_and_closed_forms(npes, n_ctr, n_items, ops):
    rng = np.random.default_rng(npes * 100 + n_ctr)
    targets = rng.integers(0, npes * n_ctr, size=(n_items, ops), dtype=np.uint16)
    a, b = ShmemOracle(npes, 256), ShmemOracle(npes, 256)
    init = rng.integers(-5, 5, size=(npes, n_ctr), dtype=np.int64)
    for p in range(npes):
        a.write(p, 64, init[p]), b.write(p, 64, init[p])
    fa = a.amo_storm_loop(64, n_ctr, targets)
    fb = b.amo_storm(64, n_ctr, targets)
    assert (fa == fb).all()
    assert all((x == y).all() for x, y in zip(a.heap, b.heap))
    counts = np.bincount(targets.reshape(-1), minlength=npes * n_ctr)
    final = np.concatenate([b.read(p, 64, 8 * n_ctr, np.int64) for p in range(npes)])
    assert (final == init.reshape(-1) + counts).all()
    for t in range(npes * n_ctr):
        got = np.sort(fb[targets == t]) - init.reshape(-1)[t]
        assert (got == np.arange(counts[t])).all()          # fetched values are exactly 0..n-1
        assert got.sum() == counts[t] * (counts[t] - 1) // 2


def test_amo_storm_rejects_bad_targets():
    o = ShmemOracle(2, 256)
    with pytest.raises(OracleError):
        o.amo_storm(64, 4, np.array([[8]], dtype=np.uint16))
    with pytest.raises(OracleError):
        o.amo_storm(60, 4, np.array([[1]], dtype=np.uint16))
