"""Pins for the oracle's data-movement and allocator model (CPU only).

The reference model used here is written independently of the oracle: plain
Python lists, one byte at a time, no slicing.
"""
import itertools
import os

import numpy as np
import pytest

from oracle.shmem_oracle import OracleError, ShmemOracle, U64_MASK

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _fill(o, seed=0):
    rng = np.random.default_rng(seed)
    for p in range(o.npes):
        o.heap[p][:] = rng.integers(0, 256, o.heap_bytes, dtype=np.uint8)
    return [[int(b) for b in o.heap[p]] for p in range(o.npes)]


def _as_lists(o):
    return [[int(b) for b in o.heap[p]] for p in range(o.npes)]


@pytest.mark.parametrize("npes", [1, 2, 3])
def test_put_get_brute_force_all_triples(npes):
    H = 14
    for me, pe in itertools.product(range(npes), repeat=2):
        for src, dst in itertools.product(range(H), repeat=2):
            for n in range(0, H - max(src, dst) + 1):
                for op in ("put", "get"):
                    o = ShmemOracle(npes, H)
                    model = _fill(o, seed=src * 31 + dst)
                    overlap = me == pe and n > 0 and src < dst + n and dst < src + n
                    if overlap:
                        with pytest.raises(OracleError):
                            getattr(o, op + "mem")(me, dst, src, n, pe)
                        continue
                    before = [row[:] for row in model]
                    if op == "put":     # me's bytes go to pe
                        for i in range(n):
                            model[pe][dst + i] = before[me][src + i]
                        o.putmem(me, dst, src, n, pe)
                    else:               # pe's bytes come to me
                        for i in range(n):
                            model[me][dst + i] = before[pe][src + i]
                        o.getmem(me, dst, src, n, pe)
                    assert _as_lists(o) == model, (op, me, pe, src, dst, n)


def test_out_of_range_and_bad_pe_are_errors():
    o = ShmemOracle(2, 32)
    for bad in [lambda: o.putmem(0, 30, 0, 3, 1), lambda: o.putmem(0, 0, 30, 3, 1),
                lambda: o.getmem(0, 0, 0, 33, 1), lambda: o.putmem(0, 0, 0, 1, 2),
                lambda: o.putmem(-1, 0, 0, 1, 1), lambda: o.putmem(0, -1, 0, 1, 1)]:
        with pytest.raises(OracleError):
            bad()


def test_golden_put_example():
    rows = [l for l in open(os.path.join(GOLDEN, "put_example.txt")) if not l.startswith("#")]
    want = [[int(x) for x in r.split()] for r in rows]
    o = ShmemOracle(3, 16)
    for p in range(3):
        o.heap[p][:] = np.arange(16 * p, 16 * p + 16, dtype=np.uint8)
    o.putmem(2, 9, 3, 5, 0)
    assert _as_lists(o) == want


def test_golden_address_rule():
    for line in open(os.path.join(GOLDEN, "address_rule.txt")):
        if line.startswith("#") or not line.strip():
            continue
        la, lb, rb, want = (int(x, 16) for x in line.split())
        assert ShmemOracle.translate(la, lb, rb) == want
    # the flat-array model is that rule with base[p] = p * heap_bytes in one address space
    o = ShmemOracle(4, 64)
    _fill(o, 3)
    flat = np.concatenate(o.heap)
    base = [p * 64 for p in range(4)]
    for me, pe, off in [(0, 3, 5), (2, 1, 63), (1, 1, 0)]:
        addr = ShmemOracle.translate(base[me] + off, base[me], base[pe])
        assert flat[addr] == o.heap[pe][off]


def test_put_then_get_round_trip_and_self_target():
    o = ShmemOracle(3, 256)
    _fill(o, 7)
    src = o.heap[0][10:110].copy()
    o.putmem(0, 120, 10, 100, 2)
    assert (o.heap[2][120:220] == src).all()
    o.getmem(1, 5, 120, 100, 2)
    assert (o.heap[1][5:105] == src).all()
    # a PE may target itself when the ranges are disjoint
    o.putmem(0, 130, 10, 100, 0)
    assert (o.heap[0][130:230] == src).all()


def test_wg_slices_partition_the_message():
    for n in list(range(0, 70)) + [255, 256, 257, 4096, 16384, 1 << 20, (1 << 20) + 5]:
        for n_wg in [1, 2, 3, 4, 7, 64, 1024]:
            sl = ShmemOracle.wg_slices(n, n_wg)
            assert len(sl) == n_wg
            cur = 0
            for lo, hi in sl:
                assert lo == cur or (lo == n and hi == n)
                assert lo <= hi <= n
                assert lo % 16 == 0 or lo == n
                cur = hi
            assert cur == n
            covered = sum(hi - lo for lo, hi in sl)
            assert covered == n


@pytest.mark.parametrize("n_wg", [1, 2, 3, 5, 64])
def test_wg_put_get_equal_plain_put_get(n_wg):
    for n in [0, 1, 15, 16, 17, 100, 333]:
        a, b = ShmemOracle(2, 1024), ShmemOracle(2, 1024)
        _fill(a, n), _fill(b, n)
        a.putmem(0, 512 + 3, 7, n, 1)
        b.wg_put(0, 512 + 3, 7, n, 1, n_wg)
        assert _as_lists(a) == _as_lists(b)
        a.getmem(1, 20, 600, n, 0)
        b.wg_get(1, 20, 600, n, 0, n_wg)
        assert _as_lists(a) == _as_lists(b)


def test_write_read_staging_typed():
    o = ShmemOracle(2, 128)
    v = np.array([1, -2, 3, 2 ** 31 - 1], dtype=np.int32)
    o.write(1, 16, v)
    assert (o.read(1, 16, 16, np.int32) == v).all()
    assert bytes(o.heap[1][16:20]) == (1).to_bytes(4, "little")
    assert not o.heap[0].any()


def test_allocator_invariants():
    rng = np.random.default_rng(5)
    o = ShmemOracle(4, 1 << 16)
    live = {}
    for step in range(600):
        if live and rng.random() < 0.45:
            off = list(live)[int(rng.integers(len(live)))]
            o.free(off)
            del live[off]
            continue
        n = int(rng.integers(1, 3000))
        align = int(2 ** rng.integers(0, 10))
        try:
            off = o.malloc(n, align)
        except OracleError:
            continue
        assert off % align == 0 and off + n <= o.heap_bytes
        for o2, n2 in live.items():
            assert off + n <= o2 or o2 + n2 <= off, "blocks overlap"
        live[off] = n
    # everything freed -> the whole heap is available again in one piece
    for off in list(live):
        o.free(off)
    assert o.malloc(o.heap_bytes, 1) == 0
    with pytest.raises(OracleError):
        o.malloc(1, 1)


def test_allocator_edge_cases():
    o = ShmemOracle(2, 4096)
    assert o.malloc(0) == U64_MASK
    o.free(U64_MASK)
    a = o.malloc(10)
    assert a % ShmemOracle.DEFAULT_ALIGN == 0
    with pytest.raises(OracleError):
        o.free(a + 1)
    with pytest.raises(OracleError):
        o.malloc(8, 3)
    with pytest.raises(OracleError):
        o.malloc(5000)
    o.heap[0][:] = 9
    o.heap[1][:] = 9
    c = o.calloc(100, 64)
    assert not o.heap[0][c:c + 100].any() and not o.heap[1][c:c + 100].any()
    assert o.heap[0][c + 100] == 9
