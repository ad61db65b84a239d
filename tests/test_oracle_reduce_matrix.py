"""Pins for the oracle's reduction matrix: hand-worked fixture, Python big-integer arithmetic,
Python-double arithmetic rounded to the element type, special cases and argument errors."""
import functools
import os
import struct

import numpy as np
import pytest

from oracle.shmem_oracle import OracleError, ShmemOracle

INT_TYPES = [np.int8, np.uint8, np.int16, np.uint16, np.int32, np.uint32, np.int64, np.uint64]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "reduce_matrix_example.txt")


def _run(npes, dtype, op, columns, src=64, dst=4096):
    """columns[p] = PE p's vector; returns PE 0's result and checks that every PE got the same."""
    dt = np.dtype(dtype)
    n = len(columns[0])
    o = ShmemOracle(npes, 1 << 16)
    for p in range(npes):
        o.write(p, src, np.asarray(columns[p], dtype=dt).view(np.uint8))
    r = o.reduce(dst, src, n, dt, op)
    outs = [o.read(p, dst, n * dt.itemsize).view(dt) for p in range(npes)]
    for p in range(1, npes):
        assert outs[p].tobytes() == outs[0].tobytes()
    assert outs[0].tobytes() == np.asarray(r, dtype=dt).tobytes()
    return outs[0]


def test_golden_worked_example():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 20
    for dtype, op, a, b, c, want in rows:
        got = _run(3, dtype, op, [[int(a)], [int(b)], [int(c)]])
        assert int(got[0]) == int(want), (dtype, op, a, b, c, int(got[0]), want)


def _wrap(v, bits, signed):
    v &= (1 << bits) - 1
    return v - (1 << bits) if signed and v >> (bits - 1) else v


PY_OPS = {"min": min, "max": max, "sum": lambda a, b: a + b, "prod": lambda a, b: a * b, "and": lambda a, b: a & b,
          "or": lambda a, b: a | b, "xor": lambda a, b: a ^ b}


@pytest.mark.parametrize("dtype", INT_TYPES)
@pytest.mark.parametrize("op", ["min", "max", "sum", "prod", "and", "or", "xor"])
def test_integers_match_big_integer_arithmetic(dtype, op):
    dt = np.dtype(dtype)
    bits, signed = dt.itemsize * 8, dt.kind == "i"
    rng = np.random.default_rng(hash((dt.name, op)) & 0xffff)
    npes, n = 5, 37                                       # 37 elements: whole 16-byte vectors plus a tail
    info = np.iinfo(dt)
    cols = [rng.integers(info.min, info.max, n, dtype=dt, endpoint=True) for _ in range(npes)]
    cols[0][0], cols[1][0] = info.max, info.max           # forced overflow / extreme values
    cols[2][1], cols[3][1] = info.min, info.min
    got = _run(npes, dt, op, cols)
    for i in range(n):
        want = _wrap(functools.reduce(PY_OPS[op], [int(c[i]) for c in cols]), bits, signed)
        assert int(got[i]) == want, (dt.name, op, i)


def _round(v, dt):
    return struct.unpack("f", struct.pack("f", v))[0] if dt == np.float32 else v


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("op", ["min", "max", "sum", "prod"])
def test_floats_match_sequential_python_arithmetic(dtype, op):
    # Python floats are IEEE doubles; for float32 every step is rounded back to single, which is
    # exact double rounding for + and * (53 >= 2 * 24 + 2).
    dt = np.dtype(dtype)
    rng = np.random.default_rng(7)
    npes, n = 6, 29
    cols = [(rng.standard_normal(n) * 3).astype(dt) for _ in range(npes)]
    got = _run(npes, dt, op, cols)
    for i in range(n):
        r = float(cols[0][i])
        for p in range(1, npes):
            r = _round(PY_OPS[op](r, float(cols[p][i])), dt)
        assert float(got[i]) == r, (dt.name, op, i)
    if op == "sum":
        exact = np.sum([c.astype(np.float64) for c in cols], axis=0)
        bound = (npes - 1) * np.finfo(dt).eps * np.sum([np.abs(c.astype(np.float64)) for c in cols], axis=0)
        assert np.all(np.abs(got.astype(np.float64) - exact) <= bound)


def test_float_sum_is_the_pinned_f32_sum():
    rng = np.random.default_rng(9)
    o = ShmemOracle(4, 1 << 16)
    for p in range(4):
        o.write(p, 0, rng.standard_normal(100).astype(np.float32).view(np.uint8))
    a = o.reduce(8192, 0, 100, np.float32, "sum")
    b = o.reduce_sum_f32(16384, 0, 100)["f32"]
    assert a.tobytes() == np.asarray(b, dtype=np.float32).tobytes()


def test_order_matters_and_ties_keep_the_earlier_operand():
    # float sum is not associative: (1e8 + -1e8) + 1 = 1 but (1 + 1e8) + -1e8 = 0 in single precision
    assert float(_run(3, np.float32, "sum", [[1e8], [-1e8], [1.0]])[0]) == 1.0
    assert float(_run(3, np.float32, "sum", [[1.0], [1e8], [-1e8]])[0]) == 0.0
    # equal zeros of different sign: the earlier PE's operand stays
    assert np.signbit(_run(2, np.float64, "min", [[-0.0], [0.0]])[0])
    assert not np.signbit(_run(2, np.float64, "min", [[0.0], [-0.0]])[0])
    assert not np.signbit(_run(2, np.float32, "max", [[0.0], [-0.0]])[0])


def test_one_pe_is_a_copy_and_empty_is_nothing():
    x = np.arange(-5, 20, dtype=np.int16)
    for op in ShmemOracle.REDUCE_OPS:
        assert np.array_equal(_run(1, np.int16, op, [x]), x)
    o = ShmemOracle(3, 4096)
    before = [h.copy() for h in o.heap]
    o.reduce(1024, 0, 0, np.uint32, "xor")
    assert all(np.array_equal(a, b) for a, b in zip(before, o.heap))


def test_identities():
    rng = np.random.default_rng(3)
    x = rng.integers(0, 1 << 32, 50, dtype=np.uint32)
    assert np.all(_run(2, np.uint32, "xor", [x, x]) == 0)
    assert np.array_equal(_run(4, np.uint32, "and", [x] * 4), x)
    assert np.array_equal(_run(4, np.uint32, "or", [x] * 4), x)
    assert np.array_equal(_run(3, np.uint32, "min", [x, x, x]), x)
    assert np.array_equal(_run(4, np.uint32, "sum", [x] * 4), x * np.uint32(4))


def test_argument_errors():
    o = ShmemOracle(2, 4096)
    with pytest.raises(OracleError):
        o.reduce(1024, 0, 8, np.float32, "xor")
    with pytest.raises(OracleError):
        o.reduce(1024, 0, 8, np.int32, "nand")
    with pytest.raises(OracleError):
        o.reduce(1024, 8, 8, np.int32, "sum")             # misaligned source
    with pytest.raises(OracleError):
        o.reduce(16, 0, 8, np.int32, "sum")               # overlap
    with pytest.raises(OracleError):
        o.reduce(4000, 0, 100, np.int32, "sum")           # leaves the heap
