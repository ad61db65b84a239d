"""GPU parity: the reduction matrix, every element type with every operator, bit for bit."""
import numpy as np
import pytest

from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20
DTYPES = {S.SHM_INT8: np.int8, S.SHM_UINT8: np.uint8, S.SHM_INT16: np.int16, S.SHM_UINT16: np.uint16, S.SHM_INT32: np.int32,
          S.SHM_UINT32: np.uint32, S.SHM_INT64: np.int64, S.SHM_UINT64: np.uint64, S.SHM_FLOAT32: np.float32,
          S.SHM_FLOAT64: np.float64}
OPS = {S.SHM_OP_MIN: "min", S.SHM_OP_MAX: "max", S.SHM_OP_SUM: "sum", S.SHM_OP_PROD: "prod", S.SHM_OP_AND: "and", S.SHM_OP_OR: "or",
       S.SHM_OP_XOR: "xor"}


def _source(rng, dt, n):
    """Integers: any bit pattern.  Floats: finite values of mixed sign and magnitude (no NaN, so the
    result does not depend on how a NaN's payload travels), with exact ties and signed zeros."""
    if dt.kind in "iu":
        return rng.integers(0, 256, n * dt.itemsize, dtype=np.uint8).view(dt)
    x = (rng.standard_normal(n) * np.exp2(rng.integers(-6, 6, n))).astype(dt)
    x[rng.integers(0, n, max(1, n // 8))] = dt.type(1.5)
    x[rng.integers(0, n, max(1, n // 16))] = dt.type(0.0)
    x[rng.integers(0, n, max(1, n // 16))] = dt.type(-0.0)
    return x


@pytest.mark.parametrize("dtype", sorted(DTYPES))
def test_every_operator(dtype):
    dt = np.dtype(DTYPES[dtype])
    npes, n = 8, 300007                                   # many groups' shares, whole vectors and a tail
    g, o = make_pair(npes, 16 * MiB)
    with g:
        fill_random(g, o, 50 + dtype, upto=12 * MiB)
        src, dst = 4096, 6 * MiB
        rng = np.random.default_rng(500 + dtype)
        for p in range(npes):
            write_both(g, o, p, src, _source(rng, dt, n).view(np.uint8))
        for op, name in OPS.items():
            if dt.kind == "f" and op >= S.SHM_OP_AND:
                with pytest.raises(S.ShmError):
                    g.launch_reduce(dst, src, n, dtype, op, 16)
                continue
            o.reduce(dst, src, n, dt, name)
            for algo in (S.SHM_REDUCE_DUPLICATE, S.SHM_REDUCE_SPLIT):
                g.launch_reduce(dst, src, n, dtype, op, 16, algo)
                g.barrier_all()
                assert_heaps_equal(g, o, upto=12 * MiB, what=f"{dt.name} {name} algo {algo}")
                for p in range(npes):                     # spoil the result so the second algorithm has to write it again
                    g.write(p, dst, np.full(n * dt.itemsize, 0xA5, np.uint8))


@pytest.mark.parametrize("npes,n,n_wg", [(1, 1000, 4), (2, 1, 1), (3, 15, 64), (16, 4097, 1024), (5, 0, 8), (12, 65536, 3)])
def test_shapes(npes, n, n_wg):
    g, o = make_pair(npes, 4 * MiB)
    with g:
        fill_random(g, o, 77, upto=3 * MiB)
        for dtype, op in [(S.SHM_INT16, S.SHM_OP_MAX), (S.SHM_UINT64, S.SHM_OP_PROD), (S.SHM_UINT8, S.SHM_OP_XOR)]:
            for algo in (S.SHM_REDUCE_DUPLICATE, S.SHM_REDUCE_SPLIT):
                o.reduce(2 * MiB, 16, n, DTYPES[dtype], OPS[op])
                g.launch_reduce(2 * MiB, 16, n, dtype, op, n_wg, algo)
                g.barrier_all()
                assert_heaps_equal(g, o, upto=3 * MiB, what=f"{dtype} {op} algo {algo}")
                for p in range(npes if n else 0):         # spoil the result so the next launch has to write it again
                    write_both(g, o, p, 2 * MiB, np.full(n * np.dtype(DTYPES[dtype]).itemsize, 0x5A, np.uint8))


@pytest.mark.parametrize("npes,n_wg", [(2, 8), (2, 100), (3, 64)])
def test_split_on_group_owned_tiles(npes, n_wg):
    """Slices of 64 tiles of 64 KiB plus a ragged rest per PE (the split form then walks group-owned
    tiles), an element tail, fewer and more groups than tiles; 2-byte and 8-byte elements."""
    nvec = npes * (64 * 4096 + 1000) - 3
    g, o = make_pair(npes, 40 * MiB)
    with g:
        fill_random(g, o, 78, upto=36 * MiB)
        for dtype, op, tail in [(S.SHM_INT16, S.SHM_OP_MAX, 5), (S.SHM_UINT64, S.SHM_OP_SUM, 1)]:
            width = np.dtype(DTYPES[dtype]).itemsize
            n = nvec * (16 // width) + tail
            o.reduce(18 * MiB + 16, 4096, n, DTYPES[dtype], OPS[op])
            for algo in (S.SHM_REDUCE_SPLIT, S.SHM_REDUCE_DUPLICATE):
                g.launch_reduce(18 * MiB + 16, 4096, n, dtype, op, n_wg, algo)
                g.barrier_all()
                assert_heaps_equal(g, o, upto=36 * MiB, what=f"{dtype} {op} algo {algo}")
                for p in range(npes):
                    g.write(p, 18 * MiB + 16, np.full(n * width, 0x5A, np.uint8))
            for p in range(npes):
                write_both(g, o, p, 18 * MiB + 16, np.full(n * width, 0x5A, np.uint8))


@pytest.mark.parametrize("npes,n_wg", [(2, 128), (3, 300)])
def test_split_by_ticket(npes, n_wg):
    """Slices of 96 tiles plus a ragged rest per PE, asked of a group per compute unit or more: the
    split form draws quarter tiles by ticket.  1-byte, 4-byte and 8-byte elements, an element tail,
    launches in a row on the same counters."""
    nvec = npes * (96 * 4096 + 1000) - 3
    g, o = make_pair(npes, 48 * MiB)
    with g:
        fill_random(g, o, 79, upto=44 * MiB)
        for dtype, op, tail in [(S.SHM_UINT8, S.SHM_OP_XOR, 9), (S.SHM_INT32, S.SHM_OP_MIN, 2), (S.SHM_INT64, S.SHM_OP_PROD, 1)]:
            width = np.dtype(DTYPES[dtype]).itemsize
            n = nvec * (16 // width) + tail
            o.reduce(22 * MiB + 16, 4096, n, DTYPES[dtype], OPS[op])
            g.launch_reduce(22 * MiB + 16, 4096, n, dtype, op, n_wg, S.SHM_REDUCE_SPLIT)
            g.barrier_all()
            assert_heaps_equal(g, o, upto=44 * MiB, what=f"{dtype} {op}")
            for p in range(npes):
                write_both(g, o, p, 22 * MiB + 16, np.full(n * width, 0x5A, np.uint8))


def test_full_size_sum_matches_the_f32_entry_point_and_the_oracle():
    # configuration 5's vector length (16 Mi elements, 8 PEs): int32 sum against the oracle, and the
    # float32 sum of the matrix against the dedicated float32 entry point
    npes, n = 8, 16 << 20
    g, o = make_pair(npes, 200 * MiB)
    with g:
        src, dst, dst2 = 0, 64 * MiB, 128 * MiB
        rng = np.random.default_rng(5)
        for p in range(npes):
            write_both(g, o, p, src, rng.integers(0, 256, 4 * n, dtype=np.uint8))
        want = o.reduce(dst, src, n, np.int32, "sum")
        for algo in (S.SHM_REDUCE_DUPLICATE, S.SHM_REDUCE_SPLIT):
            g.launch_reduce(dst, src, n, S.SHM_INT32, S.SHM_OP_SUM, 1024, algo)
            g.barrier_all()
            for p in (0, 3, 7):
                assert np.array_equal(g.read(p, dst, 4 * n).view(np.int32), want)
                g.write(p, dst, np.zeros(4096, np.uint8))
        for p in range(npes):
            g.write(p, src, rng.standard_normal(n).astype(np.float32).view(np.uint8))
        g.launch_reduce(dst, src, n, S.SHM_FLOAT32, S.SHM_OP_SUM, 1024)
        g.launch_reduce_sum_f32(dst2, src, n, 1024)
        g.barrier_all()
        for p in (0, 7):
            assert np.array_equal(g.read(p, dst, 4 * n), g.read(p, dst2, 4 * n))
