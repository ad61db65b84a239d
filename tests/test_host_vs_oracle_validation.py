"""CPU differential test of argument validation: for thousands of argument tuples drawn around the
boundaries (heap end, word alignment, overlapping ranges, PE range, strides), the library -- through
a context that makes no device call, so a valid request ends in SHM_ENODEV -- and the oracle must
agree on WHETHER the operation is defined.  Neither side computes anything for the other."""
import numpy as np
import pytest

from oracle.shmem_oracle import CMP_GE, OracleError, ShmemOracle
from paper_2409_20476_amd import shm as S

HEAP = 128 * 1024            # library partition; the usable part is what the oracle models
NPES = 3


def _pair():
    g = S.Shm(NPES, HEAP, heap_base=4096, flags=S.SHM_INIT_NO_DEVICE)
    return g, ShmemOracle(NPES, g.heap_bytes())


def _lib_defined(call):
    try:
        call()
    except S.ShmError as e:
        if e.code == S.SHM_ENODEV:
            return True              # every check passed; only the device step was refused
        assert e.code in (S.SHM_EINVAL, S.SHM_EPE, S.SHM_ERANGE), e.code
        return False
    raise AssertionError("a no-device context executed something")


def _oracle_defined(call):
    try:
        call()
    except OracleError:
        return False
    return True


def _pools(rng, u):
    offs = [0, 1, 7, 8, 15, 16, 100, 4096, u // 2, u - 4096, u - 100, u - 16, u - 8, u - 1, u, u + 1, u + 4096]
    lens = [0, 1, 8, 15, 16, 100, 4096, u // 2, u - 100, u, u + 1]
    pes = [-1, 0, 0, 1, 1, NPES - 1, NPES]
    pick = lambda pool: int(pool[rng.integers(len(pool))])
    return (lambda: pick(offs)), (lambda: pick(lens)), (lambda: pick(pes))


def _compare(name, n_cases, draw):
    g, o = _pair()
    rng = np.random.default_rng(sum(map(ord, name)))
    off, length, pe = _pools(rng, o.heap_bytes)
    defined = 0
    for i in range(n_cases):
        lib_call, oracle_call, shown = draw(g, o, rng, off, length, pe)
        a, b = _lib_defined(lib_call), _oracle_defined(oracle_call)
        assert a == b, f"{name} case {i} {shown}: library says {'defined' if a else 'undefined'}, oracle says {'defined' if b else 'undefined'}"
        defined += a
    assert 0.02 * n_cases < defined < 0.98 * n_cases, f"{name}: {defined} of {n_cases} defined -- the draw does not probe both sides"
    g.finalize()


def test_put_and_get():
    def draw(g, o, rng, off, length, pe):
        me, p, d, s, n = pe(), pe(), off(), off(), length()
        if rng.integers(2):
            return (lambda: g.putmem(me, d, s, n, p)), (lambda: o.putmem(me, d, s, n, p)), ("put", me, p, d, s, n)
        return (lambda: g.getmem(me, d, s, n, p)), (lambda: o.getmem(me, d, s, n, p)), ("get", me, p, d, s, n)
    _compare("put_get", 3000, draw)


def test_work_group_put_and_get():
    def draw(g, o, rng, off, length, pe):
        me, p, d, s, n = pe(), pe(), off(), off(), length()
        n_wg = int(rng.choice([0, 1, 1, 3, 64]))
        if rng.integers(2):
            return (lambda: g.launch_wg_put(me, p, d, s, n, n_wg)), (lambda: o.wg_put(me, d, s, n, p, n_wg)), ("wg_put", me, p, d, s, n, n_wg)
        return (lambda: g.launch_wg_get(me, p, d, s, n, n_wg)), (lambda: o.wg_get(me, d, s, n, p, n_wg)), ("wg_get", me, p, d, s, n, n_wg)
    _compare("wg", 3000, draw)


def test_put_with_signal():
    def draw(g, o, rng, off, length, pe):
        me, p, d, s, n, sig = pe(), pe(), off(), off(), length(), off()
        if rng.integers(3) == 0:
            sig = d + int(rng.integers(-8, max(1, n) + 8))          # around and inside the destination
        op = int(rng.choice([0, 1, 1, 2, -1]))
        n_wg = int(rng.choice([1, 2, 5]))
        return ((lambda: g.launch_wg_put_signal(me, p, d, s, n, max(sig, 0), 7, op, n_wg)),
                (lambda: o.put_signal(me, d, s, n, max(sig, 0), 7, op, p, n_wg)), ("put_signal", me, p, d, s, n, sig, op))
    _compare("put_signal", 4000, draw)


def test_atomics_and_waits():
    def draw(g, o, rng, off, length, pe):
        me, p, at = pe(), pe(), off()
        kind = int(rng.integers(3))
        if kind == 0:
            return (lambda: g.launch_amo(me, p, at, S.SHM_AMO_FETCH_ADD, 1)), (lambda: o.atomic_fetch_add(me, at, 1, p)), ("fetch_add", me, p, at)
        if kind == 1:
            return (lambda: g.launch_amo(me, p, at, S.SHM_AMO_COMPARE_SWAP, 1, 0)), (lambda: o.atomic_compare_swap(me, at, 0, 1, p)), ("cswap", me, p, at)
        # unsigned >= 0 holds for every value, so only the arguments decide
        return (lambda: g.launch_signal_wait_until(me, at, S.SHM_CMP_GE, 0)), (lambda: o.signal_wait_until(me, at, CMP_GE, 0)), ("wait", me, at)
    _compare("amo", 2000, draw)


def test_strided():
    def draw(g, o, rng, off, length, pe):
        me, p, d, s = pe(), pe(), off(), off()
        ds, ss = (int(rng.choice([-1, 0, 1, 1, 2, 3, 17, 1000, 1 << 40])) for _ in range(2))
        nelems = int(rng.choice([0, 1, 2, 5, 100, 1000, 1 << 20]))
        elem = int(rng.choice([1, 2, 3, 4, 8, 16, 32]))
        if rng.integers(2) and elem in (1, 2, 4, 8, 16):            # half of the time element-aligned offsets
            d, s = d // elem * elem, s // elem * elem
        if rng.integers(2):
            return ((lambda: g.launch_iput(me, p, d, s, ds, ss, nelems, elem, 2)), (lambda: o.iput(me, d, s, ds, ss, nelems, elem, p)),
                    ("iput", me, p, d, s, ds, ss, nelems, elem))
        return ((lambda: g.launch_iget(me, p, d, s, ds, ss, nelems, elem, 0)), (lambda: o.iget(me, d, s, ds, ss, nelems, elem, p)),
                ("iget", me, p, d, s, ds, ss, nelems, elem))
    _compare("strided", 4000, draw)


def test_collectives():
    def draw(g, o, rng, off, length, pe):
        d, s, n = off() // 16 * 16, off() // 16 * 16, length()
        kind = int(rng.integers(4))
        if rng.integers(4) == 0:
            n = int(rng.choice([0, 16, 100, 4096, o.heap_bytes // NPES, o.heap_bytes // NPES + 1]))
        if kind == 0:
            return (lambda: g.launch_fcollect(d, s, n, 2)), (lambda: o.fcollect(d, s, n)), ("fcollect", d, s, n)
        if kind == 1:
            sizes = [int(rng.choice([0, 1, 100, n])) for _ in range(NPES)]
            return (lambda: g.launch_collect(d, s, sizes, 2)), (lambda: o.collect(d, s, sizes)), ("collect", d, s, sizes)
        if kind == 2:
            root = pe()
            return (lambda: g.launch_broadcast(d, s, n, root, 2)), (lambda: o.broadcast(d, s, n, root)), ("broadcast", d, s, n, root)
        dt, code = [(np.int16, S.SHM_INT16), (np.uint64, S.SHM_UINT64), (np.float32, S.SHM_FLOAT32)][int(rng.integers(3))]
        op, op_code = [("sum", S.SHM_OP_SUM), ("min", S.SHM_OP_MIN), ("xor", S.SHM_OP_XOR)][int(rng.integers(3))]
        nelems = n // np.dtype(dt).itemsize
        if rng.integers(3) == 0:
            d += 8                                               # reductions want 16-byte aligned buffers
        return ((lambda: g.launch_reduce(d, s, nelems, code, op_code, 2)), (lambda: o.reduce(d, s, nelems, dt, op)),
                ("reduce", d, s, nelems, dt.__name__, op))
    _compare("collectives", 4000, draw)
