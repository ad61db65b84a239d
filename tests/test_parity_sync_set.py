"""GPU parity: wait_until / test and their all / any / some forms on 64-bit signed variables."""
import numpy as np
import pytest
import torch

from oracle.shmem_oracle import OracleError
from paper_2409_20476_amd import shm as S
from parity_util import fill_random, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20
NONE = 2 ** 64 - 1
CMPS = [S.SHM_CMP_EQ, S.SHM_CMP_NE, S.SHM_CMP_GT, S.SHM_CMP_GE, S.SHM_CMP_LT, S.SHM_CMP_LE]


def _run(g, me, off, n, status, kind, cmp, val):
    out = torch.full((1 + max(n, 1),), -7, dtype=torch.int64, device="cuda")
    st = None if status is None else torch.tensor(status, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    g.launch_sync_set(me, off, n, st, kind, cmp, val, out)
    g.quiet(me)
    return [int(v) & NONE for v in out.tolist()]


def test_every_form_against_the_oracle_on_random_sets():
    g, o = make_pair(3, MiB)
    rng = np.random.default_rng(91)
    with g:
        g.set_wait_timeout_us(300)                  # a wait the oracle calls unsatisfiable runs into this bound
        checked = timeouts = 0
        for case in range(60):
            n = int(rng.integers(0, 9))
            me, off = int(rng.integers(3)), 4096 + 8 * int(rng.integers(0, 50))
            values = rng.integers(-3, 4, max(n, 1)).astype(np.int64)
            if case % 7 == 0:
                values[0] = [-2 ** 63, 2 ** 63 - 1][case % 2]
            write_both(g, o, me, off, values)
            status = None if case % 3 == 0 else [int(x) for x in rng.integers(0, 2, n)]
            cmp, val = CMPS[case % 6], int(rng.integers(-3, 4))
            some = o.test_some(me, off, n, status, cmp, val)
            selected = n if status is None else status.count(0)
            # the tests look once
            assert _run(g, me, off, n, status, S.SHM_SYNC_TEST_ALL, cmp, val)[0] == int(o.test_all(me, off, n, status, cmp, val))
            r = _run(g, me, off, n, status, S.SHM_SYNC_TEST_SOME, cmp, val)
            assert r[0] == len(some) and r[1:1 + r[0]] == some
            r = _run(g, me, off, n, status, S.SHM_SYNC_TEST_ANY, cmp, val)
            assert (r[0] in some) if some else r[0] == NONE
            assert _run(g, me, off, 1, None, S.SHM_SYNC_TEST, cmp, val)[0] == int(o.test(me, off, cmp, val))
            # the waits either return at once with the same answers or run into the bound, as the oracle says
            for kind, fn in ((S.SHM_SYNC_WAIT_ALL, o.wait_until_all), (S.SHM_SYNC_WAIT_ANY, o.wait_until_any), (S.SHM_SYNC_WAIT_SOME, o.wait_until_some)):
                try:
                    want = fn(me, off, n, status, cmp, val)
                except OracleError:
                    want = "never"
                if want == "never":
                    with pytest.raises(S.ShmError) as e:
                        _run(g, me, off, n, status, kind, cmp, val)
                    assert e.value.code == S.SHM_ETIMEOUT
                    timeouts += 1
                    continue
                r = _run(g, me, off, n, status, kind, cmp, val)
                if kind == S.SHM_SYNC_WAIT_ALL:
                    assert r[0] == 1
                elif kind == S.SHM_SYNC_WAIT_ANY:
                    assert (r[0] in want) if selected else r[0] == NONE
                else:
                    assert r[0] == len(want) and r[1:1 + r[0]] == want
                checked += 1
            try:
                want = o.wait_until(me, off, cmp, val)
                assert _run(g, me, off, 1, None, S.SHM_SYNC_WAIT, cmp, val)[0] == want & NONE
            except OracleError:
                with pytest.raises(S.ShmError):
                    _run(g, me, off, 1, None, S.SHM_SYNC_WAIT, cmp, val)
        assert checked > 40 and timeouts > 20
        g.set_wait_timeout_us(2_000_000)


def _runs_beside(g, o, waiter, setter, off):
    """Whether a kernel on PE `setter`'s stream runs while a kernel on PE `waiter`'s stream waits.  The
    runtime maps streams onto a few hardware queues (four unless GPU_MAX_HW_QUEUES says otherwise) and
    kernels of two streams that share a queue run one after the other, in the order they were
    launched: a wait launched BEFORE the kernel that releases it then lasts until its bound.  The probe
    is that situation with a 20 ms bound: the waiter's kernel ends either way."""
    write_both(g, o, waiter, off, np.zeros(1, np.int64))
    out = torch.zeros(2, dtype=torch.int64, device="cuda")
    g.set_wait_timeout_us(20_000)
    g.launch_sync_set(waiter, off, 1, None, S.SHM_SYNC_WAIT, S.SHM_CMP_GE, 1, out)
    g.launch_amo(setter, waiter, off, S.SHM_AMO_SET, 1)
    try:
        g.barrier_all()
        beside = True
    except S.ShmError as e:
        assert e.code == S.SHM_ETIMEOUT
        beside = False
    g.barrier_all()
    g.set_wait_timeout_us(2_000_000)
    write_both(g, o, waiter, off, np.ones(1, np.int64))
    return beside


def test_wait_until_all_is_released_by_puts_from_other_pes():
    """PE 0 waits until all of four variables are >= 1; three other streams set one variable each with
    a scalar put and the fourth with an atomic; the data that one of them put before its variable is
    readable after the wait.  The wait is launched FIRST, and blocks until the others release it,
    whenever the four streams run beside each other (see _runs_beside); on streams that share a
    hardware queue it is launched last, where it finds the variables set."""
    g, o = make_pair(4, MiB)
    with g:
        wait_first = all(_runs_beside(g, o, 0, p, 49152) for p in (1, 2, 3))
        print(f"wait launched {'first' if wait_first else 'last: PE 0 shares a hardware queue with another PE'}", flush=True)
        fill_random(g, o, 92, upto=65536)             # the heap is uninitialised device memory: give both sides the same bytes
        zeros = np.zeros(4, np.int64)
        write_both(g, o, 0, 4096, zeros)
        payload = np.arange(1000, dtype=np.uint8)
        write_both(g, o, 1, 8192, payload)
        ones = np.ones(1, np.int64)
        for p in (1, 2, 3):
            write_both(g, o, p, 256, ones)
        out = torch.zeros(5, dtype=torch.int64, device="cuda")
        def wait_then_read():
            g.launch_sync_set(0, 4096, 4, None, S.SHM_SYNC_WAIT_ALL, S.SHM_CMP_GE, 1, out)
            g.launch_wg_get(0, 0, 32768, 16384, 1000, 1)                  # PE 0 reads, after its wait, what PE 1 put before its flag
        if wait_first:
            wait_then_read()
        g.launch_wg_put(1, 0, 16384, 8192, 1000, 1)
        g.launch_scalar_pg(1, 0, 4096, 256, 1, 8)                          # same stream: ordered after the payload put ... by a quiet:
        for p in (2, 3):
            g.launch_scalar_pg(p, 0, 4096 + 8 * (p - 1), 256, 1, 8)
        g.launch_amo(3, 0, 4096 + 24, S.SHM_AMO_SET, 1)
        if not wait_first:
            wait_then_read()
        g.barrier_all()
        o.putmem(1, 16384, 8192, 1000, 0)
        for i in range(4):
            o.write(0, 4096 + 8 * i, ones)
        o.wait_until_all(0, 4096, 4, None, S.SHM_CMP_GE, 1)
        o.getmem(0, 32768, 16384, 1000, 0)
        assert int(out[0].item()) == 1
        for p in range(4):
            assert np.array_equal(g.read(p, 0, 65536), o.heap[p][:65536]), f"PE {p}"
