"""GPU parity on random PROGRAMS: a few hundred operations of every family, mixed, on several PEs'
streams at once.  The oracle runs them one after another.  On the GPU two operations are ordered
when they are on the same PE's stream, or when one of them is a team launch (which joins and forks
all PE streams); the test inserts a barrier_all only between operations that conflict (one writes
what the other touches) and are ordered by neither rule.  Heaps are compared at every barrier the
program needed and at the end, so a missing wait between kernels, engines and runtime copies shows."""
import numpy as np
import pytest

from oracle.shmem_oracle import OracleError, SIGNAL_ADD, SIGNAL_SET
from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair

pytestmark = pytest.mark.gpu

MiB = 1 << 20
ARENA = 3 * MiB // 2          # operations stay in the first 1.5 MiB; the rest of the heap is canary
CHAIN = ARENA + 400 * 1024    # eight signal words per PE for the put-signal / wait chains, beyond the reach of every other
                              # operation (those start inside the arena and are at most 300 000 bytes long)


class Tracker:
    """What has been issued since the last point every stream was ordered behind."""

    def __init__(self):
        self.pending = []      # [stream, [(pe, lo, hi, is_write)], set of streams ordered behind this entry]

    def conflicts(self, stream, touched):
        for other_stream, regions, behind in self.pending:
            if other_stream == stream or stream in behind:
                continue
            for (p, lo, hi, w) in regions:
                for (q, a, b, v) in touched:
                    if p == q and (w or v) and lo < b and a < hi:
                        return True
        return False

    def add(self, stream, touched):
        self.pending.append([stream, touched, set()])
        return len(self.pending) - 1

    def order_behind(self, producer_stream, upto, consumer_stream):
        """A satisfied wait on consumer_stream for a signal whose put was entry `upto` of producer_stream:
        everything that stream enqueued up to that entry is now ordered before the consumer's later work."""
        for entry in self.pending[:upto + 1]:
            if entry[0] == producer_stream:
                entry[2].add(consumer_stream)

    def clear(self):
        self.pending = []


def _program(g, o, npes, seed, n_ops, with_engines):
    # every operation here goes through the library, so the cheap tracked ordering must serve as well as the full one
    g.set_team_sync(S.SHM_TEAM_SYNC_TRACKED if seed % 2 else S.SHM_TEAM_SYNC_FULL)
    rng = np.random.default_rng(seed)
    tr = Tracker()
    paths = [S.SHM_PATH_LDST, S.SHM_PATH_LDST, S.SHM_PATH_MEMCPY] + ([S.SHM_PATH_SDMA, S.SHM_PATH_AUTO] if with_engines else [])
    modes = [0, 0, 1, 2, 3, 4] if with_engines else [0]        # device-initiated transfers: the engine modes need the proxy
    issued = barriers = 0
    counts = {}
    # signal words of their own, outside the arena, only ever ADDed to by put-with-signal: a wait for the
    # running total is then a wait for every put issued so far, and orders the waiting stream behind them
    chain_total = {}           # (pe, k) -> total added so far
    chain_producers = {}       # (pe, k) -> [(stream, tracker entry, payload offset, payload bytes)] since the streams were last ordered
    for p in range(npes):
        zero = np.zeros(64, np.uint8)
        g.write(p, CHAIN, zero), o.write(p, CHAIN, zero)
    if with_engines:
        g.proxy_start()
        g.set_cutover(1, 100000)          # AUTO by one group takes the engines from 100 000 bytes

    def clear_all():
        tr.clear()                 # every stream has been ordered behind everything issued so far ...
        chain_producers.clear()    # ... so there is no put left that a wait would still have to order

    def off(align=1, span=ARENA):
        return int(rng.integers(0, span)) // align * align

    def size():
        return int(rng.choice([0, 1, 8, 100, 4096, 70001, 300000])) if rng.integers(4) else int(rng.integers(0, 200000))

    for i in range(n_ops):
        kind = str(rng.choice(["wg_put", "wg_get", "host_put", "host_get", "put_signal", "amo", "fcollect", "collect", "broadcast", "reduce",
                               "iput", "iget", "scalar", "thread", "dev_put", "dev_get", "wave", "chain_put", "chain_wait"]))
        me, pe = int(rng.integers(npes)), int(rng.integers(npes))
        team = kind in ("fcollect", "collect", "broadcast", "reduce")
        try:
            if kind in ("wg_put", "wg_get", "host_put", "host_get", "thread", "dev_put", "dev_get"):
                d, s, n = off(), off(), size()
                n_wg = int(rng.choice([1, 2, 7, 64]))
                is_get = kind in ("wg_get", "host_get", "dev_get") or (kind == "thread" and bool(rng.integers(2)))
                if kind == "thread":
                    n = min(n, 5000)
                (o.getmem if is_get else o.putmem)(me, d, s, n, pe)
                touched = [(pe, s, s + n, False), (me, d, d + n, True)] if is_get else [(me, s, s + n, False), (pe, d, d + n, True)]
                path = int(rng.choice(paths))
                if kind in ("wg_put", "wg_get"):
                    call = lambda: (g.launch_wg_get if is_get else g.launch_wg_put)(me, pe, d, s, n, n_wg, path)
                elif kind in ("host_put", "host_get"):
                    call = lambda: (g.getmem if is_get else g.putmem)(me, d, s, n, pe)
                elif kind == "thread":
                    call = lambda: g.launch_thread_rma(me, pe, d, s, n, is_get)
                else:
                    wg_size, mode = int(rng.choice([64, 256, 1024])), int(rng.choice(modes))
                    call = lambda: g.launch_rma_device_initiated(me, pe, d, s, n, min(n_wg, 16), is_get, mode, cutover=50000, cover=4096,
                                                                 wg_size=wg_size)
            elif kind == "put_signal":
                d, s, n, sig = off(), off(), size(), off(8)
                op = SIGNAL_ADD if rng.integers(2) else SIGNAL_SET
                val, n_wg = int(rng.integers(1, 1 << 40)), int(rng.choice([1, 3, 16]))
                o.put_signal(me, d, s, n, sig, val, op, pe, n_wg)
                touched = [(me, s, s + n, False), (pe, d, d + n, True), (pe, sig, sig + 8, True)]
                call = lambda: g.launch_wg_put_signal(me, pe, d, s, n, sig, val, op, n_wg)
            elif kind == "chain_put":
                d, s, n, k = off(), off(), size(), int(rng.integers(8))
                val, n_wg = int(rng.integers(1, 1000)), int(rng.choice([1, 3, 16]))
                o.put_signal(me, d, s, n, CHAIN + 8 * k, val, SIGNAL_ADD, pe, n_wg)
                touched = [(me, s, s + n, False), (pe, d, d + n, True)]
                call = lambda: g.launch_wg_put_signal(me, pe, d, s, n, CHAIN + 8 * k, val, SIGNAL_ADD, n_wg)
                chain = (pe, k, val, d, n)
            elif kind == "chain_wait":
                waiting = [key for key, producers in chain_producers.items() if producers]
                if not waiting:
                    continue
                pe, k = waiting[int(rng.integers(len(waiting)))]
                me = pe                                          # a PE waits on its own signal word ...
                o.signal_wait_until(pe, CHAIN + 8 * k, S.SHM_CMP_GE, chain_total[(pe, k)])
                _, _, d, n = chain_producers[(pe, k)][-1]
                scratch = off(1, ARENA - n)
                o.putmem(pe, scratch, d, n, pe)                  # ... and then reads the payload that came with it
                for stream, entry, _, _ in chain_producers[(pe, k)]:
                    tr.order_behind(stream, entry, pe)
                chain_producers[(pe, k)] = []
                touched = [(pe, d, d + n, False), (pe, scratch, scratch + n, True)]
                total = chain_total[(pe, k)]
                call = lambda: (g.launch_signal_wait_until(pe, CHAIN + 8 * k, S.SHM_CMP_GE, total), g.launch_wg_put(pe, pe, scratch, d, n, 4))
            elif kind == "wave":
                d, s, back, n = off(), off(), off(), min(size(), 100000)
                n_waves = int(rng.choice([1, 3, 8, 64]))
                flag, out = off(8, ARENA - 8 * n_waves), off(8, ARENA - 8 * n_waves)
                if me == pe or len({(flag, 8 * n_waves), (out, 8 * n_waves)}) < 2:
                    continue                                  # producer and consumer waves are two PEs' work
                regions = [(d, n), (back, n), (flag, 8 * n_waves), (out, 8 * n_waves)]
                if any(a < b + lb and b < a + la for i, (a, la) in enumerate(regions) for (b, lb) in regions[i + 1:] if la and lb):
                    continue                                  # the library wants them disjoint on the target PE
                o.wave_exchange(me, pe, d, s, back, n, n_waves, flag, out)      # raises if it is not a defined operation ...
                g.barrier_all()                                                 # ... else the flag words start at zero on both sides
                barriers += 1
                clear_all()
                g.write(pe, flag, np.zeros(8 * n_waves, np.uint8))
                touched = [(me, s, s + n, False), (pe, d, d + n, True), (pe, back, back + n, True), (pe, flag, flag + 8 * n_waves, True),
                           (pe, out, out + 8 * n_waves, True)]
                call = lambda: g.launch_wave_exchange(me, pe, d, s, back, n, n_waves, flag, out)
            elif kind == "amo":
                at, v = off(8), int(rng.integers(-1000, 1000))
                o.atomic_fetch_add(me, at, v, pe)
                touched = [(pe, at, at + 8, True)]
                call = lambda: g.launch_amo(me, pe, at, S.SHM_AMO_FETCH_ADD, v)
            elif kind == "fcollect":
                n = min(size(), ARENA // (2 * npes))
                d, s = off(1, ARENA - n * npes), off()
                o.fcollect(d, s, n)
                path, n_wg = int(rng.choice(paths)), int(rng.choice([1, 8, 32]))
                call = lambda: g.launch_fcollect(d, s, n, n_wg, path)
            elif kind == "collect":
                sizes = [min(size(), ARENA // (2 * npes)) for _ in range(npes)]
                d, s = off(1, ARENA - sum(sizes)), off()
                o.collect(d, s, sizes)
                call = lambda: g.launch_collect(d, s, sizes, int(rng.choice([1, 8])))
            elif kind == "broadcast":
                d, s, n, root = off(), off(), size(), pe
                o.broadcast(d, s, n, root)
                path = int(rng.choice(paths))
                call = lambda: g.launch_broadcast(d, s, n, root, int(rng.choice([1, 4, 32])), path)
            elif kind == "reduce":
                dt, code = [(np.uint8, S.SHM_UINT8), (np.int16, S.SHM_INT16), (np.int32, S.SHM_INT32), (np.uint64, S.SHM_UINT64)][int(rng.integers(4))]
                op, op_code = [("sum", S.SHM_OP_SUM), ("min", S.SHM_OP_MIN), ("max", S.SHM_OP_MAX), ("prod", S.SHM_OP_PROD),
                               ("xor", S.SHM_OP_XOR), ("and", S.SHM_OP_AND), ("or", S.SHM_OP_OR)][int(rng.integers(7))]
                nelems = size() // np.dtype(dt).itemsize
                d, s = off(16), off(16)
                o.reduce(d, s, nelems, dt, op)
                algo = S.SHM_REDUCE_SPLIT if rng.integers(2) else S.SHM_REDUCE_DUPLICATE
                call = lambda: g.launch_reduce(d, s, nelems, code, op_code, int(rng.choice([1, 8, 64])), algo)
            elif kind in ("iput", "iget"):
                elem = int(rng.choice([1, 2, 4, 8, 16]))
                ds, ss, nelems = int(rng.integers(1, 6)), int(rng.integers(1, 6)), int(rng.integers(0, 3000))
                d, s = off(elem), off(elem)
                is_get = kind == "iget"
                (o.iget if is_get else o.iput)(me, d, s, ds, ss, nelems, elem, pe)
                dspan = ((nelems - 1) * ds + 1) * elem if nelems else 0
                sspan = ((nelems - 1) * ss + 1) * elem if nelems else 0
                touched = [(pe, s, s + sspan, False), (me, d, d + dspan, True)] if is_get else [(me, s, s + sspan, False), (pe, d, d + dspan, True)]
                n_wg = int(rng.choice([0, 1, 5]))
                call = lambda: (g.launch_iget if is_get else g.launch_iput)(me, pe, d, s, ds, ss, nelems, elem, n_wg)
            else:       # scalar p / g
                elem = int(rng.choice([1, 2, 4, 8]))
                nelems, is_get = int(rng.integers(0, 5000)), bool(rng.integers(2))
                d, s = off(elem), off(elem)
                (o.getmem if is_get else o.putmem)(me, d, s, nelems * elem, pe)
                n = nelems * elem
                touched = [(pe, s, s + n, False), (me, d, d + n, True)] if is_get else [(me, s, s + n, False), (pe, d, d + n, True)]
                call = lambda: g.launch_scalar_pg(me, pe, d, s, nelems, elem, is_get, int(rng.choice([1, 3])))
        except OracleError:
            continue                      # not a defined operation (overlap, range): not issued on either side
        if team:
            call()                        # joins and forks every PE stream: ordered against everything
            clear_all()
        else:
            if tr.conflicts(me, touched):
                g.barrier_all()
                barriers += 1
                clear_all()
            call()
            entry = tr.add(me, touched)
            if kind == "chain_put":
                pe_, k_, val_, d_, n_ = chain
                chain_total[(pe_, k_)] = chain_total.get((pe_, k_), 0) + val_
                chain_producers.setdefault((pe_, k_), []).append((me, entry, d_, n_))
        issued += 1
        counts[kind] = counts.get(kind, 0) + 1
        if i % 40 == 39:
            g.barrier_all()
            clear_all()
            assert_heaps_equal(g, o, what=f"seed {seed}, after operation {i} ({kind}); issued so far: {counts}")
    if with_engines:
        g.proxy_stop()
    g.barrier_all()
    assert_heaps_equal(g, o, what=f"seed {seed}, end")
    return issued, barriers, counts


@pytest.mark.parametrize("npes,seed,with_engines", [(2, 101, False), (3, 102, True), (5, 103, False), (8, 104, True), (4, 105, True),
                                                    (2, 106, True), (16, 107, False), (3, 108, True), (4, 1038, True)])
def test_random_program(npes, seed, with_engines):
    g, o = make_pair(npes, 2 * MiB)
    with g:
        fill_random(g, o, seed)
        issued, barriers, counts = _program(g, o, npes, seed, 600, with_engines)
        print(f"npes {npes}: {issued} operations, {barriers} barriers for conflicts, {counts}")
        assert issued > 400 and len(counts) == 19, (issued, counts)
        assert barriers < issued // 2, "the program should mostly rely on stream order and team joins, not on host barriers"
