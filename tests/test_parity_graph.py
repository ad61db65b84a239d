"""GPU parity under HIP graph replay: the load/store launches are plain kernel launches on the PE's
stream, so a caller can record a sequence of them once and replay it.  The graph is replayed several
times with eager work (new source bytes, synchronisations) between the replays, and every replay is
checked against the oracle applying the same operations again."""
import numpy as np
import pytest
import torch

from oracle.shmem_oracle import SIGNAL_ADD
from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def test_recorded_sequence_of_puts_signal_and_atomic_replays_correctly():
    g, o = make_pair(3, 8 * MiB)
    with g:
        fill_random(g, o, 61, upto=6 * MiB)
        write_both(g, o, 1, 5 * MiB, np.zeros(16, np.uint8))          # signal word and tally start at zero
        sig, tally = 5 * MiB, 5 * MiB + 8
        ops = [("put", 0, 1, 2 * MiB + 3, 1024 + 1, 100003, 8), ("put", 0, 2, 3 * MiB, 4096, 262144 + 16, 64),
               ("get", 0, 1, 4 * MiB + 5, 2 * MiB + 3, 70001, 3)]
        stream = g.streams[0]
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            for kind, me, pe, d, s, n, n_wg in ops:
                (g.launch_wg_get if kind == "get" else g.launch_wg_put)(me, pe, d, s, n, n_wg)
            g.launch_wg_put_signal(0, 1, 1 * MiB + 7, 8192 + 2, 50001, sig, 3, SIGNAL_ADD, 5)
            g.launch_amo(0, 1, tally, S.SHM_AMO_FETCH_ADD, 11)
            g.launch_scalar_pg(0, 2, 1 * MiB, 512, 1000, 4, False, 2)
        rng = np.random.default_rng(62)
        for replay in range(4):
            # eager work between the replays: new source bytes on the calling PE, then a synchronisation
            fresh = rng.integers(0, 256, 300000, dtype=np.uint8)
            write_both(g, o, 0, 512, fresh)
            torch.cuda.synchronize()
            graph.replay()
            g.barrier_all()
            for kind, me, pe, d, s, n, n_wg in ops:
                (o.wg_get if kind == "get" else o.wg_put)(me, d, s, n, pe, n_wg)
            o.put_signal(0, 1 * MiB + 7, 8192 + 2, 50001, sig, 3, SIGNAL_ADD, 1, 5)
            o.atomic_fetch_add(0, tally, 11, 1)
            o.putmem(0, 1 * MiB, 512, 4000, 2)
            assert_heaps_equal(g, o, upto=6 * MiB, what=f"replay {replay}")
        assert o.signal_fetch(1, sig) == 12 and o.atomic_fetch(0, tally, 1) == 44


def test_recorded_team_collectives_replay_correctly():
    """Team launches are one kernel on the team stream once the caller orders the streams itself
    (team sync off): fcollect, a reduction, a broadcast and a team put recorded and replayed."""
    g, o = make_pair(4, 8 * MiB)
    with g:
        fill_random(g, o, 63, upto=7 * MiB)
        g.set_team_sync(False)
        stream = g.streams[0]
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            g.launch_fcollect(1 * MiB, 256, 100000 + 16, 8, S.SHM_PATH_LDST)
            g.launch_reduce(2 * MiB, 1 * MiB, 30001, S.SHM_INT32, S.SHM_OP_SUM, 16, S.SHM_REDUCE_SPLIT)
            g.launch_broadcast(3 * MiB + 16, 2 * MiB, 120000, 2, 4, S.SHM_PATH_LDST)
            g.launch_wg_put_all(1, 4 * MiB, 3 * MiB + 16, 120000, 8, S.SHM_PATH_LDST)
        rng = np.random.default_rng(64)
        for replay in range(3):
            for p in range(4):
                write_both(g, o, p, 256, rng.integers(0, 256, 100016, dtype=np.uint8))
            torch.cuda.synchronize()
            graph.replay()
            g.barrier_all()
            o.fcollect(1 * MiB, 256, 100016)
            o.reduce(2 * MiB, 1 * MiB, 30001, np.int32, "sum")
            o.broadcast(3 * MiB + 16, 2 * MiB, 120000, 2)
            before = [h.copy() for h in o.heap]
            for p in range(4):
                o.heap[(p + 1) % 4][4 * MiB:4 * MiB + 120000] = before[p][3 * MiB + 16:3 * MiB + 16 + 120000]
            assert_heaps_equal(g, o, upto=7 * MiB, what=f"replay {replay}")


def test_recorded_long_team_put_and_get_replay_correctly():
    """The long team put draws its pieces from counters in the heap's tail that the last group through
    sets back: two such launches recorded back to back (a put and a get, 33 MiB x 4 PEs, ragged last
    tile, byte tail) and replayed four times with fresh source bytes in between."""
    g, o = make_pair(4, 112 * MiB)
    with g:
        fill_random(g, o, 65, upto=108 * MiB)
        g.set_team_sync(False)
        n = 33 * MiB + 65536 + 16 * 5 + 3
        stream = g.streams[0]
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            g.launch_wg_put_all(1, 36 * MiB, 32, n, 1024, S.SHM_PATH_LDST)
            g.launch_wg_get_all(3, 72 * MiB + 16, 36 * MiB, n, 128, S.SHM_PATH_LDST)
        rng = np.random.default_rng(66)
        for replay in range(4):
            for p in range(4):
                write_both(g, o, p, 4096 * (replay + 1), rng.integers(0, 256, 200000, dtype=np.uint8))
            torch.cuda.synchronize()
            graph.replay()
            g.barrier_all()
            before = [h.copy() for h in o.heap]
            for p in range(4):
                o.heap[(p + 1) % 4][36 * MiB:36 * MiB + n] = before[p][32:32 + n]
            before = [h.copy() for h in o.heap]
            for p in range(4):
                o.heap[p][72 * MiB + 16:72 * MiB + 16 + n] = before[(p + 3) % 4][36 * MiB:36 * MiB + n]
            assert_heaps_equal(g, o, upto=108 * MiB, what=f"replay {replay}")


def test_recorded_long_collectives_replay_correctly():
    """A long split reduction and a long broadcast draw their pieces from one counter pair per PE that
    the last group through sets back: recorded back to back (2 PEs; slices of 96 tiles and a ragged
    rest; a block of 33 MiB and a few vectors) and replayed three times with fresh bytes in between."""
    g, o = make_pair(2, 112 * MiB)
    with g:
        fill_random(g, o, 67, upto=108 * MiB)
        g.set_team_sync(False)
        nel = 4 * (2 * (96 * 4096 + 500) - 1) + 3                     # int32 elements, 12 MiB per PE
        n = 33 * MiB + 16 * 7
        rsrc, rdst, bsrc, bdst = 64, 14 * MiB + 16, 30 * MiB, 70 * MiB + 32
        stream = g.streams[0]
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            g.launch_reduce(rdst, rsrc, nel, S.SHM_INT32, S.SHM_OP_SUM, 128, S.SHM_REDUCE_SPLIT)
            g.launch_broadcast(bdst, bsrc, n, 1, 1024, S.SHM_PATH_LDST)
            g.launch_reduce(rdst + 14 * MiB, rdst, nel, S.SHM_INT32, S.SHM_OP_MAX, 1024, S.SHM_REDUCE_SPLIT)
        rng = np.random.default_rng(68)
        for replay in range(3):
            for p in range(2):
                write_both(g, o, p, rsrc + 4096 * replay, rng.integers(0, 256, 300000, dtype=np.uint8))
                write_both(g, o, p, bsrc + 8192 * replay, rng.integers(0, 256, 300000, dtype=np.uint8))
            torch.cuda.synchronize()
            graph.replay()
            g.barrier_all()
            o.reduce(rdst, rsrc, nel, np.int32, "sum")
            o.broadcast(bdst, bsrc, n, 1)
            o.reduce(rdst + 14 * MiB, rdst, nel, np.int32, "max")
            assert_heaps_equal(g, o, upto=108 * MiB, what=f"replay {replay}")
