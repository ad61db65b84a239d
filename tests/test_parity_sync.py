"""GPU parity: device-side sync/barrier among PEs and broadcast."""
import numpy as np
import pytest
import torch

from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20


@pytest.mark.parametrize("npes,n,rounds", [(2, 1000, 2), (8, 65536 + 24, 8), (16, 4096, 5), (1, 100, 1), (5, 300001, 4)])
def test_barrier_exchange(npes, n, rounds):
    g, o = make_pair(npes, 16 * MiB)
    with g:
        fill_random(g, o, 41, upto=14 * MiB)
        src, dst, acc = 64, MiB, 8 * MiB
        for rep in range(3):                      # the sync counters and epochs carry over from launch to launch
            g.launch_barrier_exchange(dst, src + rep, acc, n, rounds)
            g.barrier_all()
            o.barrier_exchange(dst, src + rep, acc, n, rounds)
            assert_heaps_equal(g, o, upto=14 * MiB, what=f"rep {rep}")


def test_sync_all_counts_and_is_timed():
    g, o = make_pair(8, MiB)
    with g:
        t = torch.zeros(2, dtype=torch.int64, device="cuda")
        for with_quiet in (0, 1):
            t[0], t[1] = -1, 0
            torch.cuda.synchronize()
            g.launch_sync_all(100, with_quiet, t)
            g.barrier_all()
            a, b = (int(v) & ((1 << 64) - 1) for v in t.tolist())
            us = (b - a) / g.wall_clock_khz() * 1e3 / 100
            assert 0.1 < us < 1000, us


@pytest.mark.parametrize("path", [S.SHM_PATH_LDST, S.SHM_PATH_SDMA, S.SHM_PATH_MEMCPY])
@pytest.mark.parametrize("npes,n,root,n_wg,soff,doff", [(8, 100003, 3, 4, 5, 9), (2, 16, 1, 1, 0, 0), (5, 3 * MiB + 64, 0, 64, 0, 0),
                                                       (4, 0, 2, 8, 0, 0), (3, 100003, 1, 7, 16, 32), (16, 65536 + 5, 15, 2, 0, 48),
                                                       (1, 1000, 0, 3, 0, 0), (6, 4 * 256 * 16 * 5 + 7, 2, 5, 0, 0)])
def test_broadcast(path, npes, n, root, n_wg, soff, doff):
    g, o = make_pair(npes, 16 * MiB)
    with g:
        fill_random(g, o, 42, upto=12 * MiB)
        src, dst = 1024 + soff, 6 * MiB + doff
        g.launch_broadcast(dst, src, n, root, n_wg, path)
        g.barrier_all()
        o.broadcast(dst, src, n, root)
        assert_heaps_equal(g, o, upto=12 * MiB)


@pytest.mark.parametrize("npes,n,root,n_wg", [(8, 32 * MiB, 2, 1024), (3, 32 * MiB + 65536 + 16 * 3 + 5, 0, 256), (5, 33 * MiB - 16, 4, 255)])
def test_long_broadcast_by_ticket(npes, n, root, n_wg):
    """From 32 MiB, 16-byte-aligned offsets and a group per compute unit asked (256), that many groups draw 16 KiB
    pieces of the root's block by ticket: whole tiles only; a rest after the whole tiles and a byte tail; one group too
    few (the grid-strided push then).  Twice in a row with other source bytes: the counters were set back."""
    g, o = make_pair(npes, 72 * MiB)
    rng = np.random.default_rng(44)
    with g:
        fill_random(g, o, 44, upto=70 * MiB)
        src, dst = 48, 35 * MiB + 16
        for rep in range(2):
            g.launch_broadcast(dst, src, n, root, n_wg, S.SHM_PATH_LDST)
            g.barrier_all()
            o.broadcast(dst, src, n, root)
            assert_heaps_equal(g, o, upto=70 * MiB, what=f"launch {rep}")
            write_both(g, o, root, src + 8192, rng.integers(0, 256, 300000, dtype=np.uint8))


@pytest.mark.parametrize("npes,sizes,n_wg,soff,doff", [
    (4, [100003, 0, 37, 1], 4, 5, 9), (8, [4096 * (p + 1) for p in range(8)], 16, 0, 0), (3, [0, 0, 0], 2, 0, 0),
    (5, [MiB + 3, 17, MiB // 2, 0, 65536], 64, 16, 32), (1, [1000], 1, 1, 2)])
def test_collect(npes, sizes, n_wg, soff, doff):
    g, o = make_pair(npes, 16 * MiB)
    with g:
        fill_random(g, o, 43, upto=12 * MiB)
        src, dst = 1024 + soff, 6 * MiB + doff
        g.launch_collect(dst, src, sizes, n_wg)
        g.barrier_all()
        o.collect(dst, src, sizes)
        assert_heaps_equal(g, o, upto=12 * MiB)
        with pytest.raises(S.ShmError):
            g.launch_collect(dst, src, [16 * MiB] + [0] * (npes - 1), n_wg)


@pytest.mark.parametrize("sizes,n_wg", [
    ([9 * MiB + 16 * 37, 0, 8 * MiB, 16, 65536 * 3 + 48, 2 * MiB + 16, 8 * MiB + 65536 - 16, 32], 32),      # all on 16 bytes: pieces by ticket
    ([9 * MiB + 16 * 37, 0, 8 * MiB, 16, 65536 * 3 + 48, 2 * MiB + 16, 8 * MiB + 65536 - 16, 32], 1024),
    ([8 * MiB + 5, 4 * MiB, 3, 0, MiB + 16, 65536, 9 * MiB, 77], 64)])                                     # some blocks begin at odd bytes
def test_collect_of_long_blocks(sizes, n_wg):
    """Eight PEs, blocks of 0 bytes to 9 MiB: with every block on multiples of 16 bytes and a group per
    compute unit or more asked for, the groups draw 16 KiB pieces by ticket (twice in a row, so that the
    second launch depends on the first having set the counters back); with blocks at odd bytes the
    kernel pushes those the general way and the others on tiles."""
    npes = 8
    g, o = make_pair(npes, 56 * MiB)
    with g:
        fill_random(g, o, 44, upto=52 * MiB)
        src, dst = 4096, 12 * MiB + 32
        rng = np.random.default_rng(45)
        for rep in range(2):
            g.launch_collect(dst, src, sizes, n_wg)
            g.barrier_all()
            o.collect(dst, src, sizes)
            assert_heaps_equal(g, o, upto=52 * MiB, what=f"launch {rep}")
            for p in range(npes):
                write_both(g, o, p, src + 8192 * p, rng.integers(0, 256, 200000, dtype=np.uint8))


def test_collectives_on_auto_follow_their_own_cutover():
    """AUTO below and above the collective's threshold (moved down so that small cases cross it):
    the same bytes either way, and the answer of shm_choose_collective_path changes at the threshold."""
    g, o = make_pair(4, 16 * MiB)
    FC, BC = S.SHM_COLL_FCOLLECT, S.SHM_COLL_BROADCAST
    with g:
        fill_random(g, o, 44, upto=12 * MiB)
        g.set_collective_cutover(FC, 2, 50000)
        g.set_collective_cutover(BC, 8, 70000)
        assert g.choose_collective_path(FC, 49999, 2) == S.SHM_PATH_LDST and g.choose_collective_path(FC, 50000, 2) == S.SHM_PATH_MEMCPY
        assert g.choose_collective_path(BC, 69999, 8) == S.SHM_PATH_LDST and g.choose_collective_path(BC, 70000, 8) == S.SHM_PATH_MEMCPY
        for n in (49999, 50000, 300007):
            g.launch_fcollect(2 * MiB + 3, 256 + 1, n, 2, S.SHM_PATH_AUTO)
            o.fcollect(2 * MiB + 3, 256 + 1, n)
            g.launch_broadcast(6 * MiB + 5, 1024 + n % 7, n + 20000, n % 4, 8, S.SHM_PATH_AUTO)     # 69999, 70000, 320007 bytes
            o.broadcast(6 * MiB + 5, 1024 + n % 7, n + 20000, n % 4)
            g.barrier_all()
            assert_heaps_equal(g, o, upto=12 * MiB, what=f"n {n}")


@pytest.mark.parametrize("mode", [S.SHM_TEAM_SYNC_FULL, S.SHM_TEAM_SYNC_TRACKED])
@pytest.mark.parametrize("empty", ["reduce", "reduce_sum_f32", "fcollect", "collect", "broadcast"])
def test_an_empty_team_launch_still_orders_the_streams(empty, mode):
    """A slow put on PE 1's stream, a team launch with nothing to move, then -- with no host barrier --
    a get on PE 0's stream that reads what the put wrote: the team launch's join/fork is what orders
    the two, also when it has no kernel to run."""
    g, o = make_pair(3, 80 * MiB)
    with g:
        g.set_team_sync(mode)
        fill_random(g, o, 45, upto=72 * MiB)
        n = 20 * MiB + 5
        for rep in range(3):
            src, mid, dst = 1024 + rep, 24 * MiB + 16 * rep, 48 * MiB + 3 * rep
            g.launch_wg_put(1, 2, mid, src, n, 1)                     # one group: slow enough to still be running
            o.wg_put(1, mid, src, n, 2, 1)
            if empty == "reduce":
                g.launch_reduce(4096, 65536, 0, S.SHM_INT32, S.SHM_OP_SUM, 4)
            elif empty == "reduce_sum_f32":
                g.launch_reduce_sum_f32(4096, 65536, 0, 4)
            elif empty == "fcollect":
                g.launch_fcollect(4096, 65536, 0, 4)
            elif empty == "collect":
                g.launch_collect(4096, 65536, [0, 0, 0], 4)
            else:
                g.launch_broadcast(4096, 65536, 0, 1, 4)
            g.launch_wg_get(0, 2, dst, mid, n, 64)
            o.wg_get(0, dst, mid, n, 2, 64)
            g.barrier_all()
            assert_heaps_equal(g, o, upto=72 * MiB, what=f"{empty}, repetition {rep}")


@pytest.mark.parametrize("mode", [S.SHM_TEAM_SYNC_FULL, S.SHM_TEAM_SYNC_TRACKED])
@pytest.mark.parametrize("kind", ["fcollect", "broadcast", "put_all"])
def test_team_launch_on_the_engines_orders_other_pes_later_work(kind, mode):
    """Engine transfers are not on the streams.  With team sync on, work that another PE enqueues
    right after a team launch on the copy engines -- here a get of what the engines deliver to a
    third PE -- must find it delivered."""
    g, o = make_pair(4, 136 * MiB)
    with g:
        g.set_team_sync(mode)
        fill_random(g, o, 46, upto=132 * MiB)
        n = 20 * MiB + 48                                              # a third of a millisecond per engine transfer
        src, dst, back = 4096, 24 * MiB, 108 * MiB
        if kind == "fcollect":
            g.launch_fcollect(dst, src, n, 1, S.SHM_PATH_SDMA)
            o.fcollect(dst, src, n)
            take = dst + 3 * n                                         # block of PE 3, delivered to PE 2 by PE 3's transfer
        elif kind == "broadcast":
            g.launch_broadcast(dst, src, n, 3, 1, S.SHM_PATH_SDMA)
            o.broadcast(dst, src, n, 3)
            take = dst
        else:
            g.launch_wg_put_all(1, dst, src, n, 1, S.SHM_PATH_SDMA)
            for p in range(4):
                o.putmem(p, dst, src, n, (p + 1) % 4)
            take = dst
        g.launch_wg_get(0, 2, back, take, n, 64)                      # PE 0 reads PE 2's copy at once
        o.wg_get(0, back, take, n, 2, 64)
        g.barrier_all()
        assert_heaps_equal(g, o, upto=132 * MiB, what=kind)
