"""GPU parity: device-side sync/barrier among PEs and broadcast."""
import numpy as np
import pytest
import torch

from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair

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
