"""GPU parity at the limits the header states: SHM_MAX_PES logical PEs, the largest group count,
single-byte and empty messages on every team form."""
import numpy as np
import pytest

from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def test_max_pes_every_team_form():
    npes = S.SHM_MAX_PES
    g, o = make_pair(npes, 2 * MiB)
    with g:
        fill_random(g, o, 71, upto=MiB + 512 * 1024)
        # team put and get, shift 5
        g.launch_wg_put_all(5, MiB // 2 + 3, 7, 100003, 8, S.SHM_PATH_LDST)
        g.barrier_all()
        snap = [h.copy() for h in o.heap]
        for p in range(npes):
            o.heap[(p + 5) % npes][MiB // 2 + 3:MiB // 2 + 3 + 100003] = snap[p][7:7 + 100003]
        assert_heaps_equal(g, o, upto=MiB + 512 * 1024, what="team put")
        # fcollect: 32 blocks of 4 KiB + 16
        g.launch_fcollect(MiB, 64, 4112, 4, S.SHM_PATH_LDST)
        g.barrier_all()
        o.fcollect(MiB, 64, 4112)
        assert_heaps_equal(g, o, upto=MiB + 512 * 1024, what="fcollect")
        # reductions, both algorithms
        for algo in (S.SHM_REDUCE_DUPLICATE, S.SHM_REDUCE_SPLIT):
            g.launch_reduce(MiB + 256 * 1024, 4096, 10007, S.SHM_INT32, S.SHM_OP_SUM, 8, algo)
            g.barrier_all()
            o.reduce(MiB + 256 * 1024, 4096, 10007, np.int32, "sum")
            assert_heaps_equal(g, o, upto=MiB + 512 * 1024, what=f"reduce {algo}")
        rng = np.random.default_rng(74)                 # finite floats: random bytes would hold NaNs
        for p in range(npes):
            write_both(g, o, p, 8192, rng.standard_normal(5001).astype(np.float32).view(np.uint8))
        g.launch_reduce_sum_f32(MiB + 384 * 1024, 8192, 5001, 8, S.SHM_REDUCE_DUPLICATE)
        g.barrier_all()
        # broadcast from the last PE
        g.launch_broadcast(MiB + 300 * 1024, 128, 30001, npes - 1, 4, S.SHM_PATH_LDST)
        g.barrier_all()
        o.broadcast(MiB + 300 * 1024, 128, 30001, npes - 1)
        got = g.read(0, MiB + 384 * 1024, 4 * 5001).view(np.float32)
        want = o.reduce_sum_f32(MiB + 384 * 1024, 8192, 5001)["f32"]
        assert got.tobytes() == np.asarray(want, np.float32).tobytes()
        assert_heaps_equal(g, o, upto=MiB + 512 * 1024, what="broadcast + f32 reduce")


def test_max_pes_device_barrier_rounds():
    npes = S.SHM_MAX_PES
    g, o = make_pair(npes, MiB)
    with g:
        fill_random(g, o, 72, upto=512 * 1024)
        for rep in range(2):
            g.launch_barrier_exchange(64 * 1024, 128 + rep, 256 * 1024, 3001, 6)
            g.barrier_all()
            o.barrier_exchange(64 * 1024, 128 + rep, 256 * 1024, 3001, 6)
            assert_heaps_equal(g, o, upto=512 * 1024, what=f"rep {rep}")


@pytest.mark.parametrize("n", [0, 1, 15, 1000])
def test_largest_group_count_on_tiny_messages(n):
    g, o = make_pair(2, MiB)
    with g:
        fill_random(g, o, 73, upto=256 * 1024)
        g.launch_wg_put(0, 1, 128 * 1024 + 1, 3, n, 1 << 20, S.SHM_PATH_LDST)     # a million groups, nearly all without a share
        g.launch_wg_get(1, 0, 200 * 1024, 5, n, 1 << 20, S.SHM_PATH_LDST)
        g.barrier_all()
        o.wg_put(0, 128 * 1024 + 1, 3, n, 1, 1 << 20)
        o.wg_get(1, 200 * 1024, 5, n, 0, 1 << 20)
        assert_heaps_equal(g, o, upto=256 * 1024)
        with pytest.raises(S.ShmError):
            g.launch_wg_put(0, 1, 128 * 1024, 0, n, (1 << 20) + 1, S.SHM_PATH_LDST)
