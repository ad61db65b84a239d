"""GPU parity: single-thread put/get, strided put/get, and device-initiated gets (blocking,
non-blocking, engine start-up covered by loads/stores) with the landed bytes read inside the kernel."""
import numpy as np
import pytest
import torch

from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair

pytestmark = pytest.mark.gpu

MiB = 1 << 20


@pytest.mark.parametrize("is_get", [False, True])
@pytest.mark.parametrize("n,sa,da", [(0, 0, 0), (1, 3, 5), (15, 1, 0), (4096, 0, 0), (100003, 7, 9), (65536 + 48, 16, 32), (513, 0, 8),
                                     (8, 0, 0), (12, 8, 8), (15, 4, 4), (7, 8, 16), (31, 8, 24), (24, 8, 0), (14, 2, 6)])
def test_single_thread_put_get(is_get, n, sa, da):
    """Also the ends of a message that a lone thread moves in 8- and 4-byte pieces where source and
    destination are both aligned for them (8 bytes at 0/0, 8 + 4 at 8/8, 4 + bytes at 4/4 ...)."""
    g, o = make_pair(3, 4 * MiB)
    with g:
        fill_random(g, o, 61, upto=3 * MiB)
        src, dst = 4096 + sa, 2 * MiB + da
        g.launch_thread_rma(1, 2, dst, src, n, is_get, reps=2)
        g.quiet(1)
        (o.getmem if is_get else o.putmem)(1, dst, src, n, 2)
        assert_heaps_equal(g, o, upto=3 * MiB)
        # same PE, disjoint ranges
        g.launch_thread_rma(0, 0, dst, src, n, is_get)
        g.quiet(0)
        (o.getmem if is_get else o.putmem)(0, dst, src, n, 0)
        assert_heaps_equal(g, o, upto=3 * MiB)


@pytest.mark.parametrize("elem", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("n_wg", [0, 1, 7, 64])
def test_strided_put_get(elem, n_wg):
    g, o = make_pair(3, 8 * MiB)
    with g:
        fill_random(g, o, 62 + elem, upto=6 * MiB)
        cases = [(3, 2, 10007), (1, 5, 4099), (7, 1, 2500), (1, 1, 30011), (2, 2, 1), (4, 4, 0), (13, 11, 777)]
        if n_wg == 0:
            cases = [(d, s, min(n, 1200)) for d, s, n in cases]           # one work-item: keep it short
        for i, (ds, ss, n) in enumerate(cases):
            me, pe = i % 3, (i + 2) % 3
            src, dst = 16 * elem, 3 * MiB + elem
            g.launch_iput(me, pe, dst, src, ds, ss, n, elem, n_wg)
            g.quiet(me)
            o.iput(me, dst, src, ds, ss, n, elem, pe)
            assert_heaps_equal(g, o, upto=6 * MiB, what=f"iput case {i}")
            g.launch_iget(me, pe, dst + 1 * MiB, src + elem, ds, ss, n, elem, n_wg)
            g.quiet(me)
            o.iget(me, dst + 1 * MiB, src + elem, ds, ss, n, elem, pe)
            assert_heaps_equal(g, o, upto=6 * MiB, what=f"iget case {i}")


def test_strided_same_pe_and_errors():
    g, o = make_pair(2, 2 * MiB)
    with g:
        fill_random(g, o, 63, upto=MiB + 4096)
        g.launch_iput(0, 0, MiB // 2, 0, 2, 3, 5000, 4, 4)        # scatter within one PE, disjoint spans
        g.quiet(0)
        o.iput(0, MiB // 2, 0, 2, 3, 5000, 4, 0)
        assert_heaps_equal(g, o, upto=MiB + 4096)
        for bad in (lambda: g.launch_iput(0, 1, 0, 0, 0, 1, 10, 4), lambda: g.launch_iput(0, 1, 0, 0, 1, 1, 10, 3),
                    lambda: g.launch_iput(0, 1, 2, 0, 1, 1, 10, 4), lambda: g.launch_iget(0, 1, 0, 0, 1 << 40, 1, 10, 4),
                    lambda: g.launch_iput(0, 0, 0, 64, 8, 1, 100, 4)):
            with pytest.raises(S.ShmError):
                bad()


@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4])
def test_device_initiated_get_is_readable_inside_the_kernel(mode):
    """The kernel copies the destination to a consume buffer BEFORE the get (old bytes enter the
    caches) and after it; the second copy must show the new bytes although a copy engine, not a
    compute unit, may have written them."""
    g, o = make_pair(3, 24 * MiB)
    with g:
        fill_random(g, o, 64, upto=20 * MiB)
        g.proxy_start()
        cases = [(100003, 1, 17, 5), (MiB + 256, 4, 0, 0), (4096, 1, 3, 3), (3 * MiB + 1000, 16, 256, 512), (0, 2, 0, 0), (700, 8, 1, 2),
                 (2 * MiB, 2, 0, 0)]
        for i, (n, n_wg, sa, da) in enumerate(cases):
            me, pe = i % 3, (i + 1) % 3
            src, dst, cons = 1024 + sa, 6 * MiB + da, 12 * MiB + da
            g.launch_rma_device_initiated(me, pe, dst, src, n, n_wg, True, mode, cutover=65536, cover=128 * 1024, consume_off=cons,
                                          reps=1, wg_size=(64, 256, 1024)[i % 3])
            g.quiet(me)
            o.getmem(me, dst, src, n, pe)
            o.putmem(me, cons, dst, n, me)
            assert_heaps_equal(g, o, upto=20 * MiB, what=f"mode {mode} case {i}")
            # change the remote source and get again: the destination lines are now cached with the first result
            fresh = np.random.default_rng(1000 + i).integers(0, 256, max(n, 1), dtype=np.uint8)[:n]
            if n:
                g.write(pe, src, fresh), o.write(pe, src, fresh)
            g.launch_rma_device_initiated(me, pe, dst, src, n, n_wg, True, mode, cutover=65536, cover=128 * 1024, consume_off=cons,
                                          reps=2)
            g.quiet(me)
            o.getmem(me, dst, src, n, pe)
            o.putmem(me, cons, dst, n, me)
            assert_heaps_equal(g, o, upto=20 * MiB, what=f"mode {mode} case {i} again")
        g.proxy_stop()


def test_covered_put_matches_oracle_and_uses_the_engine():
    g, o = make_pair(2, 24 * MiB)
    with g:
        fill_random(g, o, 65, upto=20 * MiB)
        g.proxy_start()
        for i, (n, n_wg, cover) in enumerate([(4 * MiB + 100, 1, 256 * 1024), (4 * MiB, 4, 1000), (3000, 2, 65536), (MiB, 1, 0),
                                              (MiB, 8, MiB)]):
            before = g.proxy_stats()[1]
            g.launch_rma_device_initiated(0, 1, 8 * MiB + 16, 4096, n, n_wg, False, 4, cover=cover, reps=1)
            g.quiet(0)
            o.wg_put(0, 8 * MiB + 16, 4096, n, 1, n_wg)
            assert_heaps_equal(g, o, upto=20 * MiB, what=f"case {i}")
            copies = g.proxy_stats()[1] - before
            share = -(-n // n_wg)
            assert (copies > 0) == (share > ((cover + 255) & ~255)), (i, copies)
        g.proxy_stop()
        with pytest.raises(S.ShmError):                             # mode 4 without the proxy
            g.launch_rma_device_initiated(0, 1, 8 * MiB, 4096, MiB, 1, False, 4, cover=4096)
        with pytest.raises(S.ShmError):                             # consume needs a get
            g.launch_rma_device_initiated(0, 1, 8 * MiB, 4096, MiB, 1, False, 0, consume_off=12 * MiB)


def test_large_offloaded_transfers_are_split_over_engines():
    g, o = make_pair(2, 64 * MiB)
    with g:
        fill_random(g, o, 66, upto=60 * MiB)
        g.proxy_start()
        n = 20 * MiB + 1000                                          # five pieces of at least 4 MiB
        before = g.proxy_stats()[1]
        g.launch_rma_device_initiated(0, 1, 30 * MiB + 16, 4096 + 3, n, 1, False, 1)
        g.quiet(0)
        o.putmem(0, 30 * MiB + 16, 4096 + 3, n, 1)
        assert_heaps_equal(g, o, upto=60 * MiB, what="put")
        mid = g.proxy_stats()[1]
        assert mid - before >= 2
        g.launch_rma_device_initiated(1, 0, 30 * MiB, 256, n, 2, True, 3, consume_off=5 * MiB)   # two shares of ~10 MiB: two pieces each
        g.quiet(1)
        o.getmem(1, 30 * MiB, 256, n, 0)
        o.putmem(1, 5 * MiB, 30 * MiB, n, 1)
        assert_heaps_equal(g, o, upto=60 * MiB, what="get_nbi")
        assert g.proxy_stats()[1] - mid >= 4
        g.proxy_stop()


@pytest.mark.parametrize("n,n_waves,sa,da", [(100003, 7, 5, 9), (16, 4, 0, 0), (0, 3, 0, 0), (4096, 1, 1, 0), (100, 64, 0, 3),
                                            (3 * MiB + 17, 1024, 16, 32), (MiB, 256, 0, 0)])
def test_wave_forms_put_fence_flag_wait_fetch_get(n, n_waves, sa, da):
    g, o = make_pair(3, 16 * MiB)
    with g:
        fill_random(g, o, 67, upto=14 * MiB)
        src, dst, back, flag, out = 4096 + sa, 4 * MiB + da, 8 * MiB + da, 12 * MiB, 12 * MiB + 65536
        zeros = np.zeros(8 * n_waves, np.uint8)
        for rep in range(2):                                   # the second round finds the first round's bytes in the caches
            for p in range(3):
                g.write(p, flag, zeros), o.write(p, flag, zeros)
                g.write(p, out, zeros), o.write(p, out, zeros)
            if rep and n:
                fresh = np.random.default_rng(rep).integers(0, 256, n, dtype=np.uint8)
                g.write(2, src, fresh), o.write(2, src, fresh)
            g.launch_wave_exchange(2, 1, dst, src, back, n, n_waves, flag, out)
            g.quiet(2)
            o.wave_exchange(2, 1, dst, src, back, n, n_waves, flag, out)
            assert_heaps_equal(g, o, upto=14 * MiB, what=f"round {rep}")


def test_tuned_in_kernel_cutover_follows_the_work_items():
    """Mode 2 with SHM_CUTOVER_TUNED: a share below the threshold for the group's size moves by
    loads/stores (no engine copy), at or above it through the engine."""
    g, o = make_pair(2, 24 * MiB)
    with g:
        fill_random(g, o, 68, upto=20 * MiB)
        g.proxy_start()
        for wg_size, n, engine in [(64, MiB - 256, False), (64, MiB, True), (256, MiB, False), (256, 2 * MiB, True),
                                   (1024, 2 * MiB - 256, False), (1024, 2 * MiB + 100, True)]:
            before = g.proxy_stats()[1]
            g.launch_rma_device_initiated(0, 1, 8 * MiB + 16, 4096, n, 1, False, 2, cutover=S.SHM_CUTOVER_TUNED, wg_size=wg_size)
            g.quiet(0)
            o.putmem(0, 8 * MiB + 16, 4096, n, 1)
            assert_heaps_equal(g, o, upto=20 * MiB, what=f"{wg_size} work-items, {n} bytes")
            assert (g.proxy_stats()[1] > before) == engine, (wg_size, n)
        g.proxy_stop()


@pytest.mark.parametrize("elem", [1, 2, 4, 8])
@pytest.mark.parametrize("is_get", [False, True])
def test_scalar_p_and_g(elem, is_get):
    g, o = make_pair(3, 4 * MiB)
    with g:
        fill_random(g, o, 69 + elem, upto=3 * MiB)
        for nelems, n_wg, sa, da in [(1, 1, 0, 0), (1000, 1, 3, 5), (100003, 7, 1, 2), (0, 4, 0, 0), (65536, 64, 0, 0)]:
            src, dst = 4096 + sa * elem, 2 * MiB + da * elem
            g.launch_scalar_pg(0, 2, dst, src, nelems, elem, is_get, n_wg)
            g.quiet(0)
            (o.getmem if is_get else o.putmem)(0, dst, src, nelems * elem, 2)
            assert_heaps_equal(g, o, upto=3 * MiB, what=f"{nelems} elements of {elem} bytes")
        with pytest.raises(S.ShmError):
            g.launch_scalar_pg(0, 2, 2 * MiB + 1, 4096, 10, 8, is_get, 1)      # misaligned
        with pytest.raises(S.ShmError):
            g.launch_scalar_pg(0, 2, 2 * MiB, 4096, 10, 3, is_get, 1)          # element size
