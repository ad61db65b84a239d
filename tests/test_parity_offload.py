"""GPU parity: device-initiated copy-engine transfers through the reverse-offload ring."""
import numpy as np
import pytest
import torch

from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair

pytestmark = pytest.mark.gpu

MiB = 1 << 20
MASK = (1 << 64) - 1


def _ticks():
    t = torch.zeros(2, dtype=torch.int64, device="cuda")
    t[0] = -1
    torch.cuda.synchronize()
    return t


def _elapsed_us(g, t):
    t0, t1 = (int(v) & MASK for v in t.tolist())
    return (t1 - t0) / g.wall_clock_khz() * 1e3


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_device_initiated_put_matches_oracle(mode):
    g, o = make_pair(3, 16 * MiB)
    with g:
        fill_random(g, o, 31, upto=12 * MiB)
        g.proxy_start()
        cases = [(100003, 1, 17, 5), (MiB + 256, 4, 0, 0), (4096, 1, 3, 3), (3 * MiB + 1000, 16, 256, 512), (0, 2, 0, 0), (700, 8, 1, 2)]
        copies_before = g.proxy_stats()[1]
        for i, (n, n_wg, sa, da) in enumerate(cases):
            me, pe = i % 3, (i + 1) % 3
            src, dst = 1024 + sa, 6 * MiB + da
            t = _ticks()
            g.launch_put_device_initiated(me, pe, dst, src, n, n_wg, mode, 65536, 2, t, wg_size=(64, 256, 1024)[i % 3])
            g.quiet(me)
            o.wg_put(me, dst, src, n, pe, n_wg)
            assert_heaps_equal(g, o, upto=12 * MiB, what=f"mode {mode} case {i}")
            assert 0 < _elapsed_us(g, t) < 1e6
        requests, copies = g.proxy_stats()
        if mode == 0:
            assert copies == copies_before
        if mode in (1, 3):
            assert copies - copies_before >= 2 * (1 + 4 + 1 + 16 + 1)      # every non-empty share, twice
        g.proxy_stop()


@pytest.mark.parametrize("wg_size", [1, 16, 100, 128])
def test_device_initiated_put_by_partial_waves(wg_size):
    """The paper's work-items axis below one wave: 1, 16, ... work-items per work-group, loads/stores."""
    g, o = make_pair(2, 4 * MiB)
    with g:
        fill_random(g, o, 32, upto=3 * MiB)
        for i, (n, n_wg, sa, da) in enumerate([(10007, 1, 3, 5), (65536 + 40, 2, 0, 0), (0, 1, 0, 0), (17, 3, 1, 2)]):
            t = _ticks()
            g.launch_put_device_initiated(0, 1, 2 * MiB + da, 256 + sa, n, n_wg, 0, 0, 2, t, wg_size=wg_size)
            g.quiet(0)
            o.wg_put(0, 2 * MiB + da, 256 + sa, n, 1, n_wg)
            assert_heaps_equal(g, o, upto=3 * MiB, what=f"case {i}")
        with pytest.raises(S.ShmError):
            g.launch_put_device_initiated(0, 1, 2 * MiB, 256, 100, 1, 1, 0, 1, _ticks(), wg_size=wg_size)   # engine modes need whole waves... and the proxy


def test_ring_round_trips_rate_and_wraparound():
    g, o = make_pair(2, MiB)
    with g:
        g.proxy_start()
        t = _ticks()
        g.launch_offload_nop(0, 1, 200, True, t)                 # 200 round trips by one wave
        g.quiet(0)
        rtt = _elapsed_us(g, t) / 200
        assert 0.5 < rtt < 500, rtt
        req0 = g.proxy_stats()[0]
        assert req0 == 200
        t = _ticks()
        g.launch_offload_nop(1, 64, 300, False, t)               # 19264 requests: the 4096-slot ring wraps four times
        g.quiet(1)
        assert g.proxy_stats()[0] - req0 == 64 * 301
        rate = 64 * 301 / _elapsed_us(g, t)
        assert rate > 0.05, f"{rate} M requests/s"
        g.proxy_stop()
        # stop / start: the ring restarts from zero
        g.proxy_start()
        t = _ticks()
        g.launch_offload_nop(0, 4, 10, True, t)
        g.quiet(0)
        assert g.proxy_stats()[0] == 40
        g.proxy_stop()


def test_offload_needs_the_proxy():
    g, o = make_pair(2, MiB)
    with g:
        t = _ticks()
        with pytest.raises(S.ShmError) as e:
            g.launch_put_device_initiated(0, 1, 65536, 0, 4096, 1, 1, 0, 1, t)
        assert e.value.code == S.SHM_EINVAL
        with pytest.raises(S.ShmError):
            g.launch_offload_nop(0, 1, 1, True, t)
        g.launch_put_device_initiated(0, 1, 65536, 0, 4096, 1, 0, 0, 1, t)     # loads/stores need no proxy
        g.quiet(0)


def test_device_initiated_put_random_sizes_and_alignments():
    """Many small and medium in-kernel puts (the write-through store path up to 64 bytes per thread,
    the streaming path beyond) at random sizes, alignments, group sizes and group counts."""
    g, o = make_pair(2, 4 * MiB)
    rng = np.random.default_rng(33)
    with g:
        fill_random(g, o, 33, upto=3 * MiB)
        t = _ticks()
        for i in range(150):
            wg_size = int(rng.choice([1, 7, 64, 128, 192, 256, 512, 1024]))
            n_wg = int(rng.choice([1, 2, 3, 8]))
            n = int(rng.integers(0, 70000)) if i % 3 else int(rng.integers(0, 300))
            sa, da = int(rng.integers(0, 48)), int(rng.integers(0, 48))
            me = i & 1
            g.launch_put_device_initiated(me, 1 - me, 2 * MiB + da, 1024 + sa, n, n_wg, 0, 0, 1, t, wg_size=wg_size)
            o.wg_put(me, 2 * MiB + da, 1024 + sa, n, 1 - me, n_wg)
            if i % 10 == 9:
                g.barrier_all()
                assert_heaps_equal(g, o, upto=3 * MiB, what=f"after case {i} (wg_size {wg_size}, n_wg {n_wg}, n {n}, src+{sa}, dst+{da})")
        g.barrier_all()
        assert_heaps_equal(g, o, upto=3 * MiB, what="end")


@pytest.mark.parametrize("is_get", [False, True])
def test_nbi_transfers_of_a_kernel_complete_at_the_hosts_quiet(is_get):
    """put_nbi / get_nbi issued by kernels that never wait for them (no quiet inside the kernel):
    OpenSHMEM completes them at the PE's quiet, which here is the host's shm_quiet for that PE."""
    g, o = make_pair(3, 16 * MiB)
    with g:
        fill_random(g, o, 34, upto=12 * MiB)
        g.proxy_start()
        cases = [(5 * MiB + 1000, 16, 256, 512), (100003, 1, 17, 5), (0, 2, 0, 0), (MiB + 256, 8, 0, 0), (4096, 3, 3, 3)]
        for i, (n, n_wg, sa, da) in enumerate(cases):
            me, pe = i % 3, (i + 2) % 3
            src, dst = 1024 + sa, 6 * MiB + da
            g.launch_rma_device_initiated(me, pe, dst, src, n, n_wg, is_get, 5, wg_size=(256, 64, 1024)[i % 3])
            g.quiet(me)
            (o.getmem if is_get else o.putmem)(me, dst, src, n, pe)
            assert_heaps_equal(g, o, upto=12 * MiB, what=f"get={is_get} case {i}")
        # several PEs' transfers left in flight together, completed by one barrier_all
        for me in range(3):
            g.launch_rma_device_initiated(me, (me + 1) % 3, 6 * MiB + me * MiB, 2048 + me * 512, MiB - 7, 4, is_get, 5)
            (o.getmem if is_get else o.putmem)(me, 6 * MiB + me * MiB, 2048 + me * 512, MiB - 7, (me + 1) % 3)
        g.barrier_all()
        assert_heaps_equal(g, o, upto=12 * MiB, what=f"get={is_get} after barrier_all")
        # stopping the proxy finishes what kernels left in the ring
        g.launch_rma_device_initiated(0, 1, 9 * MiB, 4096, 2 * MiB, 8, is_get, 5)
        o_call = o.getmem if is_get else o.putmem
        o_call(0, 9 * MiB, 4096, 2 * MiB, 1)
        g.proxy_stop()
        assert_heaps_equal(g, o, upto=12 * MiB, what=f"get={is_get} after proxy_stop")
        with pytest.raises(S.ShmError):
            g.launch_rma_device_initiated(0, 1, 9 * MiB, 4096, 4096, 1, True, 5, consume_off=11 * MiB)
