"""GPU parity of an APPLICATION kernel: a separately built library that includes only the device
header, gets the device view from shm_device_context() and calls the OpenSHMEM operations from its
own kernel (all-to-all by work-group puts, device-side barrier, work-group get, fetch-add tally).
Expected state: the oracle's composition of the same operations."""
import ctypes
import os

import numpy as np
import pytest

from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair

pytestmark = pytest.mark.gpu

MiB = 1 << 20
EXAMPLE = os.path.join(os.path.dirname(os.path.abspath(S.__file__)), "libshm355_user_example.so")


def _example():
    """Load the example application.  Called once a context exists, so that the process already holds
    the HIP runtime PyTorch brought and the example binds to that one."""
    if not os.path.exists(EXAMPLE):
        raise ImportError(f"{EXAMPLE} has not been built; run `python -m paper_2409_20476_amd.build`")
    lib = ctypes.CDLL(EXAMPLE)
    lib.shmu_alltoall.restype = ctypes.c_int
    lib.shmu_alltoall.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_size_t,
                                  ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64]
    lib.shmu_device_context_bytes.restype = ctypes.c_size_t
    return lib


@pytest.mark.parametrize("npes,n", [(2, 1000), (8, 100003), (5, 0), (16, 4096 + 7), (3, 262144)])
def test_application_kernel_alltoall_barrier_get_tally(npes, n):
    g, o = make_pair(npes, 16 * MiB)
    with g:
        lib = _example()            # after the context: PyTorch's HIP runtime is the one already in the process
        fill_random(g, o, 51, upto=12 * MiB)
        view = g.device_context()
        assert len(view) == lib.shmu_device_context_bytes()
        src, dst, back, tally, seen = 1024 + 3, 5 * MiB + 5, 10 * MiB + 1, 11 * MiB, 11 * MiB + 64
        init = int(o.read(0, tally, 8, np.int64)[0])
        for rep in range(2):                                 # twice: the barrier's counters carry over
            rc = lib.shmu_alltoall(view, len(view), g.stream(0), dst, src, n, back, tally, seen)
            assert rc == 0
            g.barrier_all()
            for p in range(npes):
                for j in range(npes):
                    t = (p + j) % npes
                    o.putmem(p, dst + p * n, src + t * n, n, t)
            o.barrier_all()
            for p in range(npes):
                o.getmem(p, back, dst, n, (p + 1) % npes)
            for p in range(npes):
                o.atomic_fetch_add(p, tally, p + 1, 0)
            # what each PE fetched depends on the order the hardware served them: any order is right,
            # as long as the values chain from the initial tally to the final one
            got = {p: int(g.read(p, seen, 8, np.int64)[0]) for p in range(npes)}
            at = init
            for p in sorted(got, key=got.get):
                assert got[p] == at, f"fetched values do not chain: {got}"
                at += p + 1
            init = at
            for p in range(npes):
                o.write(p, seen, np.array([got[p]], dtype=np.int64))
            assert_heaps_equal(g, o, upto=12 * MiB, what=f"npes {npes}, n {n}, repetition {rep}")


def test_device_view_is_refused_at_another_size_and_streams_are_the_contexts():
    g, o = make_pair(2, MiB)
    with g:
        n = g.lib.shm_device_context_bytes()
        buf = ctypes.create_string_buffer(n + 8)
        assert g.lib.shm_device_context(g.ctx, buf, n + 8) == S.SHM_EINVAL
        assert g.lib.shm_device_context(g.ctx, None, n) == S.SHM_EINVAL
        assert g.stream(0) == g.streams[0].cuda_stream and g.stream(1) == g.streams[1].cuda_stream
        assert g.stream(2) == 0 and g.stream(-1) == 0
        assert _example().shmu_alltoall(buf, n + 8, g.stream(0), 0, 4096, 16, 8192, 16384, 16392) == -1


@pytest.mark.parametrize("mode", [S.SHM_TEAM_SYNC_FULL, S.SHM_TEAM_SYNC_TRACKED])
def test_application_kernel_between_team_launches_is_ordered(mode):
    """A team put produces the application kernel's input, the kernel runs on PE 2's stream, a team
    broadcast consumes its output -- no host barrier in between.  Under the tracked team sync the
    caller announces its own use of the stream with shm_stream_used."""
    npes, n = 4, 300000
    g, o = make_pair(npes, 16 * MiB)
    with g:
        lib = _example()
        g.set_team_sync(mode)
        fill_random(g, o, 52, upto=14 * MiB)
        view = g.device_context()
        pre, src, dst, back, tally, seen, out = 64, 2 * MiB, 5 * MiB, 9 * MiB, 11 * MiB, 11 * MiB + 64, 12 * MiB
        for rep in range(3):
            g.launch_wg_put_all(1, src, pre + rep, npes * n, 16)                   # input of the kernel: every PE's source blocks
            snap = [h.copy() for h in o.heap]
            for p in range(npes):
                o.heap[(p + 1) % npes][src:src + npes * n] = snap[p][pre + rep:pre + rep + npes * n]
            g.stream_used(2)
            assert lib.shmu_alltoall(view, len(view), g.stream(2), dst, src, n, back, tally, seen) == 0
            for p in range(npes):
                for j in range(npes):
                    t = (p + j) % npes
                    o.putmem(p, dst + p * n, src + t * n, n, t)
            for p in range(npes):
                o.getmem(p, back, dst, n, (p + 1) % npes)
            g.launch_broadcast(out, dst + n, 2 * n, 3, 8)                          # consumes slots 1 and 2 of PE 3's destination
            o.broadcast(out, dst + n, 2 * n, 3)
            g.barrier_all()
            for p in range(npes):                                                  # tally and fetched values: checked in the test above
                for off in (tally, seen):
                    o.write(p, off, g.read(p, off, 8))
            assert_heaps_equal(g, o, upto=14 * MiB, what=f"mode {mode}, repetition {rep}")


@pytest.mark.parametrize("npes,n,nelems,root", [(2, 4096, 1000, 1), (8, 100000, 25000, 5), (5, 16, 4, 0), (16, 20000, 17, 15), (1, 64, 16, 0)])
def test_application_kernel_calls_the_collectives(npes, n, nelems, root):
    """fcollect, two reductions and a broadcast as single device calls from one kernel of one group per PE."""
    g, o = make_pair(npes, 16 * MiB)
    with g:
        lib = _example()
        lib.shmu_collectives.restype = ctypes.c_int
        lib.shmu_collectives.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_size_t,
                                         ctypes.c_uint64, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_int]
        fill_random(g, o, 53, upto=12 * MiB)
        view = g.device_context()
        src, gather, sums, mins, bcast = 4096, 1 * MiB, 8 * MiB, 9 * MiB, 10 * MiB
        for rep in range(2):
            assert lib.shmu_collectives(view, len(view), g.stream(0), gather, src + 16 * rep, n, sums, mins, nelems, bcast, root) == 0
            g.barrier_all()
            o.fcollect(gather, src + 16 * rep, n)
            o.reduce(sums, src + 16 * rep, nelems, np.int32, "sum")
            o.reduce(mins, src + 16 * rep, 2 * nelems, np.int16, "min")
            o.broadcast(bcast, src + 16 * rep, n, root)
            assert_heaps_equal(g, o, upto=12 * MiB, what=f"repetition {rep}")


@pytest.mark.parametrize("threads,groups", [(192, 40), (64, 16), (128, 7), (256, 33), (320, 9), (512, 12), (768, 5), (1024, 6), (8, 3)])
def test_application_kernel_moves_a_long_message_on_tiles_with_its_own_group_size(threads, groups):
    """shmx_putmem_tiles / shmx_getmem_tiles from groups of 8 to 1024 work-items, among them sizes that are
    not a power of two (they take the general dealing): ragged last tile, byte tail, groups with one
    tile, with several and with none."""
    g, o = make_pair(2, 16 * MiB)
    with g:
        lib = _example()
        lib.shmu_tiles.restype = ctypes.c_int
        lib.shmu_tiles.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                   ctypes.c_size_t, ctypes.c_uint64, ctypes.c_int, ctypes.c_int]
        fill_random(g, o, 54, upto=14 * MiB)
        view = g.device_context()
        for rep, n in enumerate([3 * MiB + 65536 + 4096 + 16 * 5 + 11, 65536 * groups, 65536 * min(4 * groups, 50) + 48, 13, 0]):
            if threads < 64 and n > MiB:
                n = 200000 + rep            # a handful of lanes: keep the run short
            me, pe = rep % 2, (rep + 1) % 2
            src, dst, back = 4096 + 16 * rep, 5 * MiB + 4096 * rep, 9 * MiB + 16 * rep
            assert lib.shmu_tiles(view, len(view), g.stream(me), me, pe, dst, src, n, back, groups, threads) == 0
            g.quiet(me)
            o.putmem(me, dst, src, n, pe)
            o.getmem(me, back, dst, n, pe)
            assert_heaps_equal(g, o, upto=14 * MiB, what=f"{groups} groups of {threads}, n {n}")
