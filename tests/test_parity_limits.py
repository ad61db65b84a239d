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


def _pattern_words(first_word, count):
    """Word i of the large-message pattern (64-bit, little endian): i * 0x9E3779B97F4A7C15 mod 2^64."""
    with np.errstate(over="ignore"):
        return (np.arange(first_word, first_word + count, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15))


@pytest.mark.timeout(600)
def test_messages_beyond_4_gib_on_every_path():
    """One message of a little over 2^32 bytes: byte offsets and lengths no longer fit 32 bits anywhere.
    The oracle's statement of a put (destination bytes = source bytes) is checked in full on the device
    and, against the pattern's closed form, on windows at the start, across the 2^32 boundary and at
    the ragged end; bytes around the destination must stay untouched."""
    import torch
    GiB = 1 << 30
    heap = 10 * GiB
    g = S.Shm.on_torch(2, heap)
    with g:
        n = 4 * GiB + MiB + 48 + 5
        src, dst = 4096, 5 * GiB
        words = n // 8
        view0 = g.heap_tensor[src:src + words * 8].view(torch.int64)
        step = 1 << 27
        for a in range(0, words, step):               # the pattern, generated on the device in slabs
            b = min(words, a + step)
            view0[a:b] = torch.arange(a, b, dtype=torch.int64, device="cuda") * (-7046029254386353131)    # 0x9E3779B97F4A7C15 as int64
        g.write(0, src + words * 8, np.arange(n - words * 8, dtype=np.uint8))
        torch.cuda.synchronize()
        canary = np.arange(64, dtype=np.uint8) ^ 0x5A
        source = g.heap_tensor[src:src + n]

        def check(doff, what):
            g.barrier_all()
            landed = g.heap_tensor[heap + doff:heap + doff + n]
            assert torch.equal(landed, source), f"{what}: destination differs from source somewhere"
            for lo, ln in [(0, MiB), (4 * GiB - 512 * 1024, MiB), (n - MiB - 5, MiB + 5)]:
                lo8 = lo // 8 * 8
                want = _pattern_words(lo8 // 8, (ln + 16) // 8 + 1).view(np.uint8)[lo - lo8:lo - lo8 + ln].copy()
                tail_from = words * 8
                if lo + ln > tail_from:                   # the last n mod 8 bytes are 0, 1, 2, ...
                    k = lo + ln - tail_from
                    want[ln - k:] = np.arange(k, dtype=np.uint8)
                assert np.array_equal(g.read(1, doff + lo, ln), want), f"{what}: window at {lo}"
            assert np.array_equal(g.read(1, doff - 64, 64), canary) and np.array_equal(g.read(1, doff + n, 64), canary), f"{what}: canary"

        def prepare(doff):
            g.heap_tensor[heap + doff - 64:heap + doff + n + 64].zero_()
            torch.cuda.synchronize()
            g.write(1, doff - 64, canary), g.write(1, doff + n, canary)

        cases = [("loads/stores, 1024 groups, aligned (tiles)", dst, lambda d: g.launch_wg_put(0, 1, d, src, n, 1024, S.SHM_PATH_LDST)),
                 ("loads/stores, 64 groups, destination + 3", dst + 3, lambda d: g.launch_wg_put(0, 1, d, src, n, 64, S.SHM_PATH_LDST)),
                 ("get, 256 groups", dst + 16, lambda d: g.launch_wg_get(1, 0, d, src, n, 256, S.SHM_PATH_LDST)),
                 ("copy engines", dst, lambda d: g.launch_wg_put(0, 1, d, src, n, 1, S.SHM_PATH_SDMA)),
                 ("runtime copy", dst + 1, lambda d: g.launch_wg_put(0, 1, d, src, n, 1, S.SHM_PATH_MEMCPY))]
        for what, doff, launch in cases:
            prepare(doff)
            launch(doff)
            check(doff, what)


@pytest.mark.timeout(600)
def test_fcollect_whose_destination_exceeds_4_gib():
    """8 PEs x 640 MiB + 16: every PE's destination is 5 GiB, so block offsets pass 2^32.  Every block on
    every PE is compared with its source on the device, windows (one across the 2^32 boundary) with
    the pattern's closed form, and the bytes behind the destination stay untouched."""
    import torch
    GiB = 1 << 30
    npes, heap = 8, 6 * GiB
    g = S.Shm.on_torch(npes, heap)
    with g:
        n = 640 * MiB + 16
        src, dst = 4096, 700 * MiB
        words = n // 8
        for p in range(npes):                          # PE p's pattern starts at word p * 2^40
            view = g.heap_tensor[p * heap + src:p * heap + src + n].view(torch.int64)
            view[:] = (torch.arange(words, dtype=torch.int64, device="cuda") + (p << 40)) * (-7046029254386353131)
        canary = np.arange(64, dtype=np.uint8) ^ 0xA5
        for q in range(npes):
            g.heap_tensor[q * heap + dst:q * heap + dst + npes * n].zero_()
            g.write(q, dst + npes * n, canary)
        torch.cuda.synchronize()
        g.launch_fcollect(dst, src, n, 32, S.SHM_PATH_LDST)
        g.barrier_all()
        for q in range(npes):
            for p in range(npes):
                got = g.heap_tensor[q * heap + dst + p * n:q * heap + dst + (p + 1) * n]
                assert torch.equal(got, g.heap_tensor[p * heap + src:p * heap + src + n]), f"block {p} on PE {q}"
            assert np.array_equal(g.read(q, dst + npes * n, 64), canary), f"canary on PE {q}"
        q = 5
        boundary = (1 << 32) - dst                     # offset within the destination where the heap offset reaches 2^32
        for lo in (0, boundary - 4096, npes * n - 8192):
            p, within = divmod(lo, n)
            ln = min(8192, n - within) // 8 * 8
            within8 = within // 8 * 8
            want = _pattern_words((p << 40) + within8 // 8, ln // 8 + 2).view(np.uint8)[within - within8:within - within8 + ln]
            assert np.array_equal(g.read(q, dst + lo, ln), want), f"window at {lo}"
