"""GPU parity: work-group put/get, team forms, both transfer paths, host RMA -- bit-exact against the oracle."""
import numpy as np
import pytest

from oracle.shmem_oracle import SIGNAL_ADD
from paper_2409_20476_amd import shm as S
from parity_util import assert_heaps_equal, fill_random, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def test_alignment_sweep_single_group():
    """Every (src mod 16, dst mod 16) pair, every length 0..96, one work-group; canaries are the rest of the heap."""
    g, o = make_pair(2, MiB)
    with g:
        fill_random(g, o, 1)
        for s in range(16):
            for d in range(16):
                for n in range(97):
                    src = 1024 + s + 16 * (n % 5)
                    dst = 65536 + (d * 97 + n) * 256 + 64 + d        # own 256-byte slot per (d, n); dst mod 16 == d
                    g.launch_wg_put(0, 1, dst, src, n, 1)
                    o.wg_put(0, dst, src, n, 1, 1)
            g.barrier_all()
            assert_heaps_equal(g, o, what=f"src mod 16 = {s}")


@pytest.mark.parametrize("n_wg", [1, 3, 4, 64])
def test_put_get_sizes_tiles_and_ragged_tails(n_wg):
    g, o = make_pair(3, 8 * MiB)
    with g:
        fill_random(g, o, 2, upto=6 * MiB)
        cases = [(0, 0, 0), (4096 + 3, 0, 0), (65536 + 17, 5, 5), (MiB - 5, 3, 11), (MiB + 1, 16, 0), (300000, 1, 2),
                 (12345, 15, 15), (256 * 16 * 8 * 3 + 16, 0, 0), (15, 9, 2), (16, 0, 0), (4080, 8, 8)]
        for i, (n, sa, da) in enumerate(cases):
            me, pe = i % 3, (i + 1 + i // 3) % 3
            src, dst = 1024 + sa, 2 * MiB + 4096 + da
            g.launch_wg_put(me, pe, dst, src, n, n_wg)
            o.wg_put(me, dst, src, n, pe, n_wg)
            g.barrier_all()
            g.launch_wg_get(pe, me, 4 * MiB + 8192 + sa, 2 * MiB + 4096 + da, n, n_wg)
            o.wg_get(pe, 4 * MiB + 8192 + sa, 2 * MiB + 4096 + da, n, me, n_wg)
            g.barrier_all()
            assert_heaps_equal(g, o, upto=6 * MiB, what=f"case {i} n={n}")


def test_self_target_and_overlap_rejected():
    g, o = make_pair(2, MiB)
    with g:
        fill_random(g, o, 3)
        g.launch_wg_put(0, 0, 8192, 100, 5000, 2)
        o.wg_put(0, 8192, 100, 5000, 0, 2)
        g.barrier_all()
        assert_heaps_equal(g, o)
        with pytest.raises(S.ShmError) as e:
            g.launch_wg_put(0, 0, 200, 100, 5000, 2)
        assert e.value.code == S.SHM_EINVAL


@pytest.mark.parametrize("path", [S.SHM_PATH_LDST, S.SHM_PATH_SDMA, S.SHM_PATH_MEMCPY])
def test_team_put_get_all_paths(path):
    g, o = make_pair(8, 4 * MiB)
    with g:
        fill_random(g, o, 4)
        n = MiB + 48
        for shift in (1, 3, 0):
            dst = 2 * MiB - 64 if shift else MiB + 4096 + MiB // 2
            src = 16 if shift else 0
            if shift == 0:
                n = MiB // 4
            g.launch_wg_put_all(shift, dst, src, n, 16, path)
            for p in range(8):
                o.wg_put(p, dst, src, n, (p + shift) % 8, 16)
            g.barrier_all()
            assert_heaps_equal(g, o, upto=4 * MiB - 65536, what=f"put_all shift {shift}")
        g.launch_wg_get_all(5, 0, 2 * MiB, 70000, 7, path)
        before = [h.copy() for h in o.heap]
        for p in range(8):
            o.heap[p][0:70000] = before[(p + 5) % 8][2 * MiB:2 * MiB + 70000]
        g.barrier_all()
        assert_heaps_equal(g, o, upto=4 * MiB - 65536, what="get_all")


def test_host_rma_sdma_single_and_auto_policy():
    g, o = make_pair(4, 2 * MiB)
    with g:
        fill_random(g, o, 5)
        g.putmem(1, MiB, 7, 30001, 3)
        o.putmem(1, MiB, 7, 30001, 3)
        g.quiet(1)
        g.getmem(2, MiB + 65536, 3, 999, 0)
        o.getmem(2, MiB + 65536, 3, 999, 0)
        g.quiet(2)
        g.launch_wg_put(0, 2, MiB + 200000, 11, 12345, 4, S.SHM_PATH_SDMA)
        o.wg_put(0, MiB + 200000, 11, 12345, 2, 4)
        g.launch_wg_get(0, 2, MiB + 300000, 64, 4096, 4, S.SHM_PATH_SDMA)
        o.wg_get(0, MiB + 300000, 64, 4096, 2, 4)
        g.launch_wg_put(0, 1, MiB + 500000, 1, 7777, 4, S.SHM_PATH_MEMCPY)
        o.wg_put(0, MiB + 500000, 1, 7777, 1, 4)
        # an engine transfer followed, without quiet, by a kernel on the same PE that reads its result
        g.launch_wg_put(0, 3, MiB + 600000, 5, 50001, 2, S.SHM_PATH_SDMA)
        o.wg_put(0, MiB + 600000, 5, 50001, 3, 2)
        g.launch_wg_get(0, 3, MiB + 700000, MiB + 600000, 50001, 3, S.SHM_PATH_LDST)
        o.wg_get(0, MiB + 700000, MiB + 600000, 50001, 3, 3)
        g.quiet(0)
        # AUTO: below the cutover the kernel runs, at or above it the engine; bytes are the same either way
        g.set_cutover(4, 8192)
        assert g.get_cutover(4) == 8192 and g.get_cutover(3) == 8192 and g.get_cutover(64) == (1 << 64) - 1
        assert g.choose_path(8191, 4) == S.SHM_PATH_LDST and g.choose_path(8192, 4) == S.SHM_PATH_SDMA
        for n in (100, 8191, 8192, 50000):
            g.launch_wg_put(3, 1, MiB + 400000, 0, n, 4, S.SHM_PATH_AUTO)
            o.wg_put(3, MiB + 400000, 0, n, 1, 4)
        g.quiet(3)
        assert_heaps_equal(g, o)


def test_timed_put_moves_the_same_bytes_and_reports_device_time():
    import torch
    g, o = make_pair(2, 4 * MiB)
    with g:
        fill_random(g, o, 6)
        ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
        ticks[0] = -1
        g.launch_wg_put_timed(0, 1, 2 * MiB + 3, 17, 300001, 8, 5, ticks)
        g.quiet(0)
        o.wg_put(0, 2 * MiB + 3, 17, 300001, 1, 8)
        assert_heaps_equal(g, o)
        t0, t1 = (int(v) & ((1 << 64) - 1) for v in ticks.tolist())
        us = (t1 - t0) / g.wall_clock_khz() * 1e3
        assert 0 < us < 1e5, us


@pytest.mark.parametrize("n_wg", [65, 200, 1024])
def test_more_groups_than_vectors_and_the_minimum_share_of_put_then_quiet(n_wg):
    """Messages asked of 65, 200 and 1024 groups: plain puts and gets deal them to every group that can
    get a vector; the timed put, whose every group quiets after its share, deals only to as many groups
    as get 128 KiB each beyond 64 groups, and the others skip their quiet.  Sizes around the steps of
    that rule, shifted and aligned sources, and a put_signal by all groups."""
    import torch
    g, o = make_pair(2, 64 * MiB)
    with g:
        fill_random(g, o, 21, upto=48 * MiB)
        sig = 47 * MiB
        for i, (n, sa, da) in enumerate([(5, 0, 0), (300001, 3, 7), (8 * MiB - 16, 0, 0), (8 * MiB + 128 * 1024 * 3 + 48 + 5, 16, 32),
                                         (9 * MiB + 1, 5, 5), (17 * MiB + 4096, 32, 0)]):
            src, dst, back = 64 + sa, 20 * MiB + da, 40 * MiB - 7 * MiB * (i % 2) + sa
            g.launch_wg_put(0, 1, dst, src, n, n_wg)
            o.wg_put(0, dst, src, n, 1, n_wg)
            g.barrier_all()
            if n <= 7 * MiB:
                g.launch_wg_get(0, 1, back, dst, n, n_wg)
                o.wg_get(0, back, dst, n, 1, n_wg)
                g.barrier_all()
            assert_heaps_equal(g, o, upto=48 * MiB, what=f"n={n} by {n_wg} groups")
        ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
        ticks[0] = -1
        for m in (9 * MiB + 48 + 3, 8 * MiB + 128 * 1024 * 3 + 16 + 5, 300001):
            g.launch_wg_put_timed(1, 0, 20 * MiB + 16, 1 * MiB, m, n_wg, 3, ticks)
            g.quiet(1)
            o.wg_put(1, 20 * MiB + 16, 1 * MiB, m, 0, n_wg)
            assert_heaps_equal(g, o, upto=48 * MiB, what=f"timed put of {m} bytes by {n_wg} groups")
        z = np.zeros(8, np.uint8)
        for p in range(2):
            write_both(g, o, p, sig, z)
        g.launch_wg_put_signal(0, 1, 30 * MiB + 5, 2 * MiB + 1, 3 * MiB + 9, sig, 1, S.SHM_SIGNAL_ADD, min(n_wg, 1000))
        o.put_signal(0, 30 * MiB + 5, 2 * MiB + 1, 3 * MiB + 9, sig, 1, SIGNAL_ADD, 1)
        g.barrier_all()
        assert_heaps_equal(g, o, upto=48 * MiB, what=f"timed put and put_signal by {n_wg} groups")


def test_timed_put_of_long_messages_moves_the_same_bytes_on_both_long_message_paths():
    """9 MiB by 64 groups and 40 MiB by 48 groups stay on the virtual blocks (short message; fewer than 64
    groups); from 16 MiB and 64 groups on -- 65 MiB by 512 groups, 33 MiB by 64, 16 MiB and a bit by 100 -- the groups
    draw half-tile pieces by ticket, up to 504 repetitions, one ticket counter each; beyond, every group owns fixed tiles.  The
    launches follow one another at once: each finds the counters its predecessor used cleared."""
    import torch
    g, o = make_pair(2, 160 * MiB)
    with g:
        fill_random(g, o, 7, upto=144 * MiB)
        for n, n_wg, reps in [(9 * MiB + 16 * 3 + 5, 64, 3), (65 * MiB + 16 * 3 + 5, 512, 3), (40 * MiB + 16 * 7 + 1, 48, 3),
                              (33 * MiB + 65536 + 16 + 3, 64, 3),      # ragged last tile and a byte tail
                              (32 * MiB + 48, 1024, 1), (33 * MiB + 65536 + 16 + 3, 200, 513), (16 * MiB + 32768 + 16 + 7, 100, 2)]:
            ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
            ticks[0] = -1
            g.launch_wg_put_timed(0, 1, 70 * MiB + 16, 32, n, n_wg, reps, ticks)
            g.quiet(0)
            o.wg_put(0, 70 * MiB + 16, 32, n, 1, n_wg)
            assert_heaps_equal(g, o, upto=144 * MiB, what=f"n {n} by {n_wg} groups, {reps} repetitions")
            t = ticks.cpu().numpy()
            assert 0 < t[0] < t[1], "device clock: first start before last end"


@pytest.mark.parametrize("n_wg", [64, 100, 512, 515, 600])
def test_long_messages_by_64_groups_or_more_take_group_owned_tiles(n_wg):
    """32 MiB or more by 64 groups or more of one PE, 16-byte-aligned offsets: the launcher runs at most
    one group per four 64 KiB tiles and every group owns whole tiles.  Ragged last tile, byte tail, a
    destination 4 KiB, 1 MiB + 4 KiB ... off the source's alignment, put and get."""
    g, o = make_pair(2, 176 * MiB)
    with g:
        fill_random(g, o, 8, upto=160 * MiB)
        sizes = [70 * MiB, 70 * MiB + 48, 71 * MiB + 131072 + 16, 70 * MiB + 7]
        for rep, n in enumerate(sizes):
            me, pe = rep % 2, (rep + 1) % 2
            src, dst = 4096 + 16 * rep, 80 * MiB + (MiB + 4096) * rep + 32 * rep
            g.launch_wg_put(me, pe, dst, src, n, n_wg)
            o.wg_put(me, dst, src, n, pe, n_wg)
            g.quiet(me)
            g.launch_wg_get(pe, me, 64, dst, n, n_wg)           # read it back into the start of the caller's heap
            o.wg_get(pe, 64, dst, n, me, n_wg)
            g.quiet(pe)
            assert_heaps_equal(g, o, upto=160 * MiB, what=f"n_wg {n_wg} size {n}")


@pytest.mark.parametrize("n_wg", [8, 15, 16, 33, 100, 128, 160, 512, 600])
def test_long_messages_team_forms_on_all_long_message_paths(n_wg):
    """Team grids of 4 PEs, 33 MiB: below 64 groups in the grid (8, 15 per PE) the virtual blocks, from
    16 per PE group-owned tiles (each group more than four tiles), from 128 per PE half-tile pieces
    drawn by ticket by 128 groups per PE; put_all and get_all back to back (the second launch finds
    the counters as the first one did), ragged last tile and byte tail."""
    g, o = make_pair(4, 80 * MiB)
    with g:
        fill_random(g, o, 8, upto=76 * MiB)
        n = 33 * MiB + 65536 + 5
        g.launch_wg_put_all(3, 38 * MiB + 4096, 0, n, n_wg)
        for p in range(4):
            o.wg_put(p, 38 * MiB + 4096, 0, n, (p + 3) % 4, n_wg)
        g.barrier_all()
        g.launch_wg_get_all(1, 64, 38 * MiB + 4096, n, n_wg)
        before = [h.copy() for h in o.heap]
        for p in range(4):
            o.heap[p][64:64 + n] = before[(p + 1) % 4][38 * MiB + 4096:38 * MiB + 4096 + n]
        g.barrier_all()
        assert_heaps_equal(g, o, upto=76 * MiB, what="team forms")


def test_team_puts_by_ticket_random_sizes_and_places():
    """Ten seeded random team puts and gets of 32-36 MiB at random 16-byte-aligned offsets (and two that
    are not: those take the general dealing), random shifts and group counts from 128 up, 5 PEs, one after
    the other without anything in between but the barrier the comparison needs."""
    npes = 5
    g, o = make_pair(npes, 80 * MiB)
    rng = np.random.default_rng(20476)
    with g:
        fill_random(g, o, 10, upto=78 * MiB)
        for rep in range(10):
            n = int(rng.integers(32 * MiB, 36 * MiB))
            if rep % 3 == 0:
                n &= ~15
            align = 1 if rep in (4, 7) else 16
            a = int(rng.integers(0, (38 * MiB - n) // align)) * align
            b = 39 * MiB + int(rng.integers(0, (38 * MiB - n) // align)) * align
            src, dst = (a, b) if rep % 2 else (b, a)
            shift, n_wg = int(rng.integers(1, npes)), int(rng.integers(128, 1025))
            before = [h.copy() for h in o.heap]
            if rng.integers(2):
                g.launch_wg_put_all(shift, dst, src, n, n_wg)
                for p in range(npes):
                    o.heap[(p + shift) % npes][dst:dst + n] = before[p][src:src + n]
            else:
                g.launch_wg_get_all(shift, dst, src, n, n_wg)
                for p in range(npes):
                    o.heap[p][dst:dst + n] = before[(p + shift) % npes][src:src + n]
            g.barrier_all()
            assert_heaps_equal(g, o, upto=78 * MiB, what=f"launch {rep}: {n} bytes {src} -> {dst}, shift {shift}, {n_wg} groups")


@pytest.mark.parametrize("n_wg", [3, 64, 1024])
def test_messages_of_4_mib_and_more_are_dealt_from_a_destination_boundary(n_wg):
    """Below the long forms a message of 4 MiB or more is dealt from where the destination reaches a
    multiple of 1 KiB, the vectors before it moved by the last group: destinations and sources at odd
    bytes, 16 bytes and whole boundaries past one, equal and different modulo 16; one message just
    below 4 MiB (dealt from its first vector); team form and one PE's own launch."""
    npes = 3
    g, o = make_pair(npes, 24 * MiB)
    with g:
        fill_random(g, o, 11, upto=22 * MiB)
        cases = [(16, 0, 4 * MiB + 1024), (5, 5, 5 * MiB + 3), (1008, 1, 4 * MiB + 16), (8, 4, 6 * MiB - 7), (0, 9, 4 * MiB + 15),
                 (1023, 1023, 4 * MiB + 2048), (48, 0, 4 * MiB - 64), (1, 2, 9 * MiB + 1)]
        for rep, (da, sa, n) in enumerate(cases):
            src, dst = 1024 + sa, 11 * MiB + da
            if rep % 2 == 0:
                shift = 1 + rep % (npes - 1)
                g.launch_wg_put_all(shift, dst, src, n, n_wg, S.SHM_PATH_LDST)
                before = [h.copy() for h in o.heap]
                for p in range(npes):
                    o.heap[(p + shift) % npes][dst:dst + n] = before[p][src:src + n]
                g.barrier_all()
            else:
                me, pe = rep % npes, (rep + 1) % npes
                g.launch_wg_put(me, pe, dst, src, n, n_wg)
                o.wg_put(me, dst, src, n, pe, n_wg)
                g.quiet(me)
            assert_heaps_equal(g, o, upto=22 * MiB, what=f"case {rep}: dst+{da}, src+{sa}, {n} bytes, {n_wg} groups")


@pytest.mark.parametrize("n_wg", [32, 77, 100])
def test_a_pes_own_long_puts_asked_of_32_to_100_groups_run_by_ticket(n_wg):
    """One PE's own put or get of 32 MiB or more asked of 32-100 groups draws its pieces from that PE's
    counter pair: both PEs launching at once (each on its own pair), odd byte addresses, ragged lengths,
    launches in a row on the same pair."""
    g, o = make_pair(2, 112 * MiB)
    with g:
        fill_random(g, o, 13, upto=108 * MiB)
        cases = [(0, 0, 32 * MiB), (7, 7, 32 * MiB + 65536 + 3), (16, 5, 33 * MiB - 11)]
        for rep, (da, sa, n) in enumerate(cases):
            src, dst = 1024 + sa, 36 * MiB + da
            for me in (0, 1):
                g.launch_wg_put(me, 1 - me, dst, src, n, n_wg)
            before = [h[src:src + n].copy() for h in o.heap]
            for me in (0, 1):
                o.heap[1 - me][dst:dst + n] = before[me]
            g.quiet(0)
            g.quiet(1)
            g.launch_wg_get(rep % 2, 1 - rep % 2, 72 * MiB + sa, dst, n, n_wg)
            o.wg_get(rep % 2, 72 * MiB + sa, dst, n, 1 - rep % 2, n_wg)
            g.quiet(rep % 2)
            assert_heaps_equal(g, o, upto=108 * MiB, what=f"case {rep}: dst+{da}, src+{sa}, {n} bytes, {n_wg} groups")


@pytest.mark.timeout(600)
def test_a_pes_own_puts_of_128_mib_run_by_ticket_in_two_ways():
    """From 128 MiB a PE's own put or get asked of a group per compute unit or more is walked as two halves
    of whole tiles, each by half of the groups on its own counter pair: odd addresses, a ragged length, an
    odd number of tiles, put and get back, twice in a row on the same pairs, both PEs launching at once."""
    g, o = make_pair(2, 392 * MiB)
    with g:
        fill_random(g, o, 14, upto=390 * MiB)
        n = 128 * MiB + 65536 * 3 + 16 * 7 + 3
        src, dst, back = 1024 + 5, 130 * MiB + 11, 260 * MiB + 2
        for rep in range(2):
            for me in (0, 1):
                g.launch_wg_put(me, 1 - me, dst, src + rep, n, 256 + 768 * rep)
            before = [h[src + rep:src + rep + n].copy() for h in o.heap]
            for me in (0, 1):
                o.heap[1 - me][dst:dst + n] = before[me]
            g.quiet(0)
            g.quiet(1)
            g.launch_wg_get(rep, 1 - rep, back, dst, n, 1024)
            o.wg_get(rep, back, dst, n, 1 - rep, 1024)
            g.quiet(rep)
            assert_heaps_equal(g, o, upto=390 * MiB, what=f"launch {rep}")


@pytest.mark.timeout(600)
def test_team_puts_of_128_mib_asked_of_fewer_groups_run_by_ticket():
    """From 128 MiB per PE a team put asked of fewer groups than the ticket form's own count, but of a
    group per compute unit in all or more, runs by ticket with a whole number of groups per unit (4 PEs:
    70 asked, 64 run; 127 asked, 64 run): ragged length at an odd destination, put then get."""
    npes = 4
    g, o = make_pair(npes, 264 * MiB)
    with g:
        fill_random(g, o, 12, upto=262 * MiB)
        n = 128 * MiB + 65536 + 16 * 3 + 5
        src, dst = 64, 130 * MiB + 9
        g.launch_wg_put_all(1, dst, src, n, 70, S.SHM_PATH_LDST)
        before = [h[src:src + n].copy() for h in o.heap]
        for p in range(npes):
            o.heap[(p + 1) % npes][dst:dst + n] = before[p]
        g.barrier_all()
        g.launch_wg_get_all(3, src + 16, dst, n, 127, S.SHM_PATH_LDST)
        before = [h[dst:dst + n].copy() for h in o.heap]
        for p in range(npes):
            o.heap[p][src + 16:src + 16 + n] = before[(p + 3) % npes]
        g.barrier_all()
        assert_heaps_equal(g, o, upto=262 * MiB, what="128 MiB by ticket with fewer groups")


def test_team_puts_by_ticket_at_any_byte_address():
    """The long team put walks from the destination's next 1 KiB boundary and reads a source that is
    then off a 16-byte boundary as the aligned words around each vector: every combination class of
    destination and source address modulo 16 (equal, words apart, bytes apart, either one aligned),
    lengths that leave a byte tail, a partial tile, or neither; put and get in turn on the same counters."""
    npes = 4
    g, o = make_pair(npes, 72 * MiB)
    with g:
        fill_random(g, o, 10, upto=70 * MiB)
        cases = [(3, 3, 32 * MiB + 5), (0, 5, 32 * MiB), (9, 0, 32 * MiB + 65536 - 9), (8, 4, 33 * MiB + 1), (1, 15, 32 * MiB + 1024 - 1),
                 (13, 6, 32 * MiB + 16), (1008, 0, 32 * MiB + 16), (1023, 1, 32 * MiB), (16, 12, 32 * MiB + 32768 + 7)]
        for rep, (da, sa, n) in enumerate(cases):
            src, dst = 2048 + sa, 35 * MiB + da
            shift = 1 + rep % (npes - 1)
            if rep % 2 == 0:
                g.launch_wg_put_all(shift, dst, src, n, 128 + 50 * rep, S.SHM_PATH_LDST)
                before = [h.copy() for h in o.heap]
                for p in range(npes):
                    o.heap[(p + shift) % npes][dst:dst + n] = before[p][src:src + n]
            else:
                g.launch_wg_get_all(shift, src, dst, n, 1024, S.SHM_PATH_LDST)
                before = [h.copy() for h in o.heap]
                for p in range(npes):
                    o.heap[p][src:src + n] = before[(p + shift) % npes][dst:dst + n]
            g.barrier_all()
            assert_heaps_equal(g, o, upto=70 * MiB, what=f"case {rep}: dst+{da}, src+{sa}, {n} bytes")


@pytest.mark.parametrize("npes", [2, 3, 4, 7])
def test_team_puts_by_ticket_at_the_edges_of_the_piece_count(npes):
    """Half-tile pieces by ticket (team grids of two PEs or more, 32 MiB or more, 128 groups or more
    asked; 128 groups per PE run at even PE counts, 85 at three PEs, 109 at seven): exactly 32 MiB (1024 pieces), one vector more (a partial tile of 16 bytes), one byte more,
    one tile less than a whole number plus a byte tail, and the same sizes again at once, put and get
    in turn, so that every launch but the first depends on its predecessor having set the counters back."""
    g, o = make_pair(npes, 72 * MiB)
    with g:
        fill_random(g, o, 9, upto=70 * MiB)
        sizes = [32 * MiB, 32 * MiB + 16, 32 * MiB + 1, 33 * MiB - 65536 + 17, 32 * MiB + 32768 + 48]
        for rep, n in enumerate(sizes + sizes[:2]):
            src, dst = 16 * (rep % 3), 35 * MiB + 16 * (rep % 5)
            shift = 1 + rep % (npes - 1)
            if rep % 2 == 0:
                g.launch_wg_put_all(shift, dst, src, n, 128 + 100 * rep)
                before = [h.copy() for h in o.heap]
                for p in range(npes):
                    o.heap[(p + shift) % npes][dst:dst + n] = before[p][src:src + n]
            else:
                g.launch_wg_get_all(shift, src, dst, n, 1024)
                before = [h.copy() for h in o.heap]
                for p in range(npes):
                    o.heap[p][src:src + n] = before[(p + shift) % npes][dst:dst + n]
            g.barrier_all()
            assert_heaps_equal(g, o, upto=70 * MiB, what=f"launch {rep}, {n} bytes")
