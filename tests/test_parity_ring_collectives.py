"""GPU parity: pipelined ring (configuration 3), fcollect and float32 sum-reduce (configuration 5)."""
import numpy as np
import pytest

from paper_2409_20476_amd import shm as S, synth
from parity_util import assert_heaps_equal, fill_random, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20
GiB = 1 << 30


def _ring_case(npes, n_chunks, chunk_elems, n_prod, n_cons, heap, reps=1, n_sig=1):
    g, o = make_pair(npes, heap)
    with g:
        cb = 2 * chunk_elems
        src, slot, acc, sig = g.malloc(cb * n_chunks), g.malloc(cb * n_chunks), g.malloc(4 * chunk_elems), g.calloc(8 * n_sig, 8)
        for p in range(npes):
            chunks = synth.c3_chunks(p, n_chunks, chunk_elems)
            write_both(g, o, p, src, chunks)
            write_both(g, o, p, slot, np.full(cb * n_chunks, 0xEE, np.uint8))     # stale landing slots
            write_both(g, o, p, acc, np.full(4 * chunk_elems, 0x7F, np.uint8))
        for rep in range(reps):
            for p in range(npes):
                write_both(g, o, p, sig, np.zeros(8 * n_sig, np.uint8))
            g.launch_ring_pipeline(src, slot, sig, acc, cb, n_chunks, n_prod, n_cons, n_sig)
            g.barrier_all()
            o.ring_pipeline(src, slot, sig, acc, cb, n_chunks, n_prod, n_sig)
            for p in range(npes):
                assert g.read(p, sig, 8 * n_sig, np.uint64).tolist() == [n_chunks] * n_sig
                assert np.array_equal(g.read(p, sig, 8 * n_sig), o.read(p, sig, 8 * n_sig))
                assert np.array_equal(g.read(p, slot, cb * n_chunks), o.read(p, slot, cb * n_chunks)), f"slots of PE {p}"
                got, want = g.read(p, acc, 4 * chunk_elems, np.uint32), o.read(p, acc, 4 * chunk_elems, np.uint32)
                assert np.array_equal(got, want), f"accumulator of PE {p} (rep {rep})"
            # next repetition sends different data through the same (now stale) slots
            for p in range(npes):
                chunks = synth.c3_chunks(p + 100 * (rep + 1), n_chunks, chunk_elems)
                write_both(g, o, p, src, chunks)


@pytest.mark.parametrize("npes,n_chunks,chunk_elems,n_prod,n_cons", [
    (2, 3, 8, 1, 1), (3, 5, 2048 + 8, 2, 3), (8, 16, 16384, 4, 4), (4, 7, 8 * 2048 * 3 + 8 * 5, 3, 4), (1, 4, 4096, 2, 2)])
def test_ring_small(npes, n_chunks, chunk_elems, n_prod, n_cons):
    _ring_case(npes, n_chunks, chunk_elems, n_prod, n_cons, 8 * MiB, reps=3)


@pytest.mark.parametrize("npes,n_chunks,chunk_elems,lanes", [(2, 3, 8, 1), (3, 5, 2048 + 8, 3), (8, 16, 16384, 8),
                                                            (4, 7, 8 * 2048 * 3 + 8 * 5, 5), (2, 4, 64, 16)])
def test_ring_lanes_small(npes, n_chunks, chunk_elems, lanes):
    _ring_case(npes, n_chunks, chunk_elems, lanes, lanes, 8 * MiB, reps=3, n_sig=lanes)


@pytest.mark.timeout(600)
def test_config3_full_size():
    """8 PEs, 64 chunks of 1 MiB bf16 each, in the launch shape the benchmark times."""
    _ring_case(8, 64, 524288, 8, 32, 256 * MiB, reps=2)


@pytest.mark.timeout(600)
def test_config3_full_size_one_counter_pipelined():
    """One counter per PE with producer shares small enough for the two-half pipeline."""
    _ring_case(8, 64, 524288, 32, 32, 256 * MiB, reps=2)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("n_prod,n_cons", [(16, 32), (9, 32), (11, 40)])
def test_ring_producer_shares_of_32_to_128_kib_keep_two_blocks_in_registers(n_prod, n_cons):
    """1 MiB chunks by 16, 9 and 11 producer groups per PE: shares of 64, 114 and 93 KiB per chunk (one
    block, and two blocks with a ragged second one), the last group's share shorter than the others';
    three rounds through the same slots."""
    _ring_case(8, 24, 524288, n_prod, n_cons, 128 * MiB, reps=3)


@pytest.mark.timeout(600)
def test_config3_full_size_lanes():
    """The same with one signal counter per producer/consumer group pair."""
    _ring_case(8, 64, 524288, 32, 32, 256 * MiB, reps=2, n_sig=32)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("n_prod,n_cons,n_sig", [(16, 16, 16), (4, 16, 1), (16, 16, 1), (8, 32, 1)])
def test_ring_many_rounds_never_reads_a_stale_slot(n_prod, n_cons, n_sig):
    """Ten rounds through the same slots with fresh data each time: a signal seen before its payload
    would leave a previous round's bytes in an accumulator."""
    _ring_case(8, 32, 131072, n_prod, n_cons, 64 * MiB, reps=10, n_sig=n_sig)


def test_ring_rejects_grids_that_cannot_be_resident():
    g, o = make_pair(8, 8 * MiB)
    with g:
        with pytest.raises(S.ShmError) as e:
            g.launch_ring_pipeline(0, MiB, 4 * MiB, 2 * MiB, 65536, 4, 4096, 4096)
        assert e.value.code == S.SHM_EINVAL
        with pytest.raises(S.ShmError):
            g.launch_ring_pipeline(0, 2 * MiB, 6 * MiB, 5 * MiB, 1 << 20, 2, 1, 1)     # consumer share too big for registers
        with pytest.raises(S.ShmError):
            g.launch_ring_pipeline(0, MiB, 4 * MiB, 2 * MiB, 65536, 4, 4, 8, 4)        # lanes need equal group counts


@pytest.mark.parametrize("path", [S.SHM_PATH_LDST, S.SHM_PATH_SDMA, S.SHM_PATH_MEMCPY])
@pytest.mark.parametrize("npes,n,n_wg,soff,doff", [(8, 4096 * 17 + 16, 8, 0, 0), (3, 1000, 2, 3, 5), (8, 300016, 64, 0, 0),
                                                  (5, 7, 1, 1, 2), (2, 0, 4, 0, 0), (4, 262144 * 3 + 48, 16, 0, 0)])
def test_fcollect(path, npes, n, n_wg, soff, doff):
    g, o = make_pair(npes, 16 * MiB)
    with g:
        fill_random(g, o, 21, upto=12 * MiB)
        src, dst = 256 + soff, 2 * MiB + doff
        g.launch_fcollect(dst, src, n, n_wg, path)
        g.barrier_all()
        o.fcollect(dst, src, n)
        assert_heaps_equal(g, o, upto=12 * MiB)


@pytest.mark.parametrize("npes,n,n_wg", [(8, 8 * MiB, 1024), (8, 8 * MiB + 65536 + 48, 32), (8, 9 * MiB - 16, 31), (16, 8 * MiB + 16, 16),
                                         (6, 8 * MiB + 32, 42), (7, 9 * MiB - 48, 500)])
def test_fcollect_of_long_blocks_by_ticket(npes, n, n_wg):
    """From 8 MiB per PE, 6 PEs or more and as many groups asked as the launcher runs (256 / npes per PE)
    the groups of a PE draw 16 KiB pieces of its block by ticket: whole tiles only, a rest of less than
    a tile, one group too few (fixed tiles then), 16 PEs; twice in a row, the second launch with other
    source bytes, so that it depends on the counters having been set back."""
    g, o = make_pair(npes, (npes + 2) * 9 * MiB + MiB)
    rng = np.random.default_rng(23)
    with g:
        fill_random(g, o, 23, upto=(npes + 1) * 9 * MiB + 65536)
        src, dst = 64, 9 * MiB + 128
        for rep in range(2):
            g.launch_fcollect(dst, src, n, n_wg, S.SHM_PATH_LDST)
            g.barrier_all()
            o.fcollect(dst, src, n)
            assert_heaps_equal(g, o, upto=(npes + 1) * 9 * MiB + 65536, what=f"launch {rep}")
            for p in range(npes):
                write_both(g, o, p, src + 4096 * p, rng.integers(0, 256, 100000, dtype=np.uint8))


@pytest.mark.parametrize("algo", [S.SHM_REDUCE_DUPLICATE, S.SHM_REDUCE_SPLIT])
@pytest.mark.parametrize("npes,nelems,n_wg,soff,doff", [(8, 4096 * 5 + 3, 8, 0, 0), (3, 1001, 2, 4, 8), (8, 65536 * 9 + 4, 64, 0, 0),
                                                       (1, 777, 3, 0, 0), (5, 2, 1, 0, 0), (4, 131072 * 3 + 1, 16, 16, 32)])
def test_reduce_sum_f32(algo, npes, nelems, n_wg, soff, doff):
    g, o = make_pair(npes, 16 * MiB)
    with g:
        fill_random(g, o, 22, upto=12 * MiB)
        src, dst = 1024 + soff, 6 * MiB + doff
        for p in range(npes):
            write_both(g, o, p, src, synth.c5_reduce_source(p, nelems))
        g.launch_reduce_sum_f32(dst, src, nelems, n_wg, algo)
        g.barrier_all()
        r = o.reduce_sum_f32(dst, src, nelems)
        assert_heaps_equal(g, o, upto=12 * MiB)                       # bit-exact, every PE, canaries intact
        got = g.read(npes - 1, dst, 4 * nelems, np.float32).astype(np.float64)
        assert (np.abs(got - r["f64"]) <= 1e-6 * r["abs"]).all()      # and within the stated tolerance of the exact sum


@pytest.mark.parametrize("npes,n_wg", [(2, 8), (2, 100), (3, 64)])
def test_reduce_sum_f32_split_on_group_owned_tiles(npes, n_wg):
    """A split reduction whose per-PE slice has 64 or more 64 KiB tiles walks them as group-owned tiles:
    slices of 64 tiles plus a ragged rest, a scalar tail, fewer and more groups than tiles; also the
    duplicate form of the same size."""
    nvec = npes * (64 * 4096 + 1000) - 3
    nelems = 4 * nvec + 3
    g, o = make_pair(npes, 40 * MiB)
    with g:
        fill_random(g, o, 23, upto=36 * MiB)
        src, dst = 4096, 18 * MiB + 16
        for p in range(npes):
            write_both(g, o, p, src, synth.c5_reduce_source(p, nelems))
        r = o.reduce_sum_f32(dst, src, nelems)
        for algo in (S.SHM_REDUCE_SPLIT, S.SHM_REDUCE_DUPLICATE):
            g.launch_reduce_sum_f32(dst, src, nelems, n_wg, algo)
            g.barrier_all()
            assert_heaps_equal(g, o, upto=36 * MiB, what=f"algo {algo}")
            for p in range(npes):
                g.write(p, dst, np.full(4 * nelems, 0x5A, np.uint8))


@pytest.mark.parametrize("npes,n_wg", [(2, 128), (2, 1024), (3, 85), (3, 200)])
def test_reduce_sum_f32_split_by_ticket(npes, n_wg):
    """A split reduction with 96 or more tiles per PE, asked of a group per compute unit or more, draws
    quarter tiles by ticket: slices of 96 tiles plus a ragged rest (the last PE's slice is shorter, the
    slices start on tile boundaries), a scalar tail; three launches in a row, so that every launch but
    the first depends on its predecessor having set the counters back."""
    nvec = npes * (96 * 4096 + 1000) - 3
    nelems = 4 * nvec + 3
    g, o = make_pair(npes, 48 * MiB)
    with g:
        fill_random(g, o, 24, upto=44 * MiB)
        src, dst = 4096, 22 * MiB + 16
        for rep in range(3):
            for p in range(npes):
                write_both(g, o, p, src, synth.c5_reduce_source(p + 10 * rep, nelems))
            o.reduce_sum_f32(dst, src, nelems)
            g.launch_reduce_sum_f32(dst, src, nelems, n_wg, S.SHM_REDUCE_SPLIT)
            g.barrier_all()
            assert_heaps_equal(g, o, upto=44 * MiB, what=f"launch {rep}")


def test_reduce_sum_f32_split_when_the_last_slice_is_short():
    """Six PEs, slices rounded up to whole tiles: five PEs walk 65 group-owned tiles each and the last
    one is left with 59 tiles and some vectors, which it deals to its groups the plain way."""
    npes = 6
    nvec = npes * 64 * 4096 + 6
    nelems = 4 * nvec + 1
    g, o = make_pair(npes, 56 * MiB)
    with g:
        fill_random(g, o, 25, upto=52 * MiB)
        src, dst = 4096, 26 * MiB + 16
        for p in range(npes):
            write_both(g, o, p, src, synth.c5_reduce_source(p, nelems))
        o.reduce_sum_f32(dst, src, nelems)
        for n_wg in (16, 300):
            g.launch_reduce_sum_f32(dst, src, nelems, n_wg, S.SHM_REDUCE_SPLIT)
            g.barrier_all()
            assert_heaps_equal(g, o, upto=52 * MiB, what=f"{n_wg} groups")
            for p in range(npes):
                g.write(p, dst, np.full(4 * nelems, 0x5A, np.uint8))


@pytest.mark.timeout(900)
def test_config5_full_size():
    """8 PEs: fcollect of 64 MiB int32 per PE into 512 MiB, and a 16M-element float32 sum-reduce."""
    npes, nel = 8, 16 * MiB
    g, o = make_pair(npes, GiB)
    with g:
        fsrc, fdst = g.malloc(4 * nel), g.malloc(4 * nel * npes)
        rsrc, rdst = g.malloc(4 * nel), g.malloc(4 * nel)
        for p in range(npes):
            write_both(g, o, p, fsrc, synth.c5_fcollect_source(p, nel))
            write_both(g, o, p, rsrc, synth.c5_reduce_source(p, nel))
        g.launch_fcollect(fdst, fsrc, 4 * nel, 1024, S.SHM_PATH_LDST)
        g.barrier_all()
        o.fcollect(fdst, fsrc, 4 * nel)
        for q in range(npes):
            assert np.array_equal(g.read(q, fdst, 4 * nel * npes), o.heap[q][fdst:fdst + 4 * nel * npes]), f"fcollect on PE {q}"
        r = None
        for algo in (S.SHM_REDUCE_DUPLICATE, S.SHM_REDUCE_SPLIT):
            for q in range(npes):
                g.write(q, rdst, np.zeros(16, np.uint8))
            g.launch_reduce_sum_f32(rdst, rsrc, nel, 1024, algo)
            g.barrier_all()
            r = r or o.reduce_sum_f32(rdst, rsrc, nel)
            for q in range(npes):
                got = g.read(q, rdst, 4 * nel, np.uint32)
                assert np.array_equal(got, r["f32"].view(np.uint32)), f"reduce algo {algo} on PE {q}"
            got = g.read(0, rdst, 4 * nel, np.float32).astype(np.float64)
            assert (np.abs(got - r["f64"]) <= 1e-6 * r["abs"]).all()


@pytest.mark.timeout(900)
def test_config2_full_size_team_put():
    """8 PEs x 256 MiB float32, 1024 work-groups each, to PE (p+1) mod 8 -- the benchmark's launch."""
    npes, n = 8, 256 * MiB
    g, o = make_pair(npes, GiB)
    with g:
        src, dst = g.malloc(n), g.malloc(n)
        data = [synth.c2_source(p, n) for p in range(npes)]
        for p in range(npes):
            g.write(p, src, data[p])
            g.write(p, dst, np.zeros(4096, np.uint8))
        g.launch_wg_put_all(1, dst, src, n, 1024, S.SHM_PATH_LDST)
        g.barrier_all()
        for p in range(npes):
            assert np.array_equal(g.read((p + 1) % npes, dst, n), data[p]), f"put of PE {p}"
        # the 64 MiB and 128 MiB points of the same curve (half-tile pieces drawn by ticket by 128 groups per PE), the
        # second with a rest after the whole steps and a byte tail; put and get, other shifts
        for m, shift in ((64 * MiB, 2), (128 * MiB - 4096 * 3 + 16 + 7, 5)):
            g.launch_wg_put_all(shift, dst, src, m, 1024, S.SHM_PATH_LDST)
            g.barrier_all()
            for p in range(npes):
                got = g.read((p + shift) % npes, dst, n)
                assert np.array_equal(got[:m], data[p][:m]), f"long put of PE {p}, {m} bytes"
                assert np.array_equal(got[m:], data[(p + shift - 1) % npes][m:]), f"bytes behind the long put of PE {p}"
            g.launch_wg_put_all(1, dst, src, n, 1024, S.SHM_PATH_LDST)            # every PE holds its left neighbour's data again
            g.barrier_all()
            g.launch_wg_get_all(shift, dst, src, m, 1024, S.SHM_PATH_LDST)
            g.barrier_all()
            for p in range(npes):
                got = g.read(p, dst, n)
                assert np.array_equal(got[:m], data[(p + shift) % npes][:m]), f"long get of PE {p}, {m} bytes"
                assert np.array_equal(got[m:], data[(p - 1) % npes][m:]), f"bytes behind the long get of PE {p}"
            g.launch_wg_put_all(1, dst, src, n, 1024, S.SHM_PATH_LDST)
            g.barrier_all()
        # per-PE streams, copy-engine path, smaller message with a ragged tail
        m = 64 * MiB + 1000
        for p in range(npes):
            g.launch_wg_put(p, (p + 3) % npes, dst, src, m, 1024, S.SHM_PATH_SDMA)
        g.barrier_all()
        for p in range(npes):
            got = g.read((p + 3) % npes, dst, n)
            assert np.array_equal(got[:m], data[p][:m]) and np.array_equal(got[m:], data[(p + 2) % npes][m:])
