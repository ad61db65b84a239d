"""GPU test of the entry point that allocates nothing: shm_launch_ring_pipeline_static, called through
the C ABI, against shm_launch_ring_pipeline on the same inputs -- landing slots, accumulators and
signal words bit for bit -- twice in a row, the second call with a smaller input (fewer and shorter
chunks), so that whatever the first call left in the static scratch array is seen not to matter."""
import numpy as np
import pytest

from paper_2409_20476_amd import shm as S, synth

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def _run(g, launch, npes, src, slot, acc, sig, cb, n_chunks, n_prod, n_cons, n_sig, chunk_elems, seed):
    """Fresh inputs, stale slots and accumulators, zero signals; returns everything the ring produces."""
    for p in range(npes):
        g.write(p, src, synth.c3_chunks(p + seed, n_chunks, chunk_elems))
        g.write(p, slot, np.full(cb * n_chunks, 0xEE, np.uint8))
        g.write(p, acc, np.full(4 * chunk_elems, 0x7F, np.uint8))
        g.write(p, sig, np.zeros(8 * n_sig, np.uint8))
    launch(src, slot, sig, acc, cb, n_chunks, n_prod, n_cons, n_sig)
    g.barrier_all()
    return [(g.read(p, slot, cb * n_chunks).copy(), g.read(p, acc, 4 * chunk_elems).copy(), g.read(p, sig, 8 * n_sig).copy())
            for p in range(npes)]


@pytest.mark.parametrize("n_sig_lanes", [False, True])
def test_static_ring_matches_the_allocating_entry_point_twice_in_a_row(n_sig_lanes):
    npes = 4
    g = S.Shm.on_torch(npes, 16 * MiB)
    with g:
        big = dict(n_chunks=24, chunk_elems=8 * 2048 * 3 + 8 * 5, n_prod=3, n_cons=4)
        small = dict(n_chunks=5, chunk_elems=2048 + 8, n_prod=2, n_cons=3)
        cb_max = 2 * big["chunk_elems"]
        src, slot = g.malloc(cb_max * big["n_chunks"]), g.malloc(cb_max * big["n_chunks"])
        acc, sig = g.malloc(4 * big["chunk_elems"]), g.calloc(8 * 8, 8)
        for call, shape in enumerate((big, small)):          # two calls in a row, the second with the smaller input
            n_chunks, chunk_elems = shape["n_chunks"], shape["chunk_elems"]
            n_prod, n_cons = (4, 4) if n_sig_lanes else (shape["n_prod"], shape["n_cons"])
            n_sig = 4 if n_sig_lanes else 1
            cb = 2 * chunk_elems
            args = (npes, src, slot, acc, sig, cb, n_chunks, n_prod, n_cons, n_sig, chunk_elems, 10 * call)
            got = _run(g, g.launch_ring_pipeline_static, *args)
            want = _run(g, g.launch_ring_pipeline, *args)
            for p in range(npes):
                assert np.array_equal(got[p][2], want[p][2]) and got[p][2].view(np.uint64).tolist() == [n_chunks] * n_sig, f"signals of PE {p}"
                assert np.array_equal(got[p][0], want[p][0]), f"call {call}: landing slots of PE {p}"
                assert np.array_equal(got[p][1], want[p][1]), f"call {call}: accumulator of PE {p}"


def test_static_ring_refuses_more_chunks_than_its_scratch_holds():
    g = S.Shm.on_torch(2, 8 * MiB)
    with g:
        n = S.SHM_STATIC_RING_MAX_CHUNKS + 1
        src, slot, acc, sig = g.calloc(16 * n), g.calloc(16 * n), g.calloc(32), g.calloc(8, 8)
        with pytest.raises(S.ShmError) as e:
            g.launch_ring_pipeline_static(src, slot, sig, acc, 16, n, 1, 1, 1)
        assert e.value.code == S.SHM_EINVAL and "static scratch" in str(e.value)
        g.launch_ring_pipeline(src, slot, sig, acc, 16, n, 1, 1, 1)       # the entry point with counters in the heap takes it
        g.barrier_all()
        assert g.read(0, sig, 8, np.uint64)[0] == n
