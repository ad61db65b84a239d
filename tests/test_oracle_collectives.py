"""Pins for the oracle's collectives, the ring composite and the input generators (CPU only)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle.shmem_oracle import CMP_GE, SIGNAL_ADD, OracleError, ShmemOracle
from paper_2409_20476_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _fill(o, seed):
    rng = np.random.default_rng(seed)
    for p in range(o.npes):
        o.heap[p][:] = rng.integers(0, 256, o.heap_bytes, dtype=np.uint8)


@pytest.mark.parametrize("npes,n", [(1, 7), (2, 16), (3, 33), (8, 100)])
def test_fcollect_is_concatenate_on_every_pe(npes, n):
    o = ShmemOracle(npes, 2048)
    _fill(o, n)
    before = [h.copy() for h in o.heap]
    want = np.concatenate([before[p][40:40 + n] for p in range(npes)])     # library routine
    o.fcollect(1024, 40, n)
    for q in range(npes):
        assert (o.heap[q][1024:1024 + n * npes] == want).all()
        rest = np.ones(2048, bool)
        rest[1024:1024 + n * npes] = False
        assert (o.heap[q][rest] == before[q][rest]).all()                  # nothing else touched


def test_fcollect_equals_gets_by_every_pe():
    """Built a second way, from the already pinned getmem: PE q fetches block p from PE p."""
    a, b = ShmemOracle(4, 1024), ShmemOracle(4, 1024)
    _fill(a, 1), _fill(b, 1)
    a.fcollect(512, 8, 50)
    for q in range(4):
        for p in range(4):
            b.getmem(q, 512 + 50 * p, 8, 50, p)
    assert all((x == y).all() for x, y in zip(a.heap, b.heap))


def test_fcollect_refuses_overlapping_buffers_and_accepts_touching_ones():
    """Peers write a PE's destination while that PE's source is still being read, so an overlap has
    no unique result; buffers that merely touch are fine."""
    o = ShmemOracle(4, 1024)
    _fill(o, 2)
    before = [h.copy() for h in o.heap]
    for dst, src, n in [(0, 0, 10), (0, 39, 10), (100, 95, 10), (100, 103, 1)]:
        with pytest.raises(OracleError):
            o.fcollect(dst, src, n)
    assert all((x == y).all() for x, y in zip(before, o.heap))
    o.fcollect(0, 40, 10)            # destination [0, 40), source [40, 50)
    o.fcollect(100, 90, 10)          # source ends where the destination begins
    o.fcollect(0, 0, 0)


def test_reduce_golden_order_example():
    rows = [[float(x) for x in l.split()] for l in open(os.path.join(GOLDEN, "reduce_order_example.txt"))
            if not l.startswith("#")]
    o = ShmemOracle(3, 256)
    for p in range(3):
        o.write(p, 0, np.array(rows[p], dtype=np.float32))
    o.reduce_sum_f32(128, 0, 4)
    for q in range(3):
        assert o.read(q, 128, 16, np.float32).tolist() == rows[3]


def test_reduce_special_cases_and_bounds():
    rng = np.random.default_rng(11)
    # one PE: identity
    o = ShmemOracle(1, 4096)
    x = rng.standard_normal(100).astype(np.float32)
    o.write(0, 0, x)
    o.reduce_sum_f32(2048, 0, 100)
    assert (o.read(0, 2048, 400, np.float32) == x).all()
    # small integers: every partial sum is exact, so the result equals the integer sum
    o = ShmemOracle(8, 8192)
    ints = rng.integers(-1000, 1000, size=(8, 500))
    for p in range(8):
        o.write(p, 0, ints[p].astype(np.float32))
    o.reduce_sum_f32(4096, 0, 500)
    for q in range(8):
        assert (o.read(q, 4096, 2000, np.float32).astype(np.int64) == ints.sum(0)).all()
    # N(0,1): within (npes-1) roundings of the exact sum, |err| <= 7 * 2^-24 * sum|x|
    vals = rng.standard_normal((8, 500)).astype(np.float32)
    for p in range(8):
        o.write(p, 0, vals[p])
    r = o.reduce_sum_f32(4096, 0, 500)
    got = o.read(3, 4096, 2000, np.float32)
    for i in range(500):
        exact = math.fsum(float(v) for v in vals[:, i])
        mag = math.fsum(abs(float(v)) for v in vals[:, i])
        assert abs(float(got[i]) - exact) <= 7 * 2.0 ** -24 * mag
        assert abs(r["f64"][i] - exact) <= 1e-12 * max(mag, 1.0)
        assert abs(r["abs"][i] - mag) <= 1e-12 * max(mag, 1.0)
    with pytest.raises(OracleError):
        o.reduce_sum_f32(4098, 0, 4)


def test_bf16_widening_and_rounding_match_torch():
    rng = np.random.default_rng(2)
    bits = rng.integers(0, 65536, 5000, dtype=np.uint16)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF]                 # finite values only
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    got = ShmemOracle.bf16_bits_to_f32(bits)
    assert (got.view(np.uint32) == want.view(np.uint32)).all()
    x = (rng.random(20000, dtype=np.float32) * 2 - 1).astype(np.float32)
    x[:4] = [0.0, 1.0, -1.0, 1.00390625]                      # last one is a tie: rounds to even
    want_bits = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (synth.f32_to_bf16_bits(x) == want_bits).all()


def test_ring_slots_signal_and_accumulator():
    npes, n_chunks, nel = 4, 6, 40
    cb = 2 * nel
    o = ShmemOracle(npes, 4096)
    src, slot, sig, acc = 0, 1024, 2048, 2304
    chunks = [synth.c3_chunks(p, n_chunks, nel) for p in range(npes)]
    for p in range(npes):
        o.write(p, src, chunks[p])
    o.ring_pipeline(src, slot, sig, acc, cb, n_chunks, n_wg_prod=3)
    for p in range(npes):
        prev = (p - 1) % npes
        assert (o.read(p, slot, cb * n_chunks, np.uint16).reshape(n_chunks, nel) == chunks[prev]).all()
        assert o.signal_fetch(p, sig) == n_chunks
        got = o.read(p, acc, 4 * nel, np.float32)
        # second construction: torch widening, explicit left-to-right binary32 adds
        t = torch.zeros(nel, dtype=torch.float32)
        for k in range(n_chunks):
            t = t + torch.from_numpy(chunks[prev][k].view(np.int16).copy()).view(torch.bfloat16).float()
        assert (got == t.numpy()).all()
        for i in range(nel):
            vals = [float(ShmemOracle.bf16_bits_to_f32(chunks[prev][k, i:i + 1])[0]) for k in range(n_chunks)]
            assert abs(float(got[i]) - math.fsum(vals)) <= (n_chunks - 1) * 2.0 ** -24 * math.fsum(map(abs, vals))


def test_ring_equal_chunks_give_exact_multiple_and_order_is_chunk_order():
    o = ShmemOracle(2, 4096)
    x = np.array([0.5, -0.75, 1.0, 0.0078125], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(x)
    for p in range(2):
        o.write(p, 0, np.tile(bits, (64, 1)))
    o.ring_pipeline(0, 1024, 2048, 2056 + 8, 8, 64)
    assert (o.read(0, 2064, 16, np.float32) == 64 * x).all()
    # order: 256, then 64 values of 2^-17... use bf16-exact values where order matters in binary32
    o = ShmemOracle(1, 4096)
    seq = np.array([[16777216.0], [1.0], [1.0], [-16777216.0]], dtype=np.float32)
    o.write(0, 0, synth.f32_to_bf16_bits(seq.reshape(-1)).reshape(4, 1))
    o.ring_pipeline(0, 64, 128, 256, 2, 4)
    # ((0 + 2^24) + 1) -> 2^24 (tie to even), + 1 -> 2^24, - 2^24 -> 0; any other order gives 1 or 2
    assert o.read(0, 256, 4, np.float32)[0] == 0.0


def test_ring_equals_composition_of_pinned_ops():
    npes, n_chunks, nel = 3, 5, 24
    a, b = ShmemOracle(npes, 2048), ShmemOracle(npes, 2048)
    for p in range(npes):
        c = synth.c3_chunks(p, n_chunks, nel)
        a.write(p, 0, c), b.write(p, 0, c)
    a.ring_pipeline(0, 512, 1024, 1280, 2 * nel, n_chunks)
    accs = np.zeros((npes, nel), dtype=np.float32)
    for p in range(npes):               # a different legal order: PE by PE instead of chunk by chunk
        for k in range(n_chunks):
            b.put_signal(p, 512 + k * 2 * nel, k * 2 * nel, 2 * nel, 1024, 1, SIGNAL_ADD, (p + 1) % npes)
    for p in range(npes):
        for k in range(n_chunks):
            b.signal_wait_until(p, 1024, CMP_GE, k + 1)
            accs[p] += ShmemOracle.bf16_bits_to_f32(b.read(p, 512 + k * 2 * nel, 2 * nel, np.uint16))
        b.write(p, 1280, accs[p])
    assert all((x == y).all() for x, y in zip(a.heap, b.heap))


def test_ring_lanes_give_the_same_data_and_one_counter_per_lane():
    """Cutting every chunk into shares that travel with their own signal changes neither slots nor sums."""
    npes, n_chunks, nel = 3, 5, 72
    a, b = ShmemOracle(npes, 4096), ShmemOracle(npes, 4096)
    for p in range(npes):
        c = synth.c3_chunks(p, n_chunks, nel)
        a.write(p, 0, c), b.write(p, 0, c)
    a.ring_pipeline(0, 1024, 2048, 2304, 2 * nel, n_chunks)
    b.ring_pipeline(0, 1024, 2048, 2304, 2 * nel, n_chunks, n_sig=4)
    for p in range(npes):
        assert (a.read(p, 1024, 2 * nel * n_chunks) == b.read(p, 1024, 2 * nel * n_chunks)).all()
        assert (a.read(p, 2304, 4 * nel) == b.read(p, 2304, 4 * nel)).all()
        assert a.read(p, 2048, 32, np.uint64).tolist() == [n_chunks, 0, 0, 0]
        assert b.read(p, 2048, 32, np.uint64).tolist() == [n_chunks] * 4


def test_synth_is_seeded_and_in_range():
    assert (synth.c1_payload() == synth.c1_payload()).all()
    v = synth.c1_payload()
    assert v.dtype == np.int32 and v.min() >= 0 and v.size == 4096
    assert synth.c2_source(3, 8).size == 8 and (synth.c2_source(3, 64)[:8] == synth.c2_source(3, 8)).all()
    assert not (synth.c2_source(3, 64) == synth.c2_source(4, 64)).all()
    t = synth.c4_targets(128, 8, 16, 1024)
    assert t.dtype == np.uint16 and t.shape == (128, 8) and t.max() < 16384
    c = ShmemOracle.bf16_bits_to_f32(synth.c3_chunks(0, 2, 1000))
    assert c.min() >= -1.0 and c.max() <= 1.0
    assert synth.c5_fcollect_source(1, 10).dtype == np.int32 and synth.c5_reduce_source(1, 10).dtype == np.float32


def test_broadcast_is_a_put_from_the_root_to_everyone():
    a, b = ShmemOracle(5, 512), ShmemOracle(5, 512)
    _fill(a, 9), _fill(b, 9)
    a.broadcast(300, 17, 101, 3)
    for q in range(5):
        if q == 3:
            b.heap[3][300:401] = b.heap[3][17:118].copy()       # the root's own copy, byte for byte
        else:
            b.putmem(3, 300, 17, 101, q)
    assert all((x == y).all() for x, y in zip(a.heap, b.heap))
    with pytest.raises(OracleError):
        a.broadcast(20, 17, 101, 3)
    with pytest.raises(OracleError):
        a.broadcast(300, 17, 101, 5)


def test_barrier_exchange_delivers_every_neighbours_block():
    npes, n = 4, 24
    o = ShmemOracle(npes, 1024)
    _fill(o, 4)
    blocks = [o.heap[p][8:8 + n].copy() for p in range(npes)]
    o.barrier_exchange(256, 8, 512, n, 3)
    for p in range(npes):
        for r in range(3):
            assert (o.heap[p][512 + r * n:512 + (r + 1) * n] == blocks[(p - 1 - r) % npes]).all()
    assert o.log.count(("barrier_all",)) == 3


def test_wave_exchange_is_put_flag_wait_get_per_slice():
    # closed form: destination and back buffer equal the source, flags and fetched values are 1,
    # for ragged sizes and more waves than 16-byte units
    for n, n_waves in [(1000, 7), (16, 4), (0, 3), (4096, 1), (100, 64)]:
        o = ShmemOracle(3, 1 << 15)
        _fill(o, n + n_waves)
        before = [h.copy() for h in o.heap]
        src, dst, back, flag, out = 64, 8192, 16384, 24576, 28672
        for p in range(3):
            o.heap[p][flag:flag + 8 * n_waves] = 0
            before[p][flag:flag + 8 * n_waves] = 0
        o.wave_exchange(2, 1, dst, src, back, n, n_waves, flag, out)
        want = before[2][src:src + n]
        assert np.array_equal(o.heap[1][dst:dst + n], want)
        assert np.array_equal(o.heap[1][back:back + n], want)
        assert np.all(o.heap[1][flag:flag + 8 * n_waves].view(np.uint64) == 1)
        assert np.all(o.heap[1][out:out + 8 * n_waves].view(np.uint64) == 1)
        # nothing else changed anywhere
        touched = np.zeros(1 << 15, bool)
        for a, m in ((dst, n), (back, n), (flag, 8 * n_waves), (out, 8 * n_waves)):
            touched[a:a + m] = True
        assert np.array_equal(o.heap[1][~touched], before[1][~touched])
        assert np.array_equal(o.heap[0], before[0]) and np.array_equal(o.heap[2], before[2])


def test_collect_is_concatenate_of_unequal_blocks_and_reduces_to_fcollect():
    o = ShmemOracle(4, 1 << 14)
    _fill(o, 11)
    before = [h.copy() for h in o.heap]
    sizes = [100, 0, 37, 1]
    o.collect(4096, 64, sizes)
    want = np.concatenate([before[p][64:64 + sizes[p]] for p in range(4)])
    for q in range(4):
        assert np.array_equal(o.heap[q][4096:4096 + 138], want)
        assert np.array_equal(o.heap[q][:4096], before[q][:4096]) and np.array_equal(o.heap[q][4096 + 138:], before[q][4096 + 138:])
    # equal sizes: exactly fcollect
    a, b = ShmemOracle(3, 8192), ShmemOracle(3, 8192)
    _fill(a, 12), _fill(b, 12)
    a.collect(4096, 0, [200] * 3), b.fcollect(4096, 0, 200)
    assert all(np.array_equal(x, y) for x, y in zip(a.heap, b.heap))
    for bad in (lambda: o.collect(4096, 64, [1, 2, 3]), lambda: o.collect(4096, 64, [1, 2, 3, -1]),
                lambda: o.collect(100, 64, [100, 0, 0, 0]), lambda: o.collect(16000, 64, [200, 200, 0, 0])):
        with pytest.raises(OracleError):
            bad()
