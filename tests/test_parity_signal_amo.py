"""GPU parity: put-with-signal, signal_wait_until, bounded waits, 64-bit atomics and the atomic storm."""
import numpy as np
import pytest
import torch

from oracle.shmem_oracle import SIGNAL_ADD, SIGNAL_SET
from paper_2409_20476_amd import shm as S, synth
from parity_util import assert_heaps_equal, fill_random, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20


@pytest.mark.parametrize("n_wg", [1, 2, 5, 64])
def test_put_signal_then_wait_sees_data(n_wg):
    g, o = make_pair(4, 4 * MiB)
    with g:
        fill_random(g, o, 11)
        sig = 3 * MiB
        for p in range(4):
            write_both(g, o, p, sig, np.zeros(16, np.uint8))
        out = torch.zeros(4, dtype=torch.int64, device="cuda")
        cases = [(0, 1, 100003, SIGNAL_SET, 7, S.SHM_CMP_EQ, 7), (2, 1, 0, SIGNAL_ADD, 5, S.SHM_CMP_GE, 12),
                 (3, 0, MiB + 16, SIGNAL_ADD, (1 << 64) - 1, S.SHM_CMP_NE, 0), (1, 1, 4096, SIGNAL_SET, 1 << 63, S.SHM_CMP_GT, 1)]
        for i, (me, pe, n, op, val, cmp, cval) in enumerate(cases):
            dst, src = MiB + MiB // 2 + 8 * i, 24 + i
            g.launch_wg_put_signal(me, pe, dst, src, n, sig, val, op, n_wg)      # producer first: it never waits
            g.launch_signal_wait_until(pe, sig, cmp, cval, out[i:i + 1])
            # the waiter's stream then copies the payload onward: after the wait it must already be there
            if 0 < n <= 200000:
                g.launch_wg_put(pe, (pe + 1) % 4, 2 * MiB + MiB // 2, dst, n, 1)
            g.barrier_all()
            o.put_signal(me, dst, src, n, sig, val, op, pe, n_wg)
            want = o.signal_wait_until(pe, sig, cmp, cval)
            if 0 < n <= 200000:
                o.wg_put(pe, 2 * MiB + MiB // 2, dst, n, (pe + 1) % 4, 1)
            assert int(out[i].item()) & ((1 << 64) - 1) == want
            assert_heaps_equal(g, o, what=f"case {i}")


def test_put_signal_random_sizes_alignments_and_group_counts():
    """The write-through payload path of put_signal (aligned and re-aligned forms, head and tail
    bytes, arrival counting by several groups) at random sizes and alignments."""
    g, o = make_pair(2, 4 * MiB)
    rng = np.random.default_rng(34)
    with g:
        fill_random(g, o, 34, upto=3 * MiB)
        sig = 3 * MiB - 64
        write_both(g, o, 0, sig, np.zeros(8, np.uint8)), write_both(g, o, 1, sig, np.zeros(8, np.uint8))
        for i in range(120):
            n_wg = int(rng.choice([1, 2, 3, 5, 8, 64]))
            n = int(rng.integers(0, 200000)) if i % 3 else int(rng.integers(0, 200))
            sa, da = int(rng.integers(0, 48)), int(rng.integers(0, 48))
            me = i & 1
            op, val = (SIGNAL_ADD, 3) if i % 4 else (SIGNAL_SET, 1000 + i)
            g.launch_wg_put_signal(me, 1 - me, 2 * MiB + da, 1024 + sa, n, sig, val, op, n_wg)
            o.put_signal(me, 2 * MiB + da, 1024 + sa, n, sig, val, op, 1 - me, n_wg)
            if i % 10 == 9:
                g.barrier_all()
                assert_heaps_equal(g, o, upto=3 * MiB, what=f"after case {i} (n_wg {n_wg}, n {n}, src+{sa}, dst+{da})")
        g.barrier_all()
        assert_heaps_equal(g, o, upto=3 * MiB, what="end")


def test_wait_before_signal_on_other_stream_and_timeout_is_reported():
    g, o = make_pair(2, MiB)
    with g:
        fill_random(g, o, 12)
        write_both(g, o, 1, 4096, np.zeros(8, np.uint8))
        # a wait nobody satisfies: bounded, reported by the next quiet, and the context stays usable
        g.set_wait_timeout_us(2000)
        g.launch_signal_wait_until(1, 4096, S.SHM_CMP_EQ, 99)
        with pytest.raises(S.ShmError) as e:
            g.quiet(1)
        assert e.value.code == S.SHM_ETIMEOUT
        g.quiet(1)                              # status was cleared
        g.set_wait_timeout_us(2_000_000)
        g.launch_wg_put_signal(0, 1, 8192, 0, 1000, 4096, 99, SIGNAL_SET, 1)
        g.launch_signal_wait_until(1, 4096, S.SHM_CMP_EQ, 99)
        g.barrier_all()
        o.put_signal(0, 8192, 0, 1000, 4096, 99, SIGNAL_SET, 1)
        assert_heaps_equal(g, o)


def test_every_comparison_at_its_boundary_unsigned():
    """All six comparisons of signal_wait_until one below, at and one above the signal's value, and
    across 2^63 (the comparison is unsigned).  The oracle says whether the wait can be satisfied; on
    the GPU a wait that cannot be satisfied runs into the (here tiny) bound and is reported."""
    from oracle.shmem_oracle import OracleError
    g, o = make_pair(2, MiB)
    cmps = [S.SHM_CMP_EQ, S.SHM_CMP_NE, S.SHM_CMP_GT, S.SHM_CMP_GE, S.SHM_CMP_LT, S.SHM_CMP_LE]
    pairs = [(5, 4), (5, 5), (5, 6), (2 ** 63 + 1, 1), (1, 2 ** 63 + 1), (2 ** 64 - 1, 2 ** 64 - 1), (0, 2 ** 64 - 1)]
    with g:
        out = torch.zeros(1, dtype=torch.int64, device="cuda")
        g.set_wait_timeout_us(300)
        satisfied = 0
        for sig_value, value in pairs:
            word = np.array([sig_value], dtype=np.uint64)
            write_both(g, o, 1, 256, word)
            for cmp in cmps:
                try:
                    want = o.signal_wait_until(1, 256, cmp, value)
                except OracleError:
                    want = None
                out.fill_(-1)
                torch.cuda.synchronize()
                g.launch_signal_wait_until(1, 256, cmp, value, out)
                if want is None:
                    with pytest.raises(S.ShmError) as e:
                        g.quiet(1)
                    assert e.value.code == S.SHM_ETIMEOUT, (sig_value, value, cmp)
                else:
                    g.quiet(1)
                    assert int(out.item()) & (2 ** 64 - 1) == want == sig_value, (sig_value, value, cmp)
                    satisfied += 1
        assert satisfied == 21          # EQ 2, NE 5, GT 2, GE 4, LT 3, LE 5 of the 7 pairs
        g.set_wait_timeout_us(2_000_000)


def test_every_atomic_matches_the_oracle():
    g, o = make_pair(3, MiB)
    with g:
        fill_random(g, o, 13, upto=8192)
        out = torch.zeros(1, dtype=torch.int64, device="cuda")
        I64_MAX = 2 ** 63 - 1
        ops = [(S.SHM_AMO_SET, 64, 5, 0, 2), (S.SHM_AMO_FETCH, 64, 0, 0, 2), (S.SHM_AMO_FETCH_ADD, 64, -9, 0, 2),
               (S.SHM_AMO_ADD, 64, 100, 0, 2), (S.SHM_AMO_FETCH_INC, 64, 0, 0, 2), (S.SHM_AMO_INC, 64, 0, 0, 2),
               (S.SHM_AMO_SWAP, 64, I64_MAX, 0, 2), (S.SHM_AMO_FETCH_ADD, 64, 1, 0, 2), (S.SHM_AMO_FETCH, 64, 0, 0, 2),
               (S.SHM_AMO_COMPARE_SWAP, 64, 77, -2 ** 63, 2), (S.SHM_AMO_COMPARE_SWAP, 64, 78, 5, 2),
               (S.SHM_AMO_FETCH, 64, 0, 0, 2), (S.SHM_AMO_FETCH_ADD, 8, 3, 0, 0), (S.SHM_AMO_COMPARE_SWAP, 8, -1, 12345, 1)]
        names = {S.SHM_AMO_SET: "atomic_set", S.SHM_AMO_FETCH: "atomic_fetch", S.SHM_AMO_FETCH_ADD: "atomic_fetch_add",
                 S.SHM_AMO_ADD: "atomic_add", S.SHM_AMO_FETCH_INC: "atomic_fetch_inc", S.SHM_AMO_INC: "atomic_inc",
                 S.SHM_AMO_SWAP: "atomic_swap", S.SHM_AMO_COMPARE_SWAP: "atomic_compare_swap"}
        for i, (op, off, operand, cond, pe) in enumerate(ops):
            me = i % 3
            out.fill_(-12345)
            torch.cuda.synchronize()
            g.launch_amo(me, pe, off, op, operand, cond, out)
            g.quiet(me)
            fn = getattr(o, names[op])
            if op in (S.SHM_AMO_FETCH, S.SHM_AMO_FETCH_INC):
                want = fn(me, off, pe)
            elif op == S.SHM_AMO_INC:
                want = fn(me, off, pe)
            elif op == S.SHM_AMO_COMPARE_SWAP:
                want = fn(me, off, cond, operand, pe)
            else:
                want = fn(me, off, operand, pe)
            if want is not None:
                assert int(out.item()) == want, (i, op)
            assert_heaps_equal(g, o, upto=8192, what=f"amo {i}")
        with pytest.raises(S.ShmError):
            g.launch_amo(0, 1, 12, S.SHM_AMO_FETCH)       # misaligned target


def _check_storm(g, o, npes, n_ctr, n_items, ops, kind, ctr_off):
    targets = synth.c4_targets(n_items, ops, npes, n_ctr)
    t_dev = torch.from_numpy(targets.view(np.int16)).cuda()
    fetched = torch.empty(n_items * ops, dtype=torch.int64, device="cuda")
    n_groups = (n_items + 255) // 256
    checksum = torch.zeros(n_groups, dtype=torch.int64, device="cuda")
    g.launch_amo_storm(ctr_off, n_ctr, t_dev, n_items, ops, kind, fetched, checksum)
    g.barrier_all()
    init = np.concatenate([o.read(p, ctr_off, 8 * n_ctr, np.int64) for p in range(npes)])
    o.amo_storm(ctr_off, n_ctr, targets)           # final counters; its fetched values are one witness only
    for p in range(npes):
        assert np.array_equal(g.read(p, ctr_off, 8 * n_ctr, np.int64), o.read(p, ctr_off, 8 * n_ctr, np.int64)), f"counters of PE {p}"
    if kind == S.SHM_STORM_ADD:
        return
    flat = targets.reshape(-1).astype(np.int64)
    got = fetched.cpu().numpy() - init[flat]
    counts = np.bincount(flat, minlength=npes * n_ctr)
    assert got.min() >= 0 and (got < counts[flat]).all(), "a fetched value outside 0..n-1"
    start = np.concatenate([[0], np.cumsum(counts)[:-1]])
    hits = np.bincount(start[flat] + got, minlength=flat.size)
    assert (hits == 1).all(), "fetched values of a counter are not a permutation of 0..n-1"
    # per-group checksums equal the sum of what the group's items fetched (mod 2^64)
    per_item = fetched.cpu().numpy().reshape(n_items, ops).sum(axis=1)
    pad = np.zeros(n_groups * 256, dtype=np.int64)
    pad[:n_items] = per_item
    assert np.array_equal(checksum.cpu().numpy(), pad.reshape(n_groups, 256).sum(axis=1))


@pytest.mark.parametrize("kind", [S.SHM_STORM_FETCH_ADD, S.SHM_STORM_ADD, S.SHM_STORM_CSWAP_LOOP, S.SHM_STORM_FETCH_ADD_WG])
@pytest.mark.parametrize("npes,n_ctr,n_items,ops", [(2, 4, 1000, 10), (16, 1024, 1 << 14, 64), (3, 7, 300, 3), (5, 100, 2500, 64),
                                                    (8, 2048, 5000, 16), (1, 1, 1025, 64), (4, 300, 300000, 8), (3, 50, 2000, 100)])
def test_storm_small(kind, npes, n_ctr, n_items, ops):
    g, o = make_pair(npes, MiB)
    with g:
        rng = np.random.default_rng(5)
        for p in range(npes):
            write_both(g, o, p, 512, rng.integers(-3, 3, n_ctr, dtype=np.int64))
        _check_storm(g, o, npes, n_ctr, n_items, ops, kind, 512)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("kind", [S.SHM_STORM_FETCH_ADD, S.SHM_STORM_FETCH_ADD_WG])
def test_config4_full_size(kind):
    """16 PEs x 1024 counters, 2^20 work-items x 64 fetch-adds, scalar and batched by work-groups."""
    g, o = make_pair(16, MiB)
    with g:
        for p in range(16):
            write_both(g, o, p, 0, np.zeros(1024, np.int64))
        _check_storm(g, o, 16, 1024, 1 << 20, 64, kind, 0)


def test_batched_storm_carries_into_the_high_half_of_a_counter():
    """Counters that start just below 2^32 and at the most negative value: the group's one fetch-add
    per counter and the places added to what it fetched are 64-bit arithmetic."""
    g, o = make_pair(2, MiB)
    with g:
        start = np.array([(1 << 32) - 5, -(1 << 63), -3, (1 << 62)], dtype=np.int64)
        for p in range(2):
            write_both(g, o, p, 1024, start)
        _check_storm(g, o, 2, 4, 3000, 64, S.SHM_STORM_FETCH_ADD_WG, 1024)


@pytest.mark.parametrize("how", ["put_signal", "put_then_atomic"])
@pytest.mark.parametrize("rounds,seed", [(150, 81), (150, 82)])
def test_ping_pong_with_credits_many_rounds_without_host_synchronisation(rounds, seed, how):
    """The protocol put-with-signal exists for, all of it enqueued up front on two PEs' streams:
    PE 0 waits for a credit, puts the round's payload into ONE reused buffer on PE 1 with signal
    'data += 1'; PE 1 waits for the data, copies the payload away and returns a credit with a
    zero-byte put-with-signal.  Only the signals order the two streams: a payload read before it has
    landed, or overwritten before it was read, shows in the copies.
    how == "put_then_atomic": the payload travels with a plain work-group put and the signal is a
    separate atomic add launched behind it on the same stream -- successive launches of one PE are
    delivered in order (the host-side fence is the stream's order), which is what this form checks."""
    g, o = make_pair(2, 48 * MiB)
    rng = np.random.default_rng(seed)
    with g:
        fill_random(g, o, seed, upto=40 * MiB)
        data_sig, credit_sig, buf, keep = 39 * MiB, 39 * MiB + 64, 16 * MiB, 17 * MiB
        for p in range(2):
            write_both(g, o, p, 39 * MiB, np.zeros(128, np.uint8))
        at = keep
        for r in range(rounds):
            n = int(rng.integers(0, 120000)) if r % 5 else int(rng.choice([0, 1, 8, 16, 4096]))
            src, off, n_wg = int(rng.integers(0, 15 * MiB)), int(rng.integers(0, 16)), int(rng.choice([1, 2, 3, 16]))
            # PE 0: wait until the buffer is free again (r credits returned), then send
            g.launch_signal_wait_until(0, credit_sig, S.SHM_CMP_GE, r)
            if how == "put_signal":
                g.launch_wg_put_signal(0, 1, buf + off, src, n, data_sig, 1, SIGNAL_ADD, n_wg)
            else:
                g.launch_wg_put(0, 1, buf + off, src, n, n_wg)
                g.fence(0)
                g.launch_amo(0, 1, data_sig, S.SHM_AMO_ADD, 1)
            # PE 1: wait for round r's data, keep a copy, give the buffer back
            g.launch_signal_wait_until(1, data_sig, S.SHM_CMP_GE, r + 1)
            g.launch_wg_put(1, 1, at, buf + off, n, int(rng.choice([1, 4])))
            g.launch_wg_put_signal(1, 0, 0, 0, 0, credit_sig, 1, SIGNAL_ADD, 1)
            o.signal_wait_until(0, credit_sig, S.SHM_CMP_GE, r)
            o.put_signal(0, buf + off, src, n, data_sig, 1, SIGNAL_ADD, 1, n_wg)
            o.signal_wait_until(1, data_sig, S.SHM_CMP_GE, r + 1)
            o.putmem(1, at, buf + off, n, 1)
            o.put_signal(1, 0, 0, 0, credit_sig, 1, SIGNAL_ADD, 0, 1)
            at += n + int(rng.integers(0, 64))
        g.barrier_all()
        assert o.signal_fetch(1, data_sig) == rounds and o.signal_fetch(0, credit_sig) == rounds
        assert_heaps_equal(g, o, upto=40 * MiB, what=f"{rounds} rounds")
