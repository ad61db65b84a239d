"""GPU parity for benchmark configuration 1: put, quiet, flag, wait, get back."""
import numpy as np
import pytest

from oracle.shmem_oracle import CMP_EQ, SIGNAL_SET
from paper_2409_20476_amd import shm as S, synth
from parity_util import assert_heaps_equal, make_pair, write_both

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def test_config1_pingflag_bit_exact():
    g, o = make_pair(2, MiB)            # 2 PEs, 1 MiB symmetric heap each
    with g:
        payload = synth.c1_payload(4096)          # 16 KiB of int32
        n = payload.nbytes
        data, back, flag = g.malloc(n), g.malloc(n), g.calloc(8, 8)
        # canaries everywhere, then the payload on PE 0 and a zero flag on both
        rng = np.random.default_rng(7)
        for p in range(2):
            write_both(g, o, p, 0, rng.integers(0, 256, o.heap_bytes, dtype=np.uint8))
            write_both(g, o, p, flag, np.zeros(8, np.uint8))
        write_both(g, o, 0, data, payload)
        for rep in range(3):
            g.launch_pingflag(data, back, n, flag)
            g.barrier_all()
            # oracle: the same program in one legal sequential order
            o.wg_put(0, data, data, n, 1, 1)
            o.quiet(0)
            o.put_signal(0, data, data, 0, flag, 1, SIGNAL_SET, 1)
            assert o.signal_wait_until(1, flag, CMP_EQ, 1) == 1
            o.wg_get(1, back, data, n, 0, 1)
            assert_heaps_equal(g, o, what=f"rep {rep}")
            assert np.array_equal(g.read(1, data, n, np.int32), payload)
            assert np.array_equal(g.read(1, back, n, np.int32), payload)
            assert g.read(1, flag, 8, np.uint64)[0] == 1 and g.read(0, flag, 8, np.uint64)[0] == 0
            # new payload and a cleared flag for the next round
            payload = (payload ^ np.int32(0x5A5A5A5A)).astype(np.int32)
            write_both(g, o, 0, data, payload)
            write_both(g, o, 1, flag, np.zeros(8, np.uint8))
