"""CPU-only tests of the C ABI's host side: symbols, argument checking, allocator, policy.

They use a context built with SHM_INIT_NO_DEVICE, which makes no HIP call; nothing is computed.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2409_20476_amd import shm as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MiB = 1 << 20


def _ctx(npes=4, heap=MiB):
    return S.Shm(npes, heap, heap_base=4096, flags=S.SHM_INIT_NO_DEVICE)


def test_library_exports_every_declared_symbol_and_binding_covers_them():
    header = open(os.path.join(ROOT, "include", "shm355.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(shm_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 30
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2409_20476_amd", "libshm355.so"))
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared but not exported"
    assert declared == set(S.PROTOTYPES), declared ^ set(S.PROTOTYPES)


def test_constants_match_header():
    header = open(os.path.join(ROOT, "include", "shm355.h")).read()
    for name, val in re.findall(r"\b(SHM_[A-Z0-9_]+)\s*=\s*(-?\d+)", header):
        assert getattr(S, name) == int(val), name
    assert f"#define SHM_MAX_PES        {S.SHM_MAX_PES}" in header
    assert f"#define SHM_INTERNAL_BYTES {S.SHM_INTERNAL_BYTES}" in header


def test_init_argument_checks():
    for npes, heap, code in [(0, MiB, S.SHM_EPE), (33, MiB, S.SHM_EPE), (2, 65536, S.SHM_EINVAL), (2, MiB + 1, S.SHM_EINVAL)]:
        with pytest.raises(S.ShmError) as e:
            _ctx(npes, heap)
        assert e.value.code == code
    with pytest.raises(S.ShmError):
        S.Shm(2, MiB, heap_base=4096 + 8, flags=S.SHM_INIT_NO_DEVICE)      # misaligned base
    with pytest.raises(S.ShmError):
        S.Shm(2, MiB, heap_base=4096, flags=64)
    g = _ctx()
    assert g.n_pes() == 4 and g.heap_bytes() == MiB - S.SHM_INTERNAL_BYTES
    assert g.ptr(0, 0) == 4096 and g.ptr(16, 3) == 4096 + 3 * MiB + 16 and g.ptr(0, 4) == 0 and g.ptr(MiB, 0) == 0
    g.finalize()


def test_allocator_invariants_through_the_abi():
    g = _ctx(4, 4 * MiB)
    rng = np.random.default_rng(3)
    live = {}
    for _ in range(2000):
        if live and rng.random() < 0.45:
            off = list(live)[int(rng.integers(len(live)))]
            g.free(off)
            del live[off]
            continue
        n = int(rng.integers(1, 60000))
        align = int(2 ** rng.integers(0, 13))
        try:
            off = g.malloc(n, align)
        except S.ShmError as e:
            assert e.code == S.SHM_ENOMEM
            continue
        assert off % align == 0 and off + n <= g.heap_bytes()
        for o2, n2 in live.items():
            assert off + n <= o2 or o2 + n2 <= off, "live blocks overlap"
        live[off] = n
    for off in list(live):
        g.free(off)
    assert g.malloc(g.heap_bytes(), 1) == 0            # everything coalesced back into one extent
    with pytest.raises(S.ShmError) as e:
        g.malloc(1)
    assert e.value.code == S.SHM_ENOMEM
    g.finalize()


def test_allocator_edge_cases():
    g = _ctx()
    assert g.malloc(0) == S.SHM_NULL_OFF
    g.free(S.SHM_NULL_OFF)
    a = g.malloc(10)
    assert a % 256 == 0                                  # default alignment
    b = g.calloc(100, 64)                                # no device: allocates, zeroing is skipped
    assert b % 64 == 0 and b != a
    for bad in (lambda: g.free(a + 16), lambda: g.malloc(8, 3), lambda: g.malloc(2 * MiB)):
        with pytest.raises(S.ShmError):
            bad()
    g.free(a)
    with pytest.raises(S.ShmError):
        g.free(a)                                        # double free
    g.finalize()


def test_every_entry_point_validates_before_touching_the_device():
    g = _ctx(4, MiB)
    H = g.heap_bytes()
    E = S.ShmError

    def code(fn):
        with pytest.raises(E) as e:
            fn()
        return e.value.code

    # valid arguments reach the device step, which a no-device context refuses
    assert code(lambda: g.launch_wg_put(0, 1, 4096, 0, 100, 4)) == S.SHM_ENODEV
    assert code(lambda: g.launch_wg_put_all(1, 4096, 0, 100, 4)) == S.SHM_ENODEV
    assert code(lambda: g.putmem(0, 4096, 0, 100, 1)) == S.SHM_ENODEV
    assert code(lambda: g.quiet(0)) == S.SHM_ENODEV
    assert code(lambda: g.write(0, 0, np.zeros(4, np.uint8))) == S.SHM_ENODEV
    assert code(lambda: g.launch_pingflag(0, 16384, 16384, 40000)) == S.SHM_ENODEV
    assert code(lambda: g.launch_ring_pipeline(0, 65536, 262144, 131072, 4096, 4, 2, 2, 1)) == S.SHM_ENODEV
    assert code(lambda: g.launch_amo_storm(0, 16, 4096, 100, 8)) == S.SHM_ENODEV
    assert code(lambda: g.launch_fcollect(65536, 0, 1000, 2)) == S.SHM_ENODEV
    assert code(lambda: g.launch_reduce_sum_f32(65536, 0, 1000, 2)) == S.SHM_ENODEV
    # bad PEs
    assert code(lambda: g.launch_wg_put(4, 1, 4096, 0, 100, 4)) == S.SHM_EPE
    assert code(lambda: g.launch_wg_put(0, -1, 4096, 0, 100, 4)) == S.SHM_EPE
    assert code(lambda: g.launch_wg_put_all(4, 4096, 0, 100, 4)) == S.SHM_EPE
    assert code(lambda: g.quiet(9)) == S.SHM_EPE
    # ranges: the library's own tail of the partition is off limits
    assert code(lambda: g.launch_wg_put(0, 1, H - 50, 0, 100, 4)) == S.SHM_ERANGE
    assert code(lambda: g.launch_wg_get(0, 1, 0, H, 1, 4)) == S.SHM_ERANGE
    assert code(lambda: g.launch_wg_put(0, 1, 0, 0, 1 << 62, 4)) == S.SHM_ERANGE
    assert code(lambda: g.launch_fcollect(0, H - 8, H // 2, 2)) == S.SHM_ERANGE
    assert code(lambda: g.launch_reduce_sum_f32(0, 65536, H, 2)) == S.SHM_ERANGE
    # overlap, alignment, enumerations, counts
    assert code(lambda: g.launch_wg_put(1, 1, 50, 0, 100, 4)) == S.SHM_EINVAL
    assert code(lambda: g.launch_wg_put(0, 1, 4096, 0, 100, 0)) == S.SHM_EINVAL
    assert code(lambda: g.launch_wg_put(0, 1, 4096, 0, 100, 4, 7)) == S.SHM_EINVAL
    assert code(lambda: g.launch_wg_put_signal(0, 1, 4096, 0, 100, 8196, 1, S.SHM_SIGNAL_SET)) == S.SHM_EINVAL     # misaligned
    assert code(lambda: g.launch_wg_put_signal(0, 1, 4096, 0, 100, 4104, 1, S.SHM_SIGNAL_SET)) == S.SHM_EINVAL     # inside payload
    assert code(lambda: g.launch_wg_put_signal(0, 1, 4096, 0, 100, 8192, 1, 5)) == S.SHM_EINVAL
    assert code(lambda: g.launch_signal_wait_until(0, 8192, 9, 1)) == S.SHM_EINVAL
    assert code(lambda: g.launch_amo(0, 1, 12, S.SHM_AMO_FETCH)) == S.SHM_EINVAL
    assert code(lambda: g.launch_amo(0, 1, 16, 99)) == S.SHM_EINVAL
    assert code(lambda: g.launch_ring_pipeline(0, 65536, 262144, 131072, 4100, 4, 2, 2, 1)) == S.SHM_EINVAL     # chunk not x16
    assert code(lambda: g.launch_ring_pipeline(0, 65536, 262144, 131072, 4096, 4, 2, 3, 2)) == S.SHM_EINVAL     # lanes need equal groups
    assert code(lambda: g.launch_ring_pipeline(0, 8192, 262144, 131072, 4096, 4, 2, 2, 1)) == S.SHM_EINVAL      # src/slots overlap
    assert code(lambda: g.launch_ring_pipeline(0, 65536, 65536 + 4096, 131072, 4096, 4, 2, 2, 1)) == S.SHM_EINVAL     # signal inside the slots
    assert code(lambda: g.launch_ring_pipeline(0, 65536, 262144, 131072, 4096, 4, 1 << 21, 2, 1)) == S.SHM_EINVAL     # too many groups
    assert code(lambda: g.launch_amo_storm(0, 16, 4096 + 2, 100, 8)) == S.SHM_EINVAL                            # table alignment
    assert code(lambda: g.launch_amo_storm(0, 1 << 15, 4096, 100, 8)) == S.SHM_EINVAL                           # 16-bit ids
    assert code(lambda: g.launch_amo_storm(0, 4097, 4096, 100, 8, S.SHM_STORM_FETCH_ADD_WG)) == S.SHM_EINVAL    # batched: 4 x 4097 counters > LDS table
    assert code(lambda: g.launch_amo_storm(0, 4096, 4096, 100, 64, S.SHM_STORM_FETCH_ADD_WG)) == S.SHM_ENODEV   # ... 4 x 4096 fit
    assert code(lambda: g.launch_amo_storm(0, 16, 4096, 100, 8, S.SHM_STORM_FETCH_ADD_WG + 1)) == S.SHM_EINVAL   # unknown kind
    assert code(lambda: g.launch_reduce_sum_f32(65538, 0, 1000, 2)) == S.SHM_EINVAL
    assert code(lambda: g.launch_reduce_sum_f32(0, 0, 1000, 2, 5)) == S.SHM_EINVAL
    assert code(lambda: g.launch_fcollect(100, 0, 1000, 2)) == S.SHM_EINVAL                                     # overlap
    # strided, single-thread and general device-initiated transfers
    assert code(lambda: g.launch_iput(0, 1, 4096, 0, 2, 3, 100, 4, 0)) == S.SHM_ENODEV
    assert code(lambda: g.launch_iget(0, 1, 4096, 0, 2, 3, 100, 16, 8)) == S.SHM_ENODEV
    assert code(lambda: g.launch_iput(0, 1, 4096, 0, 0, 3, 100, 4, 0)) == S.SHM_EINVAL                        # stride < 1
    assert code(lambda: g.launch_iput(0, 1, 4096, 0, 2, 3, 100, 5, 0)) == S.SHM_EINVAL                        # element size
    assert code(lambda: g.launch_iput(0, 1, 4098, 0, 2, 3, 100, 4, 0)) == S.SHM_EINVAL                        # alignment
    assert code(lambda: g.launch_iput(0, 0, 0, 16, 8, 1, 100, 4, 0)) == S.SHM_EINVAL                          # spans overlap on one PE
    assert code(lambda: g.launch_iput(0, 1, 0, 0, H // 400 + 1, 1, 101, 4, 0)) == S.SHM_ERANGE
    assert code(lambda: g.launch_iget(0, 1, 0, 0, 1, (1 << 62), 3, 8, 0)) == S.SHM_ERANGE
    assert code(lambda: g.launch_iget(0, 1, 0, 0, 1, 1, (1 << 63), 16, 0)) == S.SHM_ERANGE
    assert code(lambda: g.launch_wave_exchange(0, 1, 4096, 0, 8192, 100, 4, 16384, 20480)) == S.SHM_ENODEV
    assert code(lambda: g.launch_wave_exchange(0, 1, 4096, 0, 4100, 100, 4, 16384, 20480)) == S.SHM_EINVAL    # back overlaps dst
    assert code(lambda: g.launch_wave_exchange(0, 1, 4096, 0, 8192, 100, 4, 16388, 20480)) == S.SHM_EINVAL    # flag alignment
    assert code(lambda: g.launch_wave_exchange(0, 1, 4096, 0, 8192, 100, 0, 16384, 20480)) == S.SHM_EINVAL
    assert code(lambda: g.launch_wave_exchange(0, 1, 4096, 0, 8192, 100, 4, H - 8, 20480)) == S.SHM_ERANGE
    assert code(lambda: g.launch_scalar_pg(0, 1, 4096, 0, 100, 8)) == S.SHM_ENODEV
    assert code(lambda: g.launch_scalar_pg(0, 1, 4096, 0, 100, 16)) == S.SHM_EINVAL
    assert code(lambda: g.launch_scalar_pg(0, 1, 4098, 0, 100, 4)) == S.SHM_EINVAL
    assert code(lambda: g.launch_scalar_pg(0, 1, 4096, 0, H, 8)) == S.SHM_ERANGE
    assert code(lambda: g.launch_thread_rma(0, 1, 4096, 0, 100)) == S.SHM_ENODEV
    assert code(lambda: g.launch_thread_rma(0, 0, 50, 0, 100)) == S.SHM_EINVAL
    assert code(lambda: g.launch_rma_device_initiated(0, 1, 4096, 0, 100, 2, True, 0)) == S.SHM_ENODEV
    assert code(lambda: g.launch_rma_device_initiated(0, 1, 4096, 0, 100, 2, True, 5)) == S.SHM_ENODEV
    assert code(lambda: g.launch_rma_device_initiated(0, 1, 4096, 0, 100, 2, True, 6)) == S.SHM_EINVAL
    assert code(lambda: g.launch_rma_device_initiated(0, 1, 4096, 0, 100, 2, True, 5, consume_off=8192)) == S.SHM_EINVAL   # nothing to consume before the host's quiet
    assert code(lambda: g.launch_rma_device_initiated(0, 1, 4096, 0, 100, 2, False, 0, consume_off=8192)) == S.SHM_EINVAL
    assert code(lambda: g.launch_rma_device_initiated(0, 1, 4096, 0, 100, 2, True, 0, consume_off=4100)) == S.SHM_EINVAL
    assert code(lambda: g.launch_rma_device_initiated(0, 1, 4096, 0, 100, 2, True, 0, consume_off=H - 10)) == S.SHM_ERANGE
    assert code(lambda: g.launch_collect(65536, 0, [100, 0, 5, 7], 2)) == S.SHM_ENODEV
    assert code(lambda: g.launch_collect(50, 0, [100, 0, 5, 7], 2)) == S.SHM_EINVAL                             # overlap
    assert code(lambda: g.launch_collect(65536, 0, [H, 1, 0, 0], 2)) == S.SHM_ERANGE
    # the reduction matrix
    assert code(lambda: g.launch_reduce(65536, 0, 1000, S.SHM_INT16, S.SHM_OP_XOR, 2)) == S.SHM_ENODEV
    assert code(lambda: g.launch_reduce(65536, 0, 1000, S.SHM_FLOAT64, S.SHM_OP_PROD, 2)) == S.SHM_ENODEV
    assert code(lambda: g.launch_reduce(65536, 0, 1000, S.SHM_FLOAT32, S.SHM_OP_AND, 2)) == S.SHM_EINVAL       # bitwise on float
    assert code(lambda: g.launch_reduce(65536, 0, 1000, S.SHM_FLOAT64, S.SHM_OP_XOR, 2)) == S.SHM_EINVAL
    assert code(lambda: g.launch_reduce(65536, 0, 1000, 10, S.SHM_OP_SUM, 2)) == S.SHM_EINVAL
    assert code(lambda: g.launch_reduce(65536, 0, 1000, S.SHM_INT8, 7, 2)) == S.SHM_EINVAL
    assert code(lambda: g.launch_reduce(65536, 0, 1000, S.SHM_INT8, S.SHM_OP_SUM, 2, 2)) == S.SHM_EINVAL      # algorithm
    assert code(lambda: g.launch_reduce(65536, 0, 1000, S.SHM_INT8, S.SHM_OP_SUM, 2, S.SHM_REDUCE_SPLIT)) == S.SHM_ENODEV
    assert code(lambda: g.launch_reduce(65536, 8, 1000, S.SHM_INT8, S.SHM_OP_SUM, 2)) == S.SHM_EINVAL         # alignment
    assert code(lambda: g.launch_reduce(512, 0, 1000, S.SHM_INT8, S.SHM_OP_SUM, 2)) == S.SHM_EINVAL           # overlap
    assert code(lambda: g.launch_reduce(0, 65536, H, S.SHM_UINT64, S.SHM_OP_SUM, 2)) == S.SHM_ERANGE
    assert code(lambda: g.set_wait_timeout_us(0)) == S.SHM_EINVAL
    g.finalize()


def test_cutover_defaults_follow_the_hardware_queue_count(monkeypatch):
    """The measured defaults come in two sets: a hardware queue per PE stream, or fewer queues than
    PEs (HIP's default is 4 queues per process; shm_init reads GPU_MAX_HW_QUEUES)."""
    never = (1 << 64) - 1
    for env, npes, want in [(None, 4, [MiB // 2, never, never, never]), (None, 8, [MiB // 4, 2 * MiB, never, never]),
                            ("8", 8, [MiB // 2, never, never, never]), ("8", 12, [MiB // 4, 2 * MiB, never, never]),
                            ("junk", 8, [MiB // 4, 2 * MiB, never, never]), ("0", 4, [MiB // 2, never, never, never])]:
        if env is None:
            monkeypatch.delenv("GPU_MAX_HW_QUEUES", raising=False)
        else:
            monkeypatch.setenv("GPU_MAX_HW_QUEUES", env)
        g = _ctx(npes)
        assert [g.get_cutover(w) for w in (1, 4, 64, 1024)] == want, (env, npes)
        g.finalize()


def test_cutover_policy_classes(monkeypatch):
    monkeypatch.delenv("GPU_MAX_HW_QUEUES", raising=False)
    g = _ctx()
    never = (1 << 64) - 1
    assert [g.get_cutover(w) for w in (1, 4, 64, 1024)] == [MiB // 2, never, never, never]      # the measured defaults, 4 PEs on 4 queues
    assert g.choose_path(MiB // 2 - 1, 1) == S.SHM_PATH_LDST and g.choose_path(MiB // 2, 1) == S.SHM_PATH_SDMA
    assert g.choose_path(1 << 40, 4) == S.SHM_PATH_LDST and g.choose_path(1 << 40, 1024) == S.SHM_PATH_LDST
    g.set_cutover(1, 4096), g.set_cutover(3, 65536), g.set_cutover(64, MiB), g.set_cutover(65, 16 * MiB)
    assert [g.get_cutover(w) for w in (1, 2, 4, 5, 64, 100, 1 << 20)] == [4096, 65536, 65536, MiB, MiB, 16 * MiB, 16 * MiB]
    assert g.choose_path(4095, 1) == S.SHM_PATH_LDST and g.choose_path(4096, 1) == S.SHM_PATH_SDMA
    assert g.choose_path(MiB - 1, 64) == S.SHM_PATH_LDST and g.choose_path(MiB, 33) == S.SHM_PATH_SDMA
    assert g.choose_path(8 * MiB, 1024) == S.SHM_PATH_LDST and g.choose_path(16 * MiB, 1024) == S.SHM_PATH_SDMA
    with pytest.raises(S.ShmError):
        g.get_cutover(0)
    g.finalize()


def test_collective_cutover_depends_on_collective_groups_and_pes():
    """The collectives have thresholds of their own (bytes per PE), tuned per collective and, for
    fcollect, by the number of PEs; above them AUTO takes host-started runtime copies."""
    never = (1 << 64) - 1
    FC, BC = S.SHM_COLL_FCOLLECT, S.SHM_COLL_BROADCAST
    for npes, want in [(2, [MiB // 2, 2 * MiB, never, never]), (4, [MiB // 2, 2 * MiB, never, never]),
                       (5, [2 * MiB, 8 * MiB, never, never]), (12, [2 * MiB, 8 * MiB, never, never])]:
        g = _ctx(npes)
        assert [g.get_collective_cutover(FC, w) for w in (1, 4, 64, 1024)] == want
        assert [g.get_collective_cutover(BC, w) for w in (1, 4, 64, 1024)] == [MiB // 4, MiB, 16 * MiB, never]
        g.finalize()
    g = _ctx(8)
    assert g.choose_collective_path(FC, 2 * MiB - 1, 1) == S.SHM_PATH_LDST and g.choose_collective_path(FC, 2 * MiB, 1) == S.SHM_PATH_MEMCPY
    assert g.choose_collective_path(FC, 8 * MiB, 2) == S.SHM_PATH_MEMCPY and g.choose_collective_path(FC, 1 << 40, 5) == S.SHM_PATH_LDST
    assert g.choose_collective_path(BC, MiB // 4, 1) == S.SHM_PATH_MEMCPY and g.choose_collective_path(BC, MiB // 4, 2) == S.SHM_PATH_LDST
    assert g.choose_collective_path(BC, 16 * MiB, 64) == S.SHM_PATH_MEMCPY and g.choose_collective_path(BC, 1 << 40, 65) == S.SHM_PATH_LDST
    g.set_collective_cutover(FC, 64, 4096)
    assert g.get_collective_cutover(FC, 33) == 4096 and g.get_collective_cutover(BC, 33) == 16 * MiB      # one table per collective
    assert g.choose_collective_path(FC, 4096, 64) == S.SHM_PATH_MEMCPY and g.choose_collective_path(FC, 4095, 64) == S.SHM_PATH_LDST
    assert g.get_cutover(64) == never                                                                      # the put policy is untouched
    for bad in (lambda: g.get_collective_cutover(2, 1), lambda: g.set_collective_cutover(-1, 1, 0), lambda: g.get_collective_cutover(FC, 0),
                lambda: g.choose_collective_path(7, 100, 1)):
        with pytest.raises(S.ShmError) as e:
            bad()
        assert e.value.code == S.SHM_EINVAL
    g.finalize()


def test_team_grids_are_bounded_by_what_one_launch_can_hold():
    """n_wg groups for each of npes PEs run as ONE grid, which may not reach 2^32 threads."""
    g = _ctx(32, MiB)
    ok, too_many = 1 << 18, 1 << 19                    # 2^19 groups x 32 PEs x 256 threads = 2^32
    for call in (lambda w: g.launch_wg_put_all(1, 4096, 0, 100, w), lambda w: g.launch_fcollect(8192, 0, 100, w),
                 lambda w: g.launch_collect(8192, 0, [10] * 32, w), lambda w: g.launch_reduce(8192, 0, 100, S.SHM_INT32, S.SHM_OP_SUM, w),
                 lambda w: g.launch_reduce_sum_f32(8192, 0, 100, w)):
        with pytest.raises(S.ShmError) as e:
            call(ok)
        assert e.value.code == S.SHM_ENODEV
        with pytest.raises(S.ShmError) as e:
            call(too_many)
        assert e.value.code == S.SHM_EINVAL
    with pytest.raises(S.ShmError) as e:
        g.launch_wg_put(0, 1, 4096, 0, 100, 1 << 20)   # one PE's own grid may have 2^20 groups
    assert e.value.code == S.SHM_ENODEV
    g.finalize()


def test_device_view_for_application_kernels():
    """The by-value view that kernels of the caller's own take: size-checked, filled from the context;
    the separately built example application agrees with the library on its layout's size."""
    g = _ctx(3, MiB)
    n = g.lib.shm_device_context_bytes()
    view = g.device_context()
    assert len(view) == n and n >= 8 * S.SHM_MAX_PES + 8
    bases = np.frombuffer(view[:8 * S.SHM_MAX_PES], dtype=np.uint64)
    assert list(bases[:3]) == [4096, 4096 + MiB, 4096 + 2 * MiB] and not bases[3:].any()     # base[pe], then unused entries
    buf = ctypes.create_string_buffer(n)
    assert g.lib.shm_device_context(g.ctx, buf, n - 1) == S.SHM_EINVAL
    assert g.lib.shm_device_context(g.ctx, None, n) == S.SHM_EINVAL
    assert g.stream(0) == 0                                 # a context without a device has no streams
    g.finalize()
    example = ctypes.CDLL(os.path.join(ROOT, "paper_2409_20476_amd", "libshm355_user_example.so"))
    example.shmu_device_context_bytes.restype = ctypes.c_size_t
    assert example.shmu_device_context_bytes() == n
    assert hasattr(example, "shmu_alltoall")


def test_team_sync_modes():
    g = _ctx()
    for mode in (S.SHM_TEAM_SYNC_OFF, S.SHM_TEAM_SYNC_TRACKED, S.SHM_TEAM_SYNC_FULL, True, False):
        g.set_team_sync(mode)
    for bad in (3, -1, 17):
        with pytest.raises(S.ShmError) as e:
            g.set_team_sync(bad)
        assert e.value.code == S.SHM_EINVAL
    g.finalize()


def test_sync_set_argument_checks():
    g = _ctx()
    H = g.heap_bytes()

    def code(fn):
        with pytest.raises(S.ShmError) as e:
            fn()
        return e.value.code

    assert code(lambda: g.launch_sync_set(0, 4096, 4, None, S.SHM_SYNC_WAIT_ALL, S.SHM_CMP_GE, 1, 8)) == S.SHM_ENODEV
    assert code(lambda: g.launch_sync_set(0, 4096, 0, None, S.SHM_SYNC_TEST, S.SHM_CMP_EQ, -5, 8)) == S.SHM_ENODEV      # single forms look at one variable
    assert code(lambda: g.launch_sync_set(4, 4096, 4, None, S.SHM_SYNC_WAIT_ALL, S.SHM_CMP_GE, 1, 8)) == S.SHM_EPE
    assert code(lambda: g.launch_sync_set(0, 4100, 4, None, S.SHM_SYNC_WAIT_ALL, S.SHM_CMP_GE, 1, 8)) == S.SHM_EINVAL   # alignment
    assert code(lambda: g.launch_sync_set(0, H - 16, 4, None, S.SHM_SYNC_TEST_SOME, S.SHM_CMP_GE, 1, 8)) == S.SHM_ERANGE
    assert code(lambda: g.launch_sync_set(0, 4096, 1 << 62, None, S.SHM_SYNC_TEST_SOME, S.SHM_CMP_GE, 1, 8)) == S.SHM_ERANGE
    assert code(lambda: g.launch_sync_set(0, 4096, 4, None, 8, S.SHM_CMP_GE, 1, 8)) == S.SHM_EINVAL
    assert code(lambda: g.launch_sync_set(0, 4096, 4, None, S.SHM_SYNC_WAIT_ANY, 6, 1, 8)) == S.SHM_EINVAL
    assert code(lambda: g.launch_sync_set(0, 4096, 4, None, S.SHM_SYNC_WAIT_ANY, S.SHM_CMP_GE, 1, None)) == S.SHM_EINVAL
    g.finalize()
