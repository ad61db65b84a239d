"""ctypes binding of libshm355.so: argument marshalling only, same names as the C ABI.

Every operation runs in the library's HIP kernels (or the copy engine it drives).
There is no fallback: if the shared library has not been built, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_int, c_int64, c_size_t, c_uint, c_uint64, c_void_p

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libshm355.so")

SHM_MAX_PES = 32
SHM_WG_SIZE = 256
SHM_INTERNAL_BYTES = 65536
SHM_NULL_OFF = (1 << 64) - 1

SHM_OK, SHM_EINVAL, SHM_EPE, SHM_ERANGE, SHM_ENOMEM, SHM_EHIP, SHM_ETIMEOUT, SHM_ENODEV = 0, -1, -2, -3, -4, -5, -6, -7
SHM_PATH_AUTO, SHM_PATH_LDST, SHM_PATH_SDMA, SHM_PATH_MEMCPY = 0, 1, 2, 3
SHM_SIGNAL_SET, SHM_SIGNAL_ADD = 0, 1
SHM_CMP_EQ, SHM_CMP_NE, SHM_CMP_GT, SHM_CMP_GE, SHM_CMP_LT, SHM_CMP_LE = range(6)
SHM_INIT_DEFAULT, SHM_INIT_NO_DEVICE = 0, 1
(SHM_AMO_FETCH, SHM_AMO_SET, SHM_AMO_SWAP, SHM_AMO_COMPARE_SWAP, SHM_AMO_FETCH_ADD, SHM_AMO_ADD, SHM_AMO_FETCH_INC,
 SHM_AMO_INC) = range(8)
SHM_STORM_FETCH_ADD, SHM_STORM_ADD, SHM_STORM_CSWAP_LOOP, SHM_STORM_PLAIN_STORE, SHM_STORM_FETCH_ADD_WG = range(5)
SHM_REDUCE_DUPLICATE, SHM_REDUCE_SPLIT = 0, 1
SHM_PROBE_READ, SHM_PROBE_WRITE, SHM_PROBE_COPY, SHM_PROBE_READ_FRONT, SHM_PROBE_WRITE_FRONT = 0, 1, 2, 3, 4
SHM_PROBE_READ_TICKETS, SHM_PROBE_WRITE_TICKETS = 5, 6
SHM_STATIC_RING_MAX_CHUNKS = 1024
SHM_COLL_FCOLLECT, SHM_COLL_BROADCAST = 0, 1
SHM_TEAM_SYNC_OFF, SHM_TEAM_SYNC_FULL, SHM_TEAM_SYNC_TRACKED = 0, 1, 2
(SHM_SYNC_WAIT, SHM_SYNC_WAIT_ALL, SHM_SYNC_WAIT_ANY, SHM_SYNC_WAIT_SOME,
 SHM_SYNC_TEST, SHM_SYNC_TEST_ALL, SHM_SYNC_TEST_ANY, SHM_SYNC_TEST_SOME) = range(8)
SHM_NO_CONSUME = (1 << 64) - 1
SHM_CUTOVER_TUNED = (1 << 64) - 2
SHM_OP_MIN, SHM_OP_MAX, SHM_OP_SUM, SHM_OP_PROD, SHM_OP_AND, SHM_OP_OR, SHM_OP_XOR = range(7)
(SHM_INT8, SHM_UINT8, SHM_INT16, SHM_UINT16, SHM_INT32, SHM_UINT32, SHM_INT64, SHM_UINT64, SHM_FLOAT32,
 SHM_FLOAT64) = range(10)

_ERR_NAMES = {SHM_EINVAL: "SHM_EINVAL", SHM_EPE: "SHM_EPE", SHM_ERANGE: "SHM_ERANGE", SHM_ENOMEM: "SHM_ENOMEM",
              SHM_EHIP: "SHM_EHIP", SHM_ETIMEOUT: "SHM_ETIMEOUT", SHM_ENODEV: "SHM_ENODEV"}

# name -> (restype, argtypes); mirrors include/shm355.h one to one
_u64p, _szp, _ip = POINTER(c_uint64), POINTER(c_size_t), POINTER(c_int)
PROTOTYPES = {
    "shm_init": (c_int, [c_int, c_size_t, c_void_p, POINTER(c_void_p), POINTER(c_void_p)]),
    "shm_init_ex": (c_int, [c_int, c_size_t, c_void_p, POINTER(c_void_p), c_uint, POINTER(c_void_p)]),
    "shm_finalize": (c_int, [c_void_p]),
    "shm_n_pes": (c_int, [c_void_p]),
    "shm_heap_bytes": (c_size_t, [c_void_p]),
    "shm_last_error": (c_char_p, []),
    "shm_malloc": (c_int, [c_void_p, c_size_t, c_size_t, _u64p]),
    "shm_calloc": (c_int, [c_void_p, c_size_t, c_size_t, _u64p]),
    "shm_free": (c_int, [c_void_p, c_uint64]),
    "shm_ptr": (c_void_p, [c_void_p, c_uint64, c_int]),
    "shm_write": (c_int, [c_void_p, c_int, c_uint64, c_void_p, c_size_t]),
    "shm_read": (c_int, [c_void_p, c_int, c_uint64, c_void_p, c_size_t]),
    "shm_putmem": (c_int, [c_void_p, c_int, c_uint64, c_uint64, c_size_t, c_int]),
    "shm_getmem": (c_int, [c_void_p, c_int, c_uint64, c_uint64, c_size_t, c_int]),
    "shm_quiet": (c_int, [c_void_p, c_int]),
    "shm_fence": (c_int, [c_void_p, c_int]),
    "shm_barrier_all": (c_int, [c_void_p]),
    "shm_set_cutover": (c_int, [c_void_p, c_int, c_size_t]),
    "shm_get_cutover": (c_int, [c_void_p, c_int, _szp]),
    "shm_choose_path": (c_int, [c_void_p, c_size_t, c_int, _ip]),
    "shm_device_context_bytes": (c_size_t, []),
    "shm_device_context": (c_int, [c_void_p, c_void_p, c_size_t]),
    "shm_stream": (c_void_p, [c_void_p, c_int]),
    "shm_stream_used": (c_int, [c_void_p, c_int]),
    "shm_set_collective_cutover": (c_int, [c_void_p, c_int, c_int, c_size_t]),
    "shm_get_collective_cutover": (c_int, [c_void_p, c_int, c_int, _szp]),
    "shm_choose_collective_path": (c_int, [c_void_p, c_int, c_size_t, c_int, _ip]),
    "shm_set_wait_timeout_us": (c_int, [c_void_p, c_uint64]),
    "shm_set_team_sync": (c_int, [c_void_p, c_int]),
    "shm_launch_wg_put": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int]),
    "shm_launch_wg_get": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int]),
    "shm_launch_wg_put_all": (c_int, [c_void_p, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int]),
    "shm_launch_wg_get_all": (c_int, [c_void_p, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int]),
    "shm_launch_wg_put_timed": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int, c_void_p]),
    "shm_wall_clock_khz": (c_int, [c_void_p]),
    "shm_launch_stream_probe": (c_int, [c_void_p, c_int, c_uint64, c_uint64, c_size_t, c_int]),
    "shm_proxy_start": (c_int, [c_void_p]),
    "shm_proxy_stop": (c_int, [c_void_p]),
    "shm_proxy_stats": (c_int, [c_void_p, _u64p, _u64p]),
    "shm_launch_put_device_initiated": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int, c_int, c_size_t, c_int, c_void_p]),
    "shm_launch_rma_device_initiated": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int, c_int, c_int, c_size_t,
                                                c_size_t, c_uint64, c_int, c_void_p]),
    "shm_launch_scalar_pg": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int, c_int]),
    "shm_launch_wave_exchange": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_uint64, c_size_t, c_int, c_uint64, c_uint64]),
    "shm_launch_thread_rma": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_size_t, c_int, c_int, c_void_p]),
    "shm_launch_iput": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_int64, c_int64, c_size_t, c_int, c_int]),
    "shm_launch_iget": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_int64, c_int64, c_size_t, c_int, c_int]),
    "shm_launch_offload_nop": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_void_p]),
    "shm_launch_wg_put_signal": (c_int, [c_void_p, c_int, c_int, c_uint64, c_uint64, c_size_t, c_uint64, c_uint64, c_int, c_int]),
    "shm_launch_signal_wait_until": (c_int, [c_void_p, c_int, c_uint64, c_int, c_uint64, c_void_p]),
    "shm_launch_sync_set": (c_int, [c_void_p, c_int, c_uint64, c_size_t, c_void_p, c_int, c_int, c_int64, c_void_p]),
    "shm_launch_amo": (c_int, [c_void_p, c_int, c_int, c_uint64, c_int, c_int64, c_int64, c_void_p]),
    "shm_launch_pingflag": (c_int, [c_void_p, c_uint64, c_uint64, c_size_t, c_uint64]),
    "shm_launch_ring_pipeline": (c_int, [c_void_p, c_uint64, c_uint64, c_uint64, c_uint64, c_size_t, c_int, c_int, c_int, c_int]),
    "shm_launch_ring_pipeline_static": (c_int, [c_void_p, c_uint64, c_uint64, c_uint64, c_uint64, c_size_t, c_int, c_int, c_int, c_int]),
    "shm_launch_amo_storm": (c_int, [c_void_p, c_uint64, c_int, c_void_p, c_uint64, c_int, c_int, c_void_p, c_void_p]),
    "shm_launch_fcollect": (c_int, [c_void_p, c_uint64, c_uint64, c_size_t, c_int, c_int]),
    "shm_launch_collect": (c_int, [c_void_p, c_uint64, c_uint64, POINTER(c_size_t), c_int]),
    "shm_launch_reduce": (c_int, [c_void_p, c_uint64, c_uint64, c_size_t, c_int, c_int, c_int, c_int]),
    "shm_launch_broadcast": (c_int, [c_void_p, c_uint64, c_uint64, c_size_t, c_int, c_int, c_int]),
    "shm_launch_sync_all": (c_int, [c_void_p, c_int, c_int, c_void_p]),
    "shm_launch_barrier_exchange": (c_int, [c_void_p, c_uint64, c_uint64, c_uint64, c_size_t, c_int]),
    "shm_launch_reduce_sum_f32": (c_int, [c_void_p, c_uint64, c_uint64, c_size_t, c_int, c_int]),
}

_lib = None


class ShmError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{_ERR_NAMES.get(code, code)}: {text}")
        self.code = code


def load_library() -> ctypes.CDLL:
    """Load libshm355.so from the package directory.  No library, no product: raises.

    A process should hold ONE HIP runtime.  PyTorch brings its own copy; a program that uses both
    imports torch (and touches the GPU) before the first context is made, as Shm.on_torch does, so
    that the library binds to the runtime already in the process."""
    global _lib
    if _lib is None:
        path = _LIB_PATH
        if os.environ.get("SHM355_LIBRARY_VARIANT"):      # e.g. "full_release": the cross-check build
            path = _LIB_PATH[:-3] + "_" + os.environ["SHM355_LIBRARY_VARIANT"] + ".so"
        if not os.path.exists(path):
            raise ImportError(f"{path} has not been built; run `python -m paper_2409_20476_amd.build` "
                              "(there is no CPU fallback)")
        lib = ctypes.CDLL(path)
        for name, (res, args) in PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _ptr(x) -> int:
    """Device pointer from an int, None, or anything with data_ptr() (a torch tensor)."""
    if x is None:
        return 0
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


class Shm:
    """One shm355 context.  Method names are the C entry points without the ``shm_`` prefix."""

    def __init__(self, npes: int, heap_bytes: int, heap_base=None, streams=None, flags: int = SHM_INIT_DEFAULT):
        self.lib = load_library()
        self._keep = (heap_base, streams)           # borrowed by the library: keep them alive
        arr = None
        if streams is not None:
            handles = [s.cuda_stream if hasattr(s, "cuda_stream") else int(s) for s in streams]
            arr = (c_void_p * len(handles))(*handles)
        ctx = c_void_p()
        self.ctx = None
        self._check(self.lib.shm_init_ex(npes, heap_bytes, _ptr(heap_base), arr, flags, byref(ctx)))
        self.ctx = ctx
        self.npes = npes

    @classmethod
    def on_torch(cls, npes: int, heap_bytes: int) -> "Shm":
        """Heap and streams come from PyTorch (device memory and streams are all it is used for)."""
        import torch
        heap = torch.empty(npes * heap_bytes, dtype=torch.uint8, device="cuda")
        streams = [torch.cuda.Stream() for _ in range(npes)]
        torch.cuda.synchronize()
        obj = cls(npes, heap_bytes, heap, streams)
        obj.heap_tensor, obj.streams = heap, streams
        return obj

    def _check(self, rc: int) -> int:
        if rc < 0:
            raise ShmError(rc, self.lib.shm_last_error().decode())
        return rc

    # ---- set-up -------------------------------------------------------------------------
    def finalize(self):
        if self.ctx is not None:
            ctx, self.ctx = self.ctx, None
            self._check(self.lib.shm_finalize(ctx))

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.finalize()

    def n_pes(self) -> int:
        return self._check(self.lib.shm_n_pes(self.ctx))

    def heap_bytes(self) -> int:
        return self.lib.shm_heap_bytes(self.ctx)

    def malloc(self, nbytes: int, align: int = 0) -> int:
        off = c_uint64()
        self._check(self.lib.shm_malloc(self.ctx, nbytes, align, byref(off)))
        return off.value

    def calloc(self, nbytes: int, align: int = 0) -> int:
        off = c_uint64()
        self._check(self.lib.shm_calloc(self.ctx, nbytes, align, byref(off)))
        return off.value

    def free(self, off: int):
        self._check(self.lib.shm_free(self.ctx, off))

    def ptr(self, off: int, pe: int) -> int:
        return self.lib.shm_ptr(self.ctx, off, pe) or 0

    def write(self, pe: int, off: int, data):
        buf = np.ascontiguousarray(data)
        self._check(self.lib.shm_write(self.ctx, pe, off, buf.ctypes.data_as(c_void_p), buf.nbytes))

    def read(self, pe: int, off: int, nbytes: int, dtype=np.uint8) -> np.ndarray:
        out = np.empty(nbytes, dtype=np.uint8)
        self._check(self.lib.shm_read(self.ctx, pe, off, out.ctypes.data_as(c_void_p), nbytes))
        return out.view(dtype)

    # ---- host RMA and ordering ----------------------------------------------------------
    def putmem(self, me, dst_off, src_off, n, pe):
        self._check(self.lib.shm_putmem(self.ctx, me, dst_off, src_off, n, pe))

    def getmem(self, me, dst_off, src_off, n, pe):
        self._check(self.lib.shm_getmem(self.ctx, me, dst_off, src_off, n, pe))

    def quiet(self, me):
        self._check(self.lib.shm_quiet(self.ctx, me))

    def fence(self, me):
        self._check(self.lib.shm_fence(self.ctx, me))

    def barrier_all(self):
        self._check(self.lib.shm_barrier_all(self.ctx))

    # ---- kernels of the caller's own ------------------------------------------------------
    def device_context(self) -> bytes:
        """The by-value device view (a shm_dev_ctx) that kernels built against shm_device.hpp take."""
        n = self.lib.shm_device_context_bytes()
        buf = ctypes.create_string_buffer(n)
        self._check(self.lib.shm_device_context(self.ctx, buf, n))
        return buf.raw

    def stream(self, pe: int) -> int:
        """PE pe's hipStream_t as an integer (0 on error)."""
        return self.lib.shm_stream(self.ctx, pe) or 0

    def stream_used(self, pe: int):
        """Tell the tracked team sync that work of the caller's own is about to go onto PE pe's stream."""
        self._check(self.lib.shm_stream_used(self.ctx, pe))

    # ---- policy ---------------------------------------------------------------------------
    def set_cutover(self, n_wg: int, nbytes: int):
        self._check(self.lib.shm_set_cutover(self.ctx, n_wg, nbytes))

    def get_cutover(self, n_wg: int) -> int:
        v = c_size_t()
        self._check(self.lib.shm_get_cutover(self.ctx, n_wg, byref(v)))
        return v.value

    def set_collective_cutover(self, collective: int, n_wg: int, nbytes: int):
        self._check(self.lib.shm_set_collective_cutover(self.ctx, collective, n_wg, nbytes))

    def get_collective_cutover(self, collective: int, n_wg: int) -> int:
        v = c_size_t()
        self._check(self.lib.shm_get_collective_cutover(self.ctx, collective, n_wg, byref(v)))
        return v.value

    def choose_collective_path(self, collective: int, bytes_per_pe: int, n_wg: int) -> int:
        v = c_int()
        self._check(self.lib.shm_choose_collective_path(self.ctx, collective, bytes_per_pe, n_wg, byref(v)))
        return v.value

    def choose_path(self, n: int, n_wg: int) -> int:
        v = c_int()
        self._check(self.lib.shm_choose_path(self.ctx, n, n_wg, byref(v)))
        return v.value

    def set_wait_timeout_us(self, us: int):
        self._check(self.lib.shm_set_wait_timeout_us(self.ctx, us))

    def set_team_sync(self, mode):
        """False / SHM_TEAM_SYNC_OFF, True / SHM_TEAM_SYNC_FULL or SHM_TEAM_SYNC_TRACKED."""
        self._check(self.lib.shm_set_team_sync(self.ctx, int(mode)))

    # ---- kernel launches --------------------------------------------------------------------
    def launch_wg_put(self, me, pe, dst_off, src_off, n, n_wg=1, path=SHM_PATH_LDST):
        self._check(self.lib.shm_launch_wg_put(self.ctx, me, pe, dst_off, src_off, n, n_wg, path))

    def launch_wg_get(self, me, pe, dst_off, src_off, n, n_wg=1, path=SHM_PATH_LDST):
        self._check(self.lib.shm_launch_wg_get(self.ctx, me, pe, dst_off, src_off, n, n_wg, path))

    def launch_wg_put_all(self, pe_shift, dst_off, src_off, n, n_wg=1, path=SHM_PATH_LDST):
        self._check(self.lib.shm_launch_wg_put_all(self.ctx, pe_shift, dst_off, src_off, n, n_wg, path))

    def launch_wg_get_all(self, pe_shift, dst_off, src_off, n, n_wg=1, path=SHM_PATH_LDST):
        self._check(self.lib.shm_launch_wg_get_all(self.ctx, pe_shift, dst_off, src_off, n, n_wg, path))

    def launch_wg_put_timed(self, me, pe, dst_off, src_off, n, n_wg, reps, dev_ticks):
        self._check(self.lib.shm_launch_wg_put_timed(self.ctx, me, pe, dst_off, src_off, n, n_wg, reps, _ptr(dev_ticks)))

    def launch_stream_probe(self, kind, dst_off, src_off, n, n_wg):
        self._check(self.lib.shm_launch_stream_probe(self.ctx, kind, dst_off, src_off, n, n_wg))

    def wall_clock_khz(self) -> int:
        return self._check(self.lib.shm_wall_clock_khz(self.ctx))

    def proxy_start(self):
        self._check(self.lib.shm_proxy_start(self.ctx))

    def proxy_stop(self):
        self._check(self.lib.shm_proxy_stop(self.ctx))

    def proxy_stats(self):
        r, c = c_uint64(), c_uint64()
        self._check(self.lib.shm_proxy_stats(self.ctx, byref(r), byref(c)))
        return r.value, c.value

    def launch_put_device_initiated(self, me, pe, dst_off, src_off, n, n_wg, mode, cutover, reps, dev_ticks, wg_size=256):
        self._check(self.lib.shm_launch_put_device_initiated(self.ctx, me, pe, dst_off, src_off, n, n_wg, wg_size, mode, cutover,
                                                             reps, _ptr(dev_ticks)))

    def launch_rma_device_initiated(self, me, pe, dst_off, src_off, n, n_wg, is_get, mode, cutover=0, cover=0,
                                    consume_off=SHM_NO_CONSUME, reps=1, dev_ticks=None, wg_size=256):
        self._check(self.lib.shm_launch_rma_device_initiated(self.ctx, me, pe, dst_off, src_off, n, n_wg, wg_size, int(is_get), mode,
                                                             cutover, cover, consume_off, reps, _ptr(dev_ticks)))

    def launch_scalar_pg(self, me, pe, dst_off, src_off, nelems, elem_bytes, is_get=False, n_wg=1):
        self._check(self.lib.shm_launch_scalar_pg(self.ctx, me, pe, dst_off, src_off, nelems, elem_bytes, int(is_get), n_wg))

    def launch_wave_exchange(self, me, pe, dst_off, src_off, back_off, n, n_waves, flag_off, out_off):
        self._check(self.lib.shm_launch_wave_exchange(self.ctx, me, pe, dst_off, src_off, back_off, n, n_waves, flag_off, out_off))

    def launch_thread_rma(self, me, pe, dst_off, src_off, n, is_get=False, reps=1, dev_ticks=None):
        self._check(self.lib.shm_launch_thread_rma(self.ctx, me, pe, dst_off, src_off, n, int(is_get), reps, _ptr(dev_ticks)))

    def launch_iput(self, me, pe, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, n_wg=0):
        self._check(self.lib.shm_launch_iput(self.ctx, me, pe, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, n_wg))

    def launch_iget(self, me, pe, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, n_wg=0):
        self._check(self.lib.shm_launch_iget(self.ctx, me, pe, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, n_wg))

    def launch_offload_nop(self, me, n_wg, reps, blocking, dev_ticks):
        self._check(self.lib.shm_launch_offload_nop(self.ctx, me, n_wg, reps, int(blocking), _ptr(dev_ticks)))

    def launch_wg_put_signal(self, me, pe, dst_off, src_off, n, sig_off, sig_val, sig_op, n_wg=1):
        self._check(self.lib.shm_launch_wg_put_signal(self.ctx, me, pe, dst_off, src_off, n, sig_off, sig_val, sig_op, n_wg))

    def launch_signal_wait_until(self, me, sig_off, cmp, val, dev_out=None):
        self._check(self.lib.shm_launch_signal_wait_until(self.ctx, me, sig_off, cmp, val, _ptr(dev_out)))

    def launch_sync_set(self, me, ivars_off, nelems, dev_status, kind, cmp, val, dev_out):
        self._check(self.lib.shm_launch_sync_set(self.ctx, me, ivars_off, nelems, _ptr(dev_status), kind, cmp, val, _ptr(dev_out)))

    def launch_amo(self, me, pe, off, op, operand=0, cond=0, dev_out=None):
        self._check(self.lib.shm_launch_amo(self.ctx, me, pe, off, op, operand, cond, _ptr(dev_out)))

    def launch_pingflag(self, data_off, back_off, n, flag_off):
        self._check(self.lib.shm_launch_pingflag(self.ctx, data_off, back_off, n, flag_off))

    def launch_ring_pipeline_static(self, src_off, slot_off, sig_off, acc_off, chunk_bytes, n_chunks, n_wg_prod, n_wg_cons, n_sig=1):
        self._check(self.lib.shm_launch_ring_pipeline_static(self.ctx, src_off, slot_off, sig_off, acc_off, chunk_bytes, n_chunks,
                                                             n_wg_prod, n_wg_cons, n_sig))

    def launch_ring_pipeline(self, src_off, slot_off, sig_off, acc_off, chunk_bytes, n_chunks, n_wg_prod, n_wg_cons, n_sig=1):
        self._check(self.lib.shm_launch_ring_pipeline(self.ctx, src_off, slot_off, sig_off, acc_off, chunk_bytes, n_chunks,
                                                      n_wg_prod, n_wg_cons, n_sig))

    def launch_amo_storm(self, ctr_off, n_ctr, dev_targets, n_items, ops_per_item, kind=SHM_STORM_FETCH_ADD,
                         dev_fetched=None, dev_checksum=None):
        self._check(self.lib.shm_launch_amo_storm(self.ctx, ctr_off, n_ctr, _ptr(dev_targets), n_items, ops_per_item, kind,
                                                  _ptr(dev_fetched), _ptr(dev_checksum)))

    def launch_fcollect(self, dst_off, src_off, bytes_per_pe, n_wg=64, path=SHM_PATH_LDST):
        self._check(self.lib.shm_launch_fcollect(self.ctx, dst_off, src_off, bytes_per_pe, n_wg, path))

    def launch_collect(self, dst_off, src_off, nbytes_per_pe, n_wg=8):
        sizes = (c_size_t * len(nbytes_per_pe))(*nbytes_per_pe)
        if len(nbytes_per_pe) != self.n_pes():
            raise ValueError("one size per PE")
        self._check(self.lib.shm_launch_collect(self.ctx, dst_off, src_off, sizes, n_wg))

    def launch_reduce(self, dst_off, src_off, nelems, dtype, op, n_wg=64, algo=SHM_REDUCE_DUPLICATE):
        self._check(self.lib.shm_launch_reduce(self.ctx, dst_off, src_off, nelems, dtype, op, n_wg, algo))

    def launch_broadcast(self, dst_off, src_off, n, root, n_wg=64, path=SHM_PATH_LDST):
        self._check(self.lib.shm_launch_broadcast(self.ctx, dst_off, src_off, n, root, n_wg, path))

    def launch_sync_all(self, rounds, with_quiet, dev_ticks):
        self._check(self.lib.shm_launch_sync_all(self.ctx, rounds, int(with_quiet), _ptr(dev_ticks)))

    def launch_barrier_exchange(self, dst_off, src_off, acc_off, n, rounds):
        self._check(self.lib.shm_launch_barrier_exchange(self.ctx, dst_off, src_off, acc_off, n, rounds))

    def launch_reduce_sum_f32(self, dst_off, src_off, nelems, n_wg=64, algo=SHM_REDUCE_DUPLICATE):
        self._check(self.lib.shm_launch_reduce_sum_f32(self.ctx, dst_off, src_off, nelems, n_wg, algo))
