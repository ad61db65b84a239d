"""Sequential CPU model of a symmetric heap and the OpenSHMEM operations built on it.

TEST INFRASTRUCTURE ONLY.  This module is the correctness oracle for the GPU
library.  It is imported by the tests, by the smoke check and by the benchmark's
CPU-baseline leg, and by nothing else; it shares no code with the GPU path and
never calls it.  It is deliberately plain and slow.

What is modelled, and the passage each part follows
---------------------------------------------------
* PGAS state (paper section "OpenSHMEM Memory and Execution Model"): ``npes``
  processing elements numbered ``0 .. npes-1``; every PE owns one symmetric heap
  of the same size with the same layout, so one byte offset names "the same
  object" on every PE while the stored values may differ from PE to PE.
* Address rule (paper section "Remote Memory Access", the scalar-put example):
  the remote location of a symmetric object is the local address minus the
  local heap base plus the remote heap base.  With one flat array per PE that
  is simply "same offset, other array"; ``translate`` writes the rule out with
  explicit base addresses so that the tests can pin it.
* Work-group put/get (paper section "Proposed Device APIs"): the threads of a
  group share one copy, each taking a piece of it.  The result is the byte
  copy itself; which thread moved which byte is not observable.  ``wg_put``
  and ``wg_get`` walk the message slice by slice only so that the slicing rule
  used for several work-groups per message can be checked to cover the message
  exactly once.
* Signalling, ordering, atomics: the paper only says these follow OpenSHMEM 1.5,
  so the 1.5 rules are used: ``put_signal`` updates a 64-bit unsigned signal
  word on the target *after* the payload; ``signal_wait_until`` compares
  unsigned; ``quiet``/``fence`` change no state in a model where every operation
  completes at once; atomics are indivisible 64-bit read-modify-writes.
* Point-to-point synchronisation (OpenSHMEM 1.5 wait_until / test with their all, any and some
  forms; the paper lists these routines as callable from the device): SIGNED comparison of 64-bit
  variables of the caller's own heap; where several answers are correct (which index ``any``
  returns) the model returns the set of correct answers.
* Push collect (paper section "Collective Operations", sync-and-broadcast
  paragraph) and the duplicated reduction (same section, reduction paragraph):
  ``fcollect`` concatenates every PE's block in PE order into every PE's
  destination; ``reduce_sum_f32`` folds the PEs' vectors element-wise in PE
  order 0, 1, ..., npes-1 in binary32 and every PE receives the same result.
* The pipelined ring (a benchmark configuration, not a paper algorithm): chunks
  travel with put-with-signal (ADD 1) to the next PE, the receiver waits for
  chunk k by ``signal >= k+1`` and adds the bf16 payload, widened exactly to
  binary32, into a binary32 accumulator in chunk order.

Semantics of time: operations are applied one after another in the order the
caller issues them and each takes full effect before the next starts.  A
``signal_wait_until`` whose condition is false at that point cannot be satisfied
by a sequential schedule, so it raises instead of blocking.

Readings taken where the paper is silent are listed in the repository's design
notes; the ones that matter here: overlapping source and destination on one PE
is an error; signal and atomic targets must be 8-byte aligned; ``put_signal``
with zero bytes still updates the signal; the signal word may not lie inside the
destination (OpenSHMEM 1.5, put-with-signal); a PE may target itself.

Parity status: every function here is pinned by the CPU tests (brute force on
tiny heaps against an independent byte-at-a-time model, closed forms, library
routines and hand-worked fixtures) except the allocator's *placement*, which is
free by design (only invariants are checked) -- "parity unpinned" for offsets.
"""
from __future__ import annotations

import numpy as np

U64_MASK = (1 << 64) - 1

SIGNAL_SET = 0
SIGNAL_ADD = 1

CMP_EQ, CMP_NE, CMP_GT, CMP_GE, CMP_LT, CMP_LE = range(6)

_CMP = {
    CMP_EQ: lambda a, b: a == b,
    CMP_NE: lambda a, b: a != b,
    CMP_GT: lambda a, b: a > b,
    CMP_GE: lambda a, b: a >= b,
    CMP_LT: lambda a, b: a < b,
    CMP_LE: lambda a, b: a <= b,
}


class OracleError(Exception):
    """An operation the OpenSHMEM rules do not define, or an illegal schedule."""


def _to_i64(x: int) -> int:
    """Two's-complement wrap of a Python int into the int64 range."""
    x &= U64_MASK
    return x - (1 << 64) if x >> 63 else x


class ShmemOracle:
    """``npes`` byte-array heaps plus the OpenSHMEM operations acting on them."""

    DEFAULT_ALIGN = 256

    def __init__(self, npes: int, heap_bytes: int):
        if npes < 1 or heap_bytes < 1:
            raise OracleError("need npes >= 1 and heap_bytes >= 1")
        self.npes = int(npes)
        self.heap_bytes = int(heap_bytes)
        self.heap = [np.zeros(self.heap_bytes, dtype=np.uint8) for _ in range(self.npes)]
        # allocator state: sorted list of (offset, size) of live blocks
        self._live: list[tuple[int, int]] = []
        self.log: list[tuple] = []  # ordering operations, in issue order

    # ------------------------------------------------------------------ checks
    def _pe(self, pe: int) -> int:
        if not (0 <= pe < self.npes):
            raise OracleError(f"PE {pe} outside 0..{self.npes - 1}")
        return pe

    def _range(self, off: int, n: int) -> None:
        if off < 0 or n < 0 or off + n > self.heap_bytes:
            raise OracleError(f"[{off}, {off}+{n}) leaves the heap of {self.heap_bytes} bytes")

    def _word(self, off: int) -> None:
        self._range(off, 8)
        if off % 8:
            raise OracleError("64-bit signal/atomic target must be 8-byte aligned")

    # --------------------------------------------------------------- allocator
    def malloc(self, nbytes: int, align: int = 0) -> int:
        """Lowest-address first fit.  One offset, valid on every PE."""
        align = align or self.DEFAULT_ALIGN
        if align & (align - 1):
            raise OracleError("alignment must be a power of two")
        if nbytes == 0:
            return U64_MASK
        cur = 0
        for o, s in self._live:
            start = -(-cur // align) * align
            if start + nbytes <= o:
                break
            cur = o + s
        start = -(-cur // align) * align
        if start + nbytes > self.heap_bytes:
            raise OracleError("symmetric heap exhausted")
        self._live.append((start, nbytes))
        self._live.sort()
        return start

    def calloc(self, nbytes: int, align: int = 0) -> int:
        off = self.malloc(nbytes, align)
        if nbytes:
            for p in range(self.npes):
                self.heap[p][off:off + nbytes] = 0
        return off

    def free(self, off: int) -> None:
        if off == U64_MASK:
            return
        for i, (o, _) in enumerate(self._live):
            if o == off:
                del self._live[i]
                return
        raise OracleError(f"free of offset {off} that is not a live block")

    # ---------------------------------------------------------------- staging
    def write(self, pe: int, off: int, data) -> None:
        buf = np.frombuffer(np.ascontiguousarray(data).tobytes(), dtype=np.uint8)
        self._pe(pe)
        self._range(off, buf.size)
        self.heap[pe][off:off + buf.size] = buf

    def read(self, pe: int, off: int, n: int, dtype=np.uint8) -> np.ndarray:
        self._pe(pe)
        self._range(off, n)
        return self.heap[pe][off:off + n].copy().view(dtype)

    # ------------------------------------------------------ address translation
    @staticmethod
    def translate(local_addr: int, local_heap_base: int, remote_heap_base: int) -> int:
        """Remote address of a symmetric object: local - local base + remote base."""
        return local_addr - local_heap_base + remote_heap_base

    # --------------------------------------------------------------------- RMA
    def putmem(self, me: int, dst: int, src: int, n: int, pe: int) -> None:
        """Bytes [src, src+n) of PE ``me`` become bytes [dst, dst+n) of PE ``pe``."""
        self._pe(me), self._pe(pe)
        self._range(src, n), self._range(dst, n)
        if me == pe and n and src < dst + n and dst < src + n:
            raise OracleError("overlapping source and destination on one PE")
        self.heap[pe][dst:dst + n] = self.heap[me][src:src + n].copy()

    def getmem(self, me: int, dst: int, src: int, n: int, pe: int) -> None:
        """Bytes [src, src+n) of PE ``pe`` become bytes [dst, dst+n) of PE ``me``."""
        self._pe(me), self._pe(pe)
        self._range(src, n), self._range(dst, n)
        if me == pe and n and src < dst + n and dst < src + n:
            raise OracleError("overlapping source and destination on one PE")
        self.heap[me][dst:dst + n] = self.heap[pe][src:src + n].copy()

    def _strided(self, me, pe, dst, src, dst_stride, src_stride, nelems, elem_bytes):
        self._pe(me), self._pe(pe)
        if elem_bytes not in (1, 2, 4, 8, 16):
            raise OracleError("element size must be 1, 2, 4, 8 or 16 bytes")
        if dst_stride < 1 or src_stride < 1:
            raise OracleError("strides are counted in elements and are at least 1")
        if dst % elem_bytes or src % elem_bytes:
            raise OracleError("strided transfers need element-aligned addresses")
        dspan = ((nelems - 1) * dst_stride + 1) * elem_bytes if nelems else 0
        sspan = ((nelems - 1) * src_stride + 1) * elem_bytes if nelems else 0
        self._range(src, sspan), self._range(dst, dspan)
        if me == pe and nelems and src < dst + dspan and dst < src + sspan:
            raise OracleError("overlapping source and destination on one PE")

    def iput(self, me: int, dst: int, src: int, dst_stride: int, src_stride: int, nelems: int, elem_bytes: int,
             pe: int) -> None:
        """Strided put (paper section "Implementation", blocked and strided RMA; OpenSHMEM iput):
        element i of the source, taken every ``src_stride`` elements on PE ``me``, becomes element
        i of the destination, placed every ``dst_stride`` elements on PE ``pe``.  Bytes between the
        destination elements are not touched."""
        self._strided(me, pe, dst, src, dst_stride, src_stride, nelems, elem_bytes)
        picked = [self.heap[me][src + i * src_stride * elem_bytes: src + i * src_stride * elem_bytes + elem_bytes].copy()
                  for i in range(nelems)]
        for i in range(nelems):
            at = dst + i * dst_stride * elem_bytes
            self.heap[pe][at:at + elem_bytes] = picked[i]

    def iget(self, me: int, dst: int, src: int, dst_stride: int, src_stride: int, nelems: int, elem_bytes: int,
             pe: int) -> None:
        """Strided get: as iput with the roles exchanged -- the source is on PE ``pe``, the
        destination on the calling PE ``me``."""
        self._strided(pe, me, dst, src, dst_stride, src_stride, nelems, elem_bytes)
        picked = [self.heap[pe][src + i * src_stride * elem_bytes: src + i * src_stride * elem_bytes + elem_bytes].copy()
                  for i in range(nelems)]
        for i in range(nelems):
            at = dst + i * dst_stride * elem_bytes
            self.heap[me][at:at + elem_bytes] = picked[i]

    @staticmethod
    def wg_slices(n: int, n_wg: int) -> list[tuple[int, int]]:
        """How ``n_wg`` work-groups share one message of ``n`` bytes.

        Every group takes one contiguous slice whose length is n / n_wg rounded
        up to a whole number of 16-byte units; late groups may get a short or an
        empty slice.  Returns ``(begin, end)`` per group.
        """
        if n_wg < 1:
            raise OracleError("need at least one work-group")
        per = -(-n // n_wg)
        per = -(-per // 16) * 16
        out = []
        for g in range(n_wg):
            lo = min(n, g * per)
            hi = min(n, lo + per)
            out.append((lo, hi))
        return out

    def wg_put(self, me: int, dst: int, src: int, n: int, pe: int, n_wg: int = 1) -> None:
        """Work-group put: each group copies its slice; together they copy the message."""
        self._pe(me), self._pe(pe)
        self._range(src, n), self._range(dst, n)
        if me == pe and n and src < dst + n and dst < src + n:
            raise OracleError("overlapping source and destination on one PE")
        for lo, hi in self.wg_slices(n, n_wg):
            self.heap[pe][dst + lo:dst + hi] = self.heap[me][src + lo:src + hi].copy()

    def wg_get(self, me: int, dst: int, src: int, n: int, pe: int, n_wg: int = 1) -> None:
        self._pe(me), self._pe(pe)
        self._range(src, n), self._range(dst, n)
        if me == pe and n and src < dst + n and dst < src + n:
            raise OracleError("overlapping source and destination on one PE")
        for lo, hi in self.wg_slices(n, n_wg):
            self.heap[me][dst + lo:dst + hi] = self.heap[pe][src + lo:src + hi].copy()

    # ----------------------------------------------------------------- signals
    def _load_u64(self, pe: int, off: int) -> int:
        return int.from_bytes(self.heap[pe][off:off + 8].tobytes(), "little")

    def _store_u64(self, pe: int, off: int, v: int) -> None:
        self.heap[pe][off:off + 8] = np.frombuffer((v & U64_MASK).to_bytes(8, "little"), dtype=np.uint8)

    def put_signal(self, me: int, dst: int, src: int, n: int, sig: int, value: int, op: int, pe: int,
                   n_wg: int = 1) -> None:
        """Payload first, then the signal word on the target PE (SET or ADD mod 2^64)."""
        self._pe(pe)
        self._word(sig)
        if op not in (SIGNAL_SET, SIGNAL_ADD):
            raise OracleError("signal operation must be SET or ADD")
        if n and sig < dst + n and dst < sig + 8:
            # OpenSHMEM 1.5, put-with-signal: destination and signal word may not overlap
            raise OracleError("the signal word lies inside the destination")
        self.wg_put(me, dst, src, n, pe, n_wg)
        if op == SIGNAL_SET:
            self._store_u64(pe, sig, value)
        else:
            self._store_u64(pe, sig, self._load_u64(pe, sig) + value)

    def signal_fetch(self, me: int, sig: int) -> int:
        self._pe(me)
        self._word(sig)
        return self._load_u64(me, sig)

    def signal_wait_until(self, me: int, sig: int, cmp: int, value: int) -> int:
        """Unsigned comparison of the local signal word; returns the satisfying value."""
        self._pe(me)
        self._word(sig)
        if cmp not in _CMP:
            raise OracleError("unknown comparison")
        cur = self._load_u64(me, sig)
        if not _CMP[cmp](cur, value & U64_MASK):
            raise OracleError(
                f"wait on PE {me} (signal={cur}, cmp={cmp}, value={value}) can never be satisfied "
                "in this sequential order")
        return cur

    # ------------------------------------------------- point-to-point synchronisation
    def _ivars(self, me: int, off: int, nelems: int, status) -> list:
        """(index, value) of every selected 64-bit signed variable of PE ``me`` (OpenSHMEM 1.5 wait/test
        sets: a nonzero status entry takes the variable out of the set)."""
        self._pe(me)
        if nelems < 0 or off % 8:
            raise OracleError("variables are 8-byte aligned and their number is not negative")
        self._range(off, 8 * nelems)
        if status is not None and len(status) != nelems:
            raise OracleError("one status entry per variable")
        return [(i, self._load_i64(me, off + 8 * i)) for i in range(nelems) if status is None or not status[i]]

    def test_some(self, me: int, off: int, nelems: int, status, cmp: int, value: int) -> list:
        """Indices of the selected variables for which ``cmp(variable, value)`` holds now; SIGNED comparison."""
        if cmp not in _CMP:
            raise OracleError("unknown comparison")
        return [i for i, v in self._ivars(me, off, nelems, status) if _CMP[cmp](v, _to_i64(value))]

    def test_all(self, me: int, off: int, nelems: int, status, cmp: int, value: int) -> bool:
        """True if every selected variable satisfies the comparison (trivially for an empty set)."""
        return len(self.test_some(me, off, nelems, status, cmp, value)) == len(self._ivars(me, off, nelems, status))

    def test_any(self, me: int, off: int, nelems: int, status, cmp: int, value: int) -> list:
        """The indices any of which a correct test_any may return (empty: it returns 'none')."""
        return self.test_some(me, off, nelems, status, cmp, value)

    def test(self, me: int, off: int, cmp: int, value: int) -> bool:
        return bool(self.test_some(me, off, 1, None, cmp, value))

    def wait_until(self, me: int, off: int, cmp: int, value: int) -> int:
        """Returns the satisfying value; a wait that nothing in this sequential order can satisfy raises."""
        if not self.test(me, off, cmp, value):
            raise OracleError("wait_until can never be satisfied in this sequential order")
        return self._load_i64(me, off)

    def wait_until_all(self, me: int, off: int, nelems: int, status, cmp: int, value: int) -> None:
        if not self.test_all(me, off, nelems, status, cmp, value):
            raise OracleError("wait_until_all can never be satisfied in this sequential order")

    def wait_until_some(self, me: int, off: int, nelems: int, status, cmp: int, value: int) -> list:
        """The satisfying indices; with a non-empty set at least one must satisfy, else the wait never ends."""
        hits = self.test_some(me, off, nelems, status, cmp, value)
        if not hits and self._ivars(me, off, nelems, status):
            raise OracleError("wait_until_some / wait_until_any can never be satisfied in this sequential order")
        return hits

    def wait_until_any(self, me: int, off: int, nelems: int, status, cmp: int, value: int) -> list:
        """The indices any of which a correct wait_until_any may return (empty set: it returns 'none')."""
        return self.wait_until_some(me, off, nelems, status, cmp, value)

    # ---------------------------------------------------------------- ordering
    def quiet(self, me: int) -> None:
        self._pe(me)
        self.log.append(("quiet", me))

    def fence(self, me: int) -> None:
        self._pe(me)
        self.log.append(("fence", me))

    def barrier_all(self) -> None:
        self.log.append(("barrier_all",))

    # ----------------------------------------------------------------- atomics
    def _load_i64(self, pe: int, off: int) -> int:
        return _to_i64(self._load_u64(pe, off))

    def atomic_fetch(self, me: int, off: int, pe: int) -> int:
        self._pe(me), self._pe(pe), self._word(off)
        return self._load_i64(pe, off)

    def atomic_set(self, me: int, off: int, value: int, pe: int) -> None:
        self._pe(me), self._pe(pe), self._word(off)
        self._store_u64(pe, off, value)

    def atomic_swap(self, me: int, off: int, value: int, pe: int) -> int:
        self._pe(me), self._pe(pe), self._word(off)
        old = self._load_i64(pe, off)
        self._store_u64(pe, off, value)
        return old

    def atomic_fetch_add(self, me: int, off: int, value: int, pe: int) -> int:
        self._pe(me), self._pe(pe), self._word(off)
        old = self._load_i64(pe, off)
        self._store_u64(pe, off, old + value)
        return old

    def atomic_add(self, me: int, off: int, value: int, pe: int) -> None:
        self.atomic_fetch_add(me, off, value, pe)

    def atomic_fetch_inc(self, me: int, off: int, pe: int) -> int:
        return self.atomic_fetch_add(me, off, 1, pe)

    def atomic_inc(self, me: int, off: int, pe: int) -> None:
        self.atomic_fetch_add(me, off, 1, pe)

    def atomic_compare_swap(self, me: int, off: int, cond: int, value: int, pe: int) -> int:
        self._pe(me), self._pe(pe), self._word(off)
        old = self._load_i64(pe, off)
        if old == _to_i64(cond):
            self._store_u64(pe, off, value)
        return old

    # -------------------------------------------------------------- collectives
    def fcollect(self, dst: int, src: int, n: int) -> None:
        """Every PE's block of ``n`` bytes, in PE order, lands in every PE's destination."""
        self._range(src, n)
        self._range(dst, n * self.npes)
        if n and src < dst + n * self.npes and dst < src + n:
            # peers write the destination while the owner's source is still being read: no unique result
            raise OracleError("overlapping source and destination")
        blocks = [self.heap[p][src:src + n].copy() for p in range(self.npes)]
        for q in range(self.npes):
            for p in range(self.npes):
                self.heap[q][dst + p * n:dst + (p + 1) * n] = blocks[p]

    def collect(self, dst: int, src: int, nbytes: list) -> None:
        """Concatenation with a different block size per PE (paper section "Collective Operations":
        push broadcast / collect / fcollect; OpenSHMEM collect): PE p contributes ``nbytes[p]``
        bytes from ``src``; every PE's destination receives the blocks in PE order, block p at the
        sum of the sizes before it."""
        if len(nbytes) != self.npes or any(n < 0 for n in nbytes):
            raise OracleError("one non-negative size per PE")
        total = sum(nbytes)
        self._range(dst, total)
        for p in range(self.npes):
            self._range(src, nbytes[p])
            if nbytes[p] and total and src < dst + total and dst < src + nbytes[p]:
                raise OracleError("overlapping source and destination")
        blocks = [self.heap[p][src:src + nbytes[p]].copy() for p in range(self.npes)]
        for q in range(self.npes):
            at = dst
            for p in range(self.npes):
                self.heap[q][at:at + nbytes[p]] = blocks[p]
                at += nbytes[p]

    def wave_exchange(self, me: int, pe: int, dst: int, src: int, back: int, n: int, n_waves: int, flag: int,
                      out: int) -> None:
        """The sub-group (wave) forms in one program (paper section "Proposed Device APIs": the
        sub-group extensions): wave w of PE ``me`` puts the w-th slice of the message to PE ``pe``,
        fences, and sets pe's w-th flag word to 1; wave w of PE ``pe`` waits for that flag, stores
        the value it fetches from it to its w-th out word, and gets the slice from its own
        destination into ``back``.  Slices as for work-groups (16-byte-rounded equal shares)."""
        self._pe(me), self._pe(pe)
        for w, (lo, hi) in enumerate(self.wg_slices(n, n_waves)):
            self.putmem(me, dst + lo, src + lo, hi - lo, pe)
            self.fence(me)
            self.atomic_set(me, flag + 8 * w, 1, pe)
        for w, (lo, hi) in enumerate(self.wg_slices(n, n_waves)):
            self.signal_wait_until(pe, flag + 8 * w, CMP_EQ, 1)
            self._store_u64(pe, out + 8 * w, self.signal_fetch(pe, flag + 8 * w))
            self.getmem(pe, back + lo, dst + lo, hi - lo, pe)

    REDUCE_OPS = ("min", "max", "sum", "prod", "and", "or", "xor")

    def reduce(self, dst: int, src: int, nelems: int, dtype, op: str) -> np.ndarray:
        """Element-wise ``x0 op x1 op ... `` over PEs in the order 0, 1, ..., npes-1; every PE's
        destination receives the result.  Integer sum/prod wrap to the element width; min/max keep
        the earlier operand on ties; and/or/xor are for integer types only."""
        dt = np.dtype(dtype)
        if op not in self.REDUCE_OPS:
            raise OracleError("unknown reduction")
        if op in ("and", "or", "xor") and dt.kind not in "iu":
            raise OracleError("bitwise reductions need an integer type")
        nb = dt.itemsize * nelems
        self._range(src, nb), self._range(dst, nb)
        if src % 16 or dst % 16:
            raise OracleError("reduction buffers must be 16-byte aligned")
        if nelems and src < dst + nb and dst < src + nb:
            raise OracleError("overlapping source and destination")
        vecs = [self.heap[p][src:src + nb].copy().view(dt) for p in range(self.npes)]
        r = vecs[0].copy()
        with np.errstate(over="ignore"):
            for p in range(1, self.npes):
                x = vecs[p]
                if op == "min":
                    r = np.where(x < r, x, r)
                elif op == "max":
                    r = np.where(x > r, x, r)
                elif op == "sum":
                    r = (r + x).astype(dt)
                elif op == "prod":
                    r = (r * x).astype(dt)
                elif op == "and":
                    r = r & x
                elif op == "or":
                    r = r | x
                else:
                    r = r ^ x
        out = np.ascontiguousarray(r, dtype=dt).view(np.uint8)
        for q in range(self.npes):
            self.heap[q][dst:dst + nb] = out
        return r

    def broadcast(self, dst: int, src: int, n: int, root: int) -> None:
        """Bytes [src, src+n) of PE ``root`` land at [dst, dst+n) of every PE, the root included."""
        self._pe(root)
        self._range(src, n), self._range(dst, n)
        if n and src < dst + n and dst < src + n:
            raise OracleError("overlapping source and destination")
        block = self.heap[root][src:src + n].copy()
        for q in range(self.npes):
            self.heap[q][dst:dst + n] = block

    def sync_all(self) -> None:
        """Every PE waits for every other; no data moves and nothing is ordered."""
        self.log.append(("sync_all",))

    def barrier_exchange(self, dst: int, src: int, acc: int, n: int, rounds: int) -> None:
        """Round r: every PE p puts its block into slot p of PE (p+1+r) mod npes; barrier; every PE
        copies the slot just filled for it (that of PE (p-1-r) mod npes) to ``acc + r*n``."""
        for r in range(rounds):
            for p in range(self.npes):
                self.putmem(p, dst + p * n, src, n, (p + 1 + r) % self.npes)
            self.barrier_all()
            for p in range(self.npes):
                frm = (p - 1 - r) % self.npes
                self.getmem(p, acc + r * n, dst + frm * n, n, p)

    def reduce_sum_f32(self, dst: int, src: int, nelems: int) -> dict:
        """Element-wise binary32 sum over PEs in the order 0, 1, ..., npes-1.

        Every PE's destination receives the same vector.  Also returns the
        binary64 sum and the sum of magnitudes, for error-bound checks.
        """
        nb = 4 * nelems
        self._range(src, nb)
        self._range(dst, nb)
        if src % 4 or dst % 4:
            raise OracleError("float32 vectors must be 4-byte aligned")
        vecs = [self.heap[p][src:src + nb].copy().view(np.float32) for p in range(self.npes)]
        r = vecs[0].copy()
        for p in range(1, self.npes):
            r = (r + vecs[p]).astype(np.float32)
        r64 = np.zeros(nelems, dtype=np.float64)
        mag = np.zeros(nelems, dtype=np.float64)
        for v in vecs:
            r64 += v.astype(np.float64)
            mag += np.abs(v.astype(np.float64))
        out = r.view(np.uint8)
        for q in range(self.npes):
            self.heap[q][dst:dst + nb] = out
        return {"f32": r, "f64": r64, "abs": mag}

    # ----------------------------------------------------- benchmark composites
    @staticmethod
    def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
        """bf16 is the top half of binary32: widening is a 16-bit left shift, exact."""
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)

    def ring_pipeline(self, src: int, slot: int, sig: int, acc: int, chunk_bytes: int, n_chunks: int,
                      n_wg_prod: int = 1, n_sig: int = 1) -> None:
        """Pipelined ring: PE p sends chunk k to slot k of PE (p+1) mod npes with
        put-with-signal (ADD 1); the receiver waits ``signal >= k+1`` and adds the
        bf16 chunk, widened to binary32, into its binary32 accumulator, k ascending.
        The accumulator is zeroed first; the signal words must start at zero.

        n_sig == 1: one signal word; the chunk travels as one put-with-signal shared
        by n_wg_prod groups.  n_sig > 1: lanes -- the chunk is cut into n_sig shares,
        share j travels with its own put-with-signal on word ``sig + 8*j`` and the
        receiver waits on that word before adding that share.
        """
        if chunk_bytes % 2:
            raise OracleError("a chunk holds whole bf16 values")
        nel = chunk_bytes // 2
        self._range(src, chunk_bytes * n_chunks)
        self._range(slot, chunk_bytes * n_chunks)
        self._range(acc, 4 * nel)
        shares = [(0, chunk_bytes)] if n_sig == 1 else self.wg_slices(chunk_bytes, n_sig)
        # one legal sequential schedule: all sends of chunk k, then all consumes of chunk k
        accs = [np.zeros(nel, dtype=np.float32) for _ in range(self.npes)]
        for k in range(n_chunks):
            for p in range(self.npes):
                for j, (lo, hi) in enumerate(shares):
                    self.put_signal(p, slot + k * chunk_bytes + lo, src + k * chunk_bytes + lo, hi - lo,
                                    sig + 8 * j, 1, SIGNAL_ADD, (p + 1) % self.npes, n_wg_prod if n_sig == 1 else 1)
            for p in range(self.npes):
                for j, (lo, hi) in enumerate(shares):
                    self.signal_wait_until(p, sig + 8 * j, CMP_GE, k + 1)
                    bits = self.heap[p][slot + k * chunk_bytes + lo:slot + k * chunk_bytes + hi].copy().view(np.uint16)
                    accs[p][lo // 2:hi // 2] = (accs[p][lo // 2:hi // 2] + self.bf16_bits_to_f32(bits)).astype(np.float32)
        for p in range(self.npes):
            self.heap[p][acc:acc + 4 * nel] = accs[p].view(np.uint8)

    def amo_storm_loop(self, ctr: int, n_ctr: int, targets: np.ndarray) -> np.ndarray:
        """One fetch-add(+1) per entry of ``targets`` in row-major order, one at a time.

        ``targets`` has shape [n_items, ops_per_item]; entry t selects counter
        ``t % n_ctr`` of PE ``t // n_ctr``.  Work-item g is issued by PE
        ``g * npes // n_items``.  Returns the fetched values, same shape.  Pure
        Python loop: for small cases only.
        """
        n_items = targets.shape[0]
        out = np.zeros(targets.shape, dtype=np.int64)
        for g in range(n_items):
            me = g * self.npes // n_items
            for j in range(targets.shape[1]):
                t = int(targets[g, j])
                out[g, j] = self.atomic_fetch_add(me, ctr + 8 * (t % n_ctr), 1, t // n_ctr)
        return out

    def amo_storm(self, ctr: int, n_ctr: int, targets: np.ndarray) -> np.ndarray:
        """Same result as ``amo_storm_loop`` computed with array operations.

        In row-major issue order the value fetched by an operation is the counter's
        initial value plus the number of earlier operations on the same counter;
        the final counter is the initial value plus the total count.
        """
        flat = targets.reshape(-1).astype(np.int64)
        if flat.size and (flat.min() < 0 or flat.max() >= self.npes * n_ctr):
            raise OracleError("target outside the counter set")
        self._range(ctr, 8 * n_ctr)
        if ctr % 8:
            raise OracleError("counters must be 8-byte aligned")
        order = np.argsort(flat, kind="stable")
        sorted_t = flat[order]
        first = np.searchsorted(sorted_t, sorted_t, side="left")
        rank_sorted = np.arange(flat.size, dtype=np.int64) - first
        rank = np.empty(flat.size, dtype=np.int64)
        rank[order] = rank_sorted
        counts = np.bincount(flat, minlength=self.npes * n_ctr).astype(np.int64)
        init = np.concatenate([self.heap[p][ctr:ctr + 8 * n_ctr].copy().view(np.int64) for p in range(self.npes)])
        fetched = (init[flat] + rank).reshape(targets.shape)
        final = init + counts
        for p in range(self.npes):
            self.heap[p][ctr:ctr + 8 * n_ctr] = final[p * n_ctr:(p + 1) * n_ctr].view(np.uint8)
        return fetched
