"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws numbers.  It holds none of the library's or the oracle's
arithmetic, imports neither, and is the one piece both sides of a parity test
share: the same arrays are written into the oracle's heaps and into the GPU
heaps.  All generators are numpy ``default_rng`` streams derived from
``BASE_SEED``, the configuration number and the PE, so any PE's data can be
produced on its own.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20476


def _rng(config: int, pe: int = 0, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED + config, pe, stream])


def c1_payload(nelems: int = 4096) -> np.ndarray:
    """Config 1: int32 values uniform in [0, 2^31) held by PE 0."""
    return _rng(1).integers(0, 2 ** 31, size=nelems, dtype=np.int64).astype(np.int32)


def c2_source(pe: int, nbytes: int) -> np.ndarray:
    """Config 2: the first ``nbytes`` of PE ``pe``'s float32 N(0,1) buffer, as bytes.

    Sizes below 4 bytes (not used by the sweep, but legal for putmem) take a prefix
    of the first value's bytes.
    """
    nel = max(1, -(-nbytes // 4))
    v = _rng(2, pe).standard_normal(nel, dtype=np.float32)
    return v.view(np.uint8)[:nbytes].copy()


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round binary32 to bf16 (round to nearest, ties to even); returns the 16-bit patterns.

    Input preparation only: both the oracle and the GPU receive these bits.
    Inputs are finite, so no NaN handling is needed.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = u + np.uint64(0x7FFF) + lsb
    return (u >> np.uint64(16)).astype(np.uint16)


def c3_chunks(pe: int, n_chunks: int = 64, chunk_elems: int = 524288) -> np.ndarray:
    """Config 3: PE ``pe``'s chunks, bf16 bit patterns of uniform [-1, 1) values; shape [n_chunks, chunk_elems]."""
    v = _rng(3, pe).random((n_chunks, chunk_elems), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    return f32_to_bf16_bits(v).reshape(n_chunks, chunk_elems)


def c4_targets(n_items: int = 1 << 20, ops_per_item: int = 64, npes: int = 16, n_ctr: int = 1024) -> np.ndarray:
    """Config 4: one (target PE, counter) pair per atomic, packed as ``pe * n_ctr + index``.

    Shape [n_items, ops_per_item], uint16, uniform over all npes * n_ctr counters.
    """
    if npes * n_ctr > 65536:
        raise ValueError("target ids are 16-bit")
    return _rng(4).integers(0, npes * n_ctr, size=(n_items, ops_per_item), dtype=np.uint16)


def c5_fcollect_source(pe: int, nelems: int) -> np.ndarray:
    """Config 5: int32 uniform in [0, 2^31)."""
    return _rng(5, pe, 0).integers(0, 2 ** 31, size=nelems, dtype=np.int64).astype(np.int32)


def c5_reduce_source(pe: int, nelems: int) -> np.ndarray:
    """Config 5: float32 N(0,1)."""
    return _rng(5, pe, 1).standard_normal(nelems, dtype=np.float32)
