"""Shared pieces of the GPU parity tests: run the HIP path and the CPU oracle on
the same seeded inputs and compare.

Tolerance for floating-point outputs (averaged block, x, e, m, y), written out:
    element-wise  |gpu - ora| <= 1e-6*|ora| + 1e-6*rms(ora)
    and norm-wise ||gpu - ora||_2 <= 1e-6*||ora||_2.
The absolute floor is there because the averaged block is a mean of zero-mean
values, whose entries cancel to near zero.  Both sides round every operation
separately in binary32 and add the workers in the same order, so in practice the
buffers are bit-identical; the tests record whether they are.
Integer results (block start, block length) and the error-memory zeroing inside
the block are compared bit for bit.
"""
from __future__ import annotations

import numpy as np

REL = 1e-6


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32)


def bit_equal(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and bool(np.array_equal(bits(a), bits(b)))


def assert_close(name: str, gpu: np.ndarray, ora: np.ndarray, rel: float = REL) -> None:
    assert gpu.shape == ora.shape, (name, gpu.shape, ora.shape)
    if bit_equal(gpu, ora):
        return
    g64, o64 = gpu.astype(np.float64), ora.astype(np.float64)
    finite = np.isfinite(o64)
    assert np.array_equal(np.isnan(g64), np.isnan(o64)), f"{name}: NaN pattern differs"
    assert np.array_equal(g64[~finite & ~np.isnan(o64)], o64[~finite & ~np.isnan(o64)]), \
        f"{name}: infinities differ"
    g64, o64 = g64[finite], o64[finite]
    rms = float(np.sqrt(np.mean(o64 ** 2))) if o64.size else 0.0
    err = np.abs(g64 - o64)
    bound = rel * np.abs(o64) + rel * rms
    worst = int(np.argmax(err - bound)) if err.size else 0
    assert (err <= bound).all(), (f"{name}: element {worst}: gpu {g64[worst]!r} oracle {o64[worst]!r} "
                                  f"err {err[worst]:.3e} > {bound[worst]:.3e}")
    assert np.linalg.norm(g64 - o64) <= rel * np.linalg.norm(o64), f"{name}: norm-wise bound"


def in_block_mask(d: int, s: int, B: int) -> np.ndarray:
    """Independent of the oracle's predicate: enumerate the kept indices."""
    mask = np.zeros(d, dtype=bool)
    first = min(B, d - s)
    mask[s:s + first] = True
    mask[:B - first] = True
    return mask
