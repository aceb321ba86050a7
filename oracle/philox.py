"""Shared-seed block start for RBGS (arXiv 2004.05298, Sec. 1: every worker is
given the same random seed and samples one start index uniformly).

TEST INFRASTRUCTURE ONLY (part of the CPU oracle).

The paper does not name a generator.  The reading taken here: a counter-based
draw, so that the start of step t is a pure function of (seed, t):

    s_t = Philox4x64-10(counter = (t, 0, 0, 0), key = (seed, 0))[0]  mod  d

Philox4x64-10 is the generator of Salmon, Moraes, Dror and Shaw, "Parallel
random numbers: as easy as 1, 2, 3" (SC 2011): ten rounds, each multiplying two
counter words by fixed 64-bit constants and mixing the high/low halves of the
128-bit products with the other words and the key, the key advancing by the
Weyl constants between rounds.  Written here with Python integers so that no
word-size detail can hide a mistake.  The modulo bias is below d / 2^64.
"""
from __future__ import annotations

from typing import List, Sequence

_MASK = (1 << 64) - 1
_MUL_A = 0xD2E7470EE14C6C93      # multiplier for counter word 0
_MUL_B = 0xCA5A826395121157      # multiplier for counter word 2
_WEYL_A = 0x9E3779B97F4A7C15     # golden-ratio increment for key word 0
_WEYL_B = 0xBB67AE8584CAA73B     # sqrt(3)-1 increment for key word 1


def philox4x64_10(counter: Sequence[int], key: Sequence[int]) -> List[int]:
    c0, c1, c2, c3 = (int(v) & _MASK for v in counter)
    k0, k1 = (int(v) & _MASK for v in key)
    for _ in range(10):
        prod_a = _MUL_A * c0
        prod_b = _MUL_B * c2
        c0, c1, c2, c3 = ((prod_b >> 64) ^ c1 ^ k0, prod_b & _MASK,
                          (prod_a >> 64) ^ c3 ^ k1, prod_a & _MASK)
        k0 = (k0 + _WEYL_A) & _MASK
        k1 = (k1 + _WEYL_B) & _MASK
    return [c0, c1, c2, c3]


def block_start(seed: int, t: int, d: int) -> int:
    """s_t in [0, d): the start index of the block kept at step t."""
    if d < 1:
        raise ValueError("d >= 1")
    return philox4x64_10((int(t) & _MASK, 0, 0, 0), (int(seed) & _MASK, 0))[0] % int(d)
