"""Writes tests/golden/tiny_digest.txt: the block starts and SHA-256 digests of
(x, e, m, y) after the T steps of the tiny workload, computed by the numpy
oracle alone.  A guard against silent drift of the oracle's arithmetic or of the
input generators; it calls nothing but oracle/ and the input generators.

    python tests/golden/make_tiny_digest.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.def_oracle import DefOracle          # noqa: E402
from paper_2004_05298_amd import workloads as wl  # noqa: E402


def digest_lines():
    w = wl.tiny()
    o = DefOracle(wl.initial_params(w), w.W, w.R, w.lr, w.momentum, w.weight_decay, w.seed)
    pool = wl.gradient_pool(w, threads=1)
    starts = [o.step(pool[t % w.pool]) for t in range(w.T)]
    lines = [f"workload {w.name} d={w.d} W={w.W} R={w.R} B={w.B} T={w.T} seed={w.seed}",
             "starts " + " ".join(str(s) for s in starts)]
    for name, arr in (("x", o.x), ("e", o.e), ("m", o.m), ("y", o.y())):
        lines.append(f"{name} {hashlib.sha256(np.ascontiguousarray(arr).tobytes()).hexdigest()}")
    return lines


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_digest.txt")
    with open(out, "w") as f:
        f.write("\n".join(digest_lines()) + "\n")
    print(open(out).read())
