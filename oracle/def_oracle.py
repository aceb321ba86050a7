"""CPU oracle for the DEF / DEF-A compression-and-update step with RBGS.

TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition the HIP path is
checked against.  It shares no code with the HIP library; only tests, the smoke
check and the benchmark's CPU-baseline leg may import it.

What it follows (arXiv 2004.05298):

* Algorithm 1 ("Detached Error Feedback"), the error-feedback, residual,
  all-reduce and update lines:  p_k = eta*g_k + e_k ;  e_k <- p_k - C(p_k) ;
  C(p) = (1/K) sum_k C(p_k) ;  x <- x - C(p).
* Sec. 3.2 "Momentum Variant", Eq. (11):  m_k <- mu*m_k + g_k ;  p_k = eta*m_k + e_k,
  with m_{k,0} = 0.
* Algorithm 1 "Output" / Sec. 3.2 Eq. (8):  y = x - (1/K) sum_k e_k for
  DEF, x itself for DEF-A.  DEF and DEF-A run the same iteration.
* Algorithm 1, "detach" line:  worker k evaluates its next gradient at
  x - lambda*e_k  (`detached_points`).
* Sec. 1 (RBGS): the compressor C keeps ONE contiguous block of the flattened
  vector whose start index is sampled uniformly; all workers share the seed and
  therefore the block.

Readings taken where the paper is silent (each is listed in the design notes):
block length B = ceil(d/R) for an integer ratio R; the block wraps circularly
past index d-1; the start index is a counter-based Philox4x64-10 draw keyed by
the seed with the step number as counter (oracle/philox.py), reduced mod d;
weight decay is folded into the gradient at the shared iterate, g' = g + wd*x;
every multiply and add is rounded separately in the working precision (no
fused multiply-add); the cross-worker sum runs k = 0..W-1 in order starting
from +0 and is divided once by W; the error memory inside the block is the
literal +0.

The working precision is a parameter: float32 is the precision the method
communicates and stores in (Sec. 2, "32-bit gradient component") and is what
the HIP path is compared with; float64 serves the invariant pins.

A column subset can be simulated exactly: every column i of (x, e, m) evolves
independently of all other columns once the block of each step is known, so
`index` may hold any set of global indices and the state then has one column
per entry of `index`.
"""
from __future__ import annotations

from typing import Callable, Optional

import numpy as np

from .philox import block_start


def block_length(d: int, R: int) -> int:
    """B = ceil(d / R) for an integer compression ratio R (Sec. 4, Assumption 4.2,
    the delta-approximate compressor: delta equals the kept fraction; Tables 1-2
    use integer ratios)."""
    if R < 1 or R > d:
        raise ValueError("need 1 <= R <= d")
    return -(-d // R)


def in_block(index: np.ndarray, s: int, B: int, d: int) -> np.ndarray:
    """Membership of global indices in the circular block {(s+j) mod d : 0<=j<B}
    (Sec. 1: one uniformly sampled start index, one contiguous block)."""
    index = np.asarray(index, dtype=np.int64)
    return ((index - np.int64(s)) % np.int64(d)) < np.int64(B)


class DefOracle:
    """State (x, e_k, m_k, seed, t) and one-step transition of DEF / DEF-A."""

    def __init__(self, x0, W: int, R: int, lr: float, momentum: float = 0.0,
                 weight_decay: float = 0.0, seed: int = 0, d: Optional[int] = None,
                 index=None, dtype=np.float32,
                 compressor: Optional[Callable[[np.ndarray, int], np.ndarray]] = None):
        self.dtype = np.dtype(dtype)
        self.x = np.array(x0, dtype=self.dtype).copy()
        n = self.x.shape[0]
        self.d = int(n if d is None else d)
        self.index = (np.arange(n, dtype=np.int64) if index is None
                      else np.asarray(index, dtype=np.int64).copy())
        if self.index.shape != (n,):
            raise ValueError("index must have one entry per column of x0")
        if W < 1:
            raise ValueError("W >= 1")
        self.W = int(W)
        self.R = int(R)
        self.B = block_length(self.d, self.R)
        self.lr = self.dtype.type(lr)
        self.mu = self.dtype.type(momentum)
        self.wd = self.dtype.type(weight_decay)
        self.seed = int(seed)
        self.t = 0
        self.e = np.zeros((self.W, n), dtype=self.dtype)          # e_{k,0} = 0 (Alg. 1, Initialize)
        self.m = np.zeros((self.W, n), dtype=self.dtype)          # m_{k,0} = 0 (Momentum Variant)
        self.compressor = compressor                              # pins only; None = RBGS
        self.last_start: Optional[int] = None
        self.last_mask: Optional[np.ndarray] = None
        self.last_cbar_dense: Optional[np.ndarray] = None         # C(p_t), dense, zero off-block
        self.last_p: Optional[np.ndarray] = None                  # p_{k,t}, kept when record_p

    # -- hyper-parameters that may change between steps ---------------------- #
    def set_lr(self, lr: float) -> None:
        self.lr = self.dtype.type(lr)

    def set_seed(self, seed: int) -> None:
        """New seed; the step counter keeps counting."""
        self.seed = int(seed)

    def set_step(self, t: int) -> None:
        self.t = int(t)

    # -- one iteration -------------------------------------------------------- #
    def step(self, g, start: Optional[int] = None, record_p: bool = False) -> int:
        """Consume gradients g[W][n] (columns matching `index`) and advance the
        state by one iteration.  Returns the block start used.  `start`
        overrides the seeded draw (forced wrap positions, enumeration pins)."""
        ft = self.dtype.type
        g = np.asarray(g, dtype=self.dtype)
        if g.shape != self.e.shape:
            raise ValueError(f"g must be {self.e.shape}, got {g.shape}")
        s = block_start(self.seed, self.t, self.d) if start is None else int(start)
        if not 0 <= s < self.d:
            raise ValueError("start out of range")
        mask = in_block(self.index, s, self.B, self.d)
        zero = np.zeros_like(self.x)
        acc = np.zeros_like(self.x)                                 # running sum starts at +0
        if record_p:
            self.last_p = np.empty_like(self.e)
        for k in range(self.W):
            gk = g[k]
            if self.wd != ft(0):
                gk = gk + self.wd * self.x                          # g' = g + wd*x_t (shared iterate)
            if self.mu != ft(0):
                mk = self.mu * self.m[k] + gk                       # m_{k,t+1} = mu*m_{k,t} + g_{k,t}
                self.m[k] = mk
            else:
                mk = gk                                             # Algorithm 1 as printed (no momentum)
            p = self.lr * mk + self.e[k]                            # p_{k,t} = eta*m_{k,t+1} + e_{k,t}
            if record_p:
                self.last_p[k] = p
            if self.compressor is None:
                cp = np.where(mask, p, zero)                        # C(p_k): the block, zero elsewhere
                self.e[k] = np.where(mask, zero, p)                 # e_{k,t+1} = p_k - C(p_k); +0 in block
            else:
                cp = self.compressor(p, self.t).astype(self.dtype)
                self.e[k] = p - cp
            acc = acc + cp                                          # k ascending
        cbar = acc / ft(self.W)                                     # (1/K) sum_k C(p_k)
        self.x = self.x - cbar                                      # x_{t+1} = x_t - C(p_t)
        self.last_start, self.last_mask, self.last_cbar_dense = s, mask, cbar
        self.t += 1
        return s

    # -- outputs -------------------------------------------------------------- #
    def y(self) -> np.ndarray:
        """DEF's returned model y = x - (1/K) sum_k e_k (k ascending, one
        division); DEF-A returns x."""
        acc = np.zeros_like(self.x)
        for k in range(self.W):
            acc = acc + self.e[k]
        return self.x - acc / self.dtype.type(self.W)

    def detached_points(self, lam: float) -> np.ndarray:
        """The points w_k = x - lambda*e_k at which worker k evaluates its next
        gradient (Algorithm 1, "detach" line), one row per worker.  lambda*e_k
        and the subtraction round separately."""
        lam = self.dtype.type(lam)
        out = np.empty_like(self.e)
        for k in range(self.W):
            out[k] = self.x - lam * self.e[k]
        return out

    def diagnostics(self, lam: float) -> dict:
        """Error-memory statistics of Sec. 3.2 / Appendix A, in float64 from the
        stored error memories: with e_t = (1/K) sum_k e_k,
          bar_sq   = ||e_t||^2                      (EF's distance ||x_t - y_t||^2)
          mean_sq  = (1/K) sum_k ||e_k||^2
          lam_star = bar_sq / mean_sq               (lambda*(t), Sec. 3.2 item (2))
          dist     = (1/K) sum_k ||e_t - lam*e_k||^2   (Eq. (9)), summed directly."""
        e = self.e.astype(np.float64)
        acc = np.zeros(e.shape[1], dtype=np.float64)
        for k in range(self.W):
            acc = acc + e[k]
        e_bar = acc / np.float64(self.W)
        bar_sq = float(np.sum(e_bar * e_bar))
        mean_sq = float(sum(np.sum(e[k] * e[k]) for k in range(self.W)) / self.W)
        dist = float(sum(np.sum((e_bar - np.float64(lam) * e[k]) ** 2) for k in range(self.W)) / self.W)
        return dict(bar_sq=bar_sq, mean_sq=mean_sq,
                    lam_star=(bar_sq / mean_sq if mean_sq > 0 else 0.0), dist=dist)

    def diagnostics_workers(self) -> dict:
        """Per-worker statistics of Sec. 3.2 item (1) / Appendix A, first display, in
        float64: with e_t = (1/K) sum_k e_k, for every worker k
          norm_sq[k]  = ||e_k||^2
          inner[k]    = <e_t, e_k>
          lam_star[k] = inner[k] / norm_sq[k]      (lambda*(k,t), the lambda that brings
                        worker k's evaluation point x - lambda*e_k closest to y; 0 when
                        e_k = 0)."""
        e = self.e.astype(np.float64)
        acc = np.zeros(e.shape[1], dtype=np.float64)
        for k in range(self.W):
            acc = acc + e[k]
        mean_e = acc / np.float64(self.W)                           # e_t
        norm_sq = np.array([np.sum(e[k] * e[k]) for k in range(self.W)], dtype=np.float64)
        inner = np.array([np.sum(mean_e * e[k]) for k in range(self.W)], dtype=np.float64)
        lam_star = np.array([inner[k] / norm_sq[k] if norm_sq[k] > 0 else 0.0
                             for k in range(self.W)], dtype=np.float64)
        return dict(norm_sq=norm_sq, inner=inner, lam_star=lam_star)

    def compact_block(self) -> np.ndarray:
        """The averaged block of the last step as the B-vector that would be
        all-reduced: entry j belongs to global index (s+j) mod d.  Needs the
        full index range."""
        if self.index.shape[0] != self.d or not np.array_equal(self.index, np.arange(self.d)):
            raise ValueError("compact_block needs the full index range")
        j = (np.int64(self.last_start) + np.arange(self.B, dtype=np.int64)) % np.int64(self.d)
        return self.last_cbar_dense[j]

    # -- checkpoint ----------------------------------------------------------- #
    def get_state(self) -> dict:
        return dict(x=self.x.copy(), e=self.e.copy(), m=self.m.copy(), t=self.t, seed=self.seed,
                    lr=float(self.lr))

    def set_state(self, st: dict) -> None:
        self.x = np.array(st["x"], dtype=self.dtype)
        self.e = np.array(st["e"], dtype=self.dtype)
        self.m = np.array(st["m"], dtype=self.dtype)
        self.t = int(st["t"])
        self.seed = int(st["seed"])
        self.lr = self.dtype.type(st["lr"])
