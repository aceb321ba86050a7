"""A small closed-loop problem for DEF / DEF-A: a separable quadratic whose
gradient is element-wise, so that the gradient computation itself rounds
identically in numpy and in torch on the GPU and whole trajectories can be
compared bit for bit.

Worker k holds  f_k(theta) = 0.5 * sum_i a_i * (theta_i - c_{k,i})^2  and reports
g_k = a * (w_k - c_k) + noise_{k,t}  evaluated at its detached point
w_k = x - lambda*e_k (Algorithm 1 of arXiv 2004.05298, "detach" line).  The
curvatures a_i are shared, the optima c_k = c + spread*z_k differ per worker, and
the noise is drawn from a seeded pool.  This module only produces the problem data
and evaluates the objective; it holds none of the method's arithmetic.
"""
from __future__ import annotations

import numpy as np


class ToyProblem:
    def __init__(self, d: int, W: int, seed: int = 0, pool: int = 8, noise: float = 0.05,
                 spread: float = 0.2):
        rng = np.random.default_rng([200405298, 404, seed, d, W])
        self.d, self.W, self.pool = d, W, pool
        self.a = np.exp(rng.uniform(np.log(0.05), np.log(1.0), size=d)).astype(np.float32)
        self.c_mean = rng.standard_normal(d).astype(np.float32)
        self.c = (self.c_mean[None, :] + spread * rng.standard_normal((W, d))).astype(np.float32)
        self.noise = (noise * rng.standard_normal((pool, W, d))).astype(np.float32)
        self.x0 = (self.c_mean + rng.standard_normal(d)).astype(np.float32)

    def gradients(self, w: np.ndarray, t: int) -> np.ndarray:
        """numpy float32: (w - c) then * a then + noise, one rounding each."""
        out = w - self.c
        out = out * self.a[None, :]
        return out + self.noise[t % self.pool]

    def objective(self, theta: np.ndarray) -> float:
        """F(theta) = mean_k f_k(theta), float64."""
        diff = theta.astype(np.float64)[None, :] - self.c.astype(np.float64)
        return float(0.5 * np.mean(np.sum(self.a.astype(np.float64)[None, :] * diff * diff, axis=1)))

    def minimum(self) -> float:
        return self.objective(self.c.astype(np.float64).mean(axis=0).astype(np.float32))
