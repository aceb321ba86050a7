"""Pins for the CPU oracle: every check here compares the oracle with something
the paper or the mathematics fixes, never with the oracle's own formula.

Citations are to arXiv 2004.05298.
"""
import itertools

import numpy as np
import pytest
import scipy.signal
import torch

from oracle.brute_force import brute_force_step
from oracle.c_oracle import DefOracleC
from oracle.def_oracle import DefOracle, block_length, in_block
from oracle.philox import block_start, philox4x64_10


# tests/test_oracle_mutants.py swaps in deliberately broken copies of the numpy
# oracle through this hook to show that the pins notice them.
NUMPY_ORACLE = DefOracle


def make(kind, x0, W, R, lr, mu=0.0, wd=0.0, seed=0, **kw):
    if kind == "np32":
        return NUMPY_ORACLE(x0, W, R, lr, mu, wd, seed, dtype=np.float32, **kw)
    if kind == "np64":
        return NUMPY_ORACLE(x0, W, R, lr, mu, wd, seed, dtype=np.float64, **kw)
    if kind == "c32":
        return DefOracleC(x0, W, R, lr, mu, wd, seed, **kw)
    raise ValueError(kind)


def bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint32 if a.dtype == np.float32 else np.uint64)


KINDS = ["np32", "np64", "c32"]
KINDS32 = ["np32", "c32"]


# --------------------------------------------------------------------------- #
# Block start: Sec. 1 (RBGS), "the same random seed" -> one shared start index.
# --------------------------------------------------------------------------- #
def _numpy_philox_word0(counter_words, key_words):
    # numpy's Philox is Philox4x64-10; it advances its 256-bit counter by one
    # before producing a block, so ask it for counter-1.
    v = sum(int(c) << (64 * i) for i, c in enumerate(counter_words))
    v = (v - 1) % (1 << 256)
    ctr = np.array([(v >> (64 * i)) & ((1 << 64) - 1) for i in range(4)], dtype=np.uint64)
    bg = np.random.Philox(counter=ctr, key=np.array(key_words, dtype=np.uint64))
    return [int(r) for r in bg.random_raw(4)]


@pytest.mark.parametrize("ctr,key", [
    ((0, 0, 0, 0), (0, 0)),
    ((1, 0, 0, 0), (200405298, 0)),
    ((2**64 - 1, 2**64 - 1, 2**64 - 1, 2**64 - 1), (2**64 - 1, 2**64 - 1)),
    ((7, 9, 11, 13), (17, 19)),
    ((123456789012345, 0, 0, 0), (0xDEADBEEFCAFEF00D, 0)),
])
def test_philox_matches_library_generator(ctr, key):
    assert philox4x64_10(ctr, key) == _numpy_philox_word0(ctr, key)


def test_block_start_is_library_draw_mod_d():
    for seed, d in [(0, 1), (1, 7), (200405298, 65536), (2**63 + 5, 25557032), (42, 138357544)]:
        for t in list(range(6)) + [10**6, 2**40 + 3]:
            ref = _numpy_philox_word0((t, 0, 0, 0), (seed, 0))[0] % d
            assert block_start(seed, t, d) == ref
            assert 0 <= ref < d


def test_block_start_roughly_uniform():
    d = 16
    counts = np.bincount([block_start(5, t, d) for t in range(16000)], minlength=d)
    # chi-square with 15 dof: 99.9 % quantile is 37.7
    chi2 = float(((counts - 1000.0) ** 2 / 1000.0).sum())
    assert chi2 < 37.7, chi2


@pytest.mark.parametrize("kind", KINDS)
def test_start_is_pure_function_of_seed_and_step(kind):
    """P2: s_t depends on (seed, t) only: not on gradients, learning rate, call
    history or a restore; set_seed changes the seed and keeps t."""
    d, W, R = 97, 3, 5
    rng = np.random.default_rng(1)
    a = make(kind, rng.standard_normal(d), W, R, 0.1, 0.9, seed=11)
    b = make(kind, rng.standard_normal(d), W, R, 0.5, 0.0, seed=11)
    sa, sb = [], []
    for t in range(12):
        if t == 5:
            a.set_lr(0.01)
        sa.append(a.step(rng.standard_normal((W, d)).astype(np.float32)))
        sb.append(b.step(rng.standard_normal((W, d)).astype(np.float32)))
    assert sa == sb == [block_start(11, t, d) for t in range(12)]
    a.set_seed(12)
    assert a.step(np.zeros((W, d), np.float32)) == block_start(12, 12, d)
    a.set_step(3)
    a.set_seed(11)
    assert a.step(np.zeros((W, d), np.float32)) == sa[3]


# --------------------------------------------------------------------------- #
# Compressor properties: Assumption 3.3 (linearity), Assumption 4.2 (delta-approximate
# compressor) and Remark 4.11, E_C[C(D)] = delta*D (RBGS keeps a fraction delta = B/d).
# --------------------------------------------------------------------------- #
def test_block_length_is_the_ceiling():
    """Reading of "a block" for an integer ratio R that does not divide d:
    B = ceil(d/R), the smallest block whose kept fraction B/d is at least 1/R
    (Assumption 4.2: delta is the compression ratio).  The five listed values are
    the block lengths of the five workload configurations."""
    for d, R, B in [(65536, 16, 4096), (853018, 32, 26657), (11689512, 64, 182649),
                    (25557032, 128, 199665), (138357544, 256, 540460)]:
        assert block_length(d, R) == B
    for d in range(1, 40):
        for R in range(1, d + 1):
            B = block_length(d, R)
            assert B * R >= d > (B - 1) * R
    assert block_length(9, 1) == 9 and block_length(9, 9) == 1
    for bad in [(5, 0), (5, 6)]:
        with pytest.raises(ValueError):
            block_length(*bad)


@pytest.mark.parametrize("d,R", [(12, 3), (13, 3), (13, 13), (9, 2), (7, 1), (16, 5)])
def test_enumerating_all_starts_covers_each_index_B_times(d, R):
    """P6 (index part): with circular wrap every index is kept by exactly B of
    the d possible starts; without wrap the first and last indices would not be."""
    B = block_length(d, R)
    cover = np.zeros(d, dtype=int)
    for s in range(d):
        mask = in_block(np.arange(d), s, B, d)
        assert mask.sum() == B
        assert mask[s] and mask[(s + B - 1) % d]
        if B < d:
            assert not mask[(s + B) % d] and not mask[(s - 1) % d]
        cover += mask
    assert (cover == B).all()


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("d,R", [(12, 3), (13, 3), (10, 4)])
def test_compressor_expectation_and_contraction(kind, d, R):
    """P6 (value part): one step from e=0, m=0 with eta=1, mu=0 gives
    x_1 = x_0 - C(g) for W=1, so C(g) is observable as x_0 - x_1.  With
    integer-valued g all sums are exact:  sum_s C_s(g) = B*g  and
    mean_s ||C_s(g) - g||^2 = (1 - B/d)*||g||^2."""
    B = block_length(d, R)
    rng = np.random.default_rng(3)
    g = rng.integers(-8, 9, size=(1, d)).astype(np.float32)
    total = np.zeros(d)
    err = 0.0
    for s in range(d):
        o = make(kind, np.zeros(d), 1, R, 1.0, 0.0, seed=0)
        o.step(g, start=s)
        c = -np.asarray(o.x, dtype=np.float64)
        total += c
        err += float(((c - g[0]) ** 2).sum())
        # residual is what was not sent
        assert np.array_equal(np.asarray(o.e[0], dtype=np.float64), g[0] - c)
    assert np.array_equal(total, B * g[0].astype(np.float64))
    assert err / d == pytest.approx((1 - B / d) * float((g[0].astype(np.float64) ** 2).sum()), rel=1e-12)


@pytest.mark.parametrize("kind", KINDS32)
def test_split_is_exact_and_block_is_literal_zero(kind):
    """P1 + zeroing: after a step the new error is bit-for-bit the compensated
    vector outside the block and the bit pattern 0x00000000 inside it; the sent
    block is bit-for-bit the compensated vector there (Algorithm 1, residual
    line).  The compensated vector is recomputed here for mu=0, wd=0 where it
    is a single multiply-add of inputs."""
    d, W, R = 50, 3, 4
    rng = np.random.default_rng(5)
    o = make(kind, rng.standard_normal(d), W, R, 0.25, 0.0, seed=9)
    e_prev = np.zeros((W, d), np.float32)
    for t in range(20):
        g = rng.standard_normal((W, d)).astype(np.float32)
        if t == 7:
            g[0, :] = -0.0  # p = -0 inside the block must still leave +0 behind
        x_prev = np.asarray(o.x).copy()
        s = o.step(g)
        p = np.float32(0.25) * g + e_prev
        mask = in_block(np.arange(d), s, o.B, d)
        e_now = np.asarray(o.e)
        assert (bits(e_now[:, mask]) == 0).all()
        assert np.array_equal(bits(e_now[:, ~mask]), bits(p[:, ~mask]))
        # x moved only inside the block, by the mean of p over workers
        assert np.array_equal(bits(np.asarray(o.x)[~mask]), bits(x_prev[~mask]))
        moved = x_prev[mask].astype(np.float64) - np.asarray(o.x)[mask].astype(np.float64)
        assert np.allclose(moved, p[:, mask].astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-7)
        e_prev = e_now.copy()


@pytest.mark.parametrize("kind", ["np64"])
def test_allreduce_compatibility_whole_iteration(kind):
    """P5: C is linear (Assumption 3.3), so W workers fed g_k and one worker fed
    mean_k g_k produce the same x path, and the single worker's error memory is
    the mean of the W error memories (mu and wd included: both are linear)."""
    d, W, R, T = 40, 4, 6, 15
    rng = np.random.default_rng(8)
    x0 = rng.standard_normal(d)
    many = make(kind, x0, W, R, 0.1, 0.9, 1e-2, seed=4)
    one = make(kind, x0, 1, R, 0.1, 0.9, 1e-2, seed=4)
    for t in range(T):
        g = rng.standard_normal((W, d))
        many.step(g)
        one.step(g.mean(axis=0, keepdims=True))
        assert np.allclose(many.x, one.x, rtol=1e-12, atol=1e-13)
        assert np.allclose(many.e.mean(axis=0), one.e[0], rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------- #
# Special case R = 1: uncompressed distributed momentum SGD (Sec. 2, the plain
# update theta <- theta - eta*g_t; Sec. 3.2 momentum variant).
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kind,tol", [("np64", 1e-12), ("np32", 2e-5), ("c32", 2e-5)])
@pytest.mark.parametrize("mu,wd", [(0.9, 0.0), (0.9, 5e-4), (0.0, 0.0), (0.0, 1e-2)])
def test_ratio_one_is_momentum_sgd(kind, tol, mu, wd):
    """P3: with R=1 the whole vector is the block, the error memory stays zero
    and x follows torch.optim.SGD(momentum, dampening=0, weight_decay) fed the
    mean gradient."""
    d, W, T = 33, 5, 25
    rng = np.random.default_rng(13)
    x0 = rng.standard_normal(d)
    o = make(kind, x0, W, 1, 0.1, mu, wd, seed=2)
    param = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([param], lr=0.1, momentum=mu, dampening=0.0, weight_decay=wd)
    for t in range(T):
        g = rng.standard_normal((W, d)).astype(np.float32)
        o.step(g)
        param.grad = torch.tensor(g.astype(np.float64).mean(axis=0))
        opt.step()
        assert not np.asarray(o.e).any()
        ref = param.detach().numpy()
        assert np.allclose(np.asarray(o.x, dtype=np.float64), ref, rtol=tol, atol=tol)


# --------------------------------------------------------------------------- #
# Trajectory identity y_{t+1} = y_t - eta*g_t (Sec. 3.2, Eq. (8);
# Appendix A, main proof, first display), momentum form.
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kind,tol", [("np64", 1e-12), ("np32", 3e-5), ("c32", 3e-5)])
@pytest.mark.parametrize("d,W,R", [(64, 4, 8), (61, 3, 7), (30, 1, 30), (17, 2, 1)])
def test_y_follows_uncompressed_momentum_path(kind, tol, d, W, R):
    """P4: y_t = x_t - mean_k e_{k,t} does not depend on the compressor:
    y_T = x_0 - eta * sum_t mean_k m_{k,t+1}, where m is the IIR filter
    m_{t+1} = mu*m_t + g_t of the inputs (computed here by scipy's lfilter)."""
    T, lr, mu = 30, 0.1, 0.9
    rng = np.random.default_rng(21)
    x0 = rng.standard_normal(d)
    o = make(kind, x0, W, R, lr, mu, 0.0, seed=77)
    G = rng.standard_normal((T, W, d)).astype(np.float32)
    ys = []
    for t in range(T):
        o.step(G[t], start=(d - 2 if t % 5 == 4 else None))   # includes wrapped blocks
        ys.append(np.asarray(o.y(), dtype=np.float64))
    m = scipy.signal.lfilter([1.0], [1.0, -mu], G.astype(np.float64), axis=0)   # m_{k,t+1}
    x0_stored = np.asarray(x0, dtype=o.dtype).astype(np.float64)
    y_ref = x0_stored[None, :] - lr * np.cumsum(m.mean(axis=1), axis=0)
    for t in range(T):
        assert np.allclose(ys[t], y_ref[t], rtol=tol, atol=tol), t


# --------------------------------------------------------------------------- #
# Single worker: Lemma C.1 (Appendix C) and the iterate-averaging special case
# (Sec. 3.2 "DEF-A", Eq. (12); Appendix C first displays).
# --------------------------------------------------------------------------- #
def test_single_worker_lemma_x_chases_sgd_path():
    """P7a: for K=1, x_{t+1} = x_t + C_t(y_{t+1} - x_t) with {y_t} the plain SGD
    path y_{t+1} = y_t - eta*g_t."""
    d, R, T, lr = 24, 5, 20, 0.2
    rng = np.random.default_rng(31)
    x0 = rng.standard_normal(d)
    o = make("np64", x0, 1, R, lr, 0.0, 0.0, seed=3)
    y = x0.copy()
    x = x0.copy()
    for t in range(T):
        g = rng.standard_normal((1, d))
        s = o.step(g)
        y = y - lr * g[0]
        keep = np.zeros(d, bool)
        keep[[(s + j) % d for j in range(o.B)]] = True
        x = x + np.where(keep, y - x, 0.0)
        assert np.allclose(o.x, x, rtol=1e-12, atol=1e-13)
        assert np.allclose(o.y(), y, rtol=1e-12, atol=1e-13)


def test_scaling_compressor_gives_iterate_averaging():
    """P7b: K=1 with the (oracle-only) compressor C(D)=delta*D turns x_t into
    the exponential average (1-delta)^t y_0 + sum_{t'} delta(1-delta)^{t-t'} y_{t'}
    of the SGD path."""
    d, T, lr, delta = 10, 25, 0.1, 0.3
    rng = np.random.default_rng(41)
    x0 = rng.standard_normal(d)
    o = DefOracle(x0, 1, 1, lr, 0.0, 0.0, 0, dtype=np.float64,
                  compressor=lambda p, t: delta * p)
    ys = [x0.copy()]
    for t in range(T):
        g = rng.standard_normal((1, d))
        o.step(g)
        ys.append(ys[-1] - lr * g[0])
        tt = t + 1
        ref = (1 - delta) ** tt * ys[0] + sum(delta * (1 - delta) ** (tt - u) * ys[u]
                                              for u in range(1, tt + 1))
        assert np.allclose(o.x, ref, rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------- #
# Detached evaluation points (Algorithm 1, "detach" line; Sec. 3.2 items (1)-(3);
# Appendix A, first display).
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kind", KINDS)
def test_detached_points_special_cases(kind):
    """lambda = 0 is plain error feedback (gradient at x); K = 1 with lambda = 1
    evaluates at y = x - e, the SGD path (Sec. 3.2, text after Eq. (8))."""
    d, R, T = 41, 6, 9
    rng = np.random.default_rng(91)
    many = make(kind, rng.standard_normal(d), 3, R, 0.2, 0.9, 0.0, seed=12)
    one = make(kind, rng.standard_normal(d), 1, R, 0.2, 0.9, 0.0, seed=12)
    for t in range(T):
        many.step(rng.standard_normal((3, d)).astype(np.float32))
        one.step(rng.standard_normal((1, d)).astype(np.float32))
    w0 = np.asarray(many.detached_points(0.0))
    assert w0.shape == (3, d)
    for k in range(3):
        assert np.array_equal(w0[k], np.asarray(many.x))
    assert np.array_equal(np.asarray(one.detached_points(1.0))[0], np.asarray(one.y()))
    assert np.asarray(many.e).any()


def test_detached_points_distance_identity():
    """(1/K) sum_k ||w_k - y||^2 = (1/K) sum_k ||e_t - lambda e_k||^2
    = lambda^2 * mean_k||e_k||^2 - 2 lambda ||e_t||^2 + ||e_t||^2  with e_t the mean
    error (Sec. 3.2, Eq. (9); Appendix A, first display), and lambda*(t) =
    ||e_t||^2 / mean_k||e_k||^2 minimises it."""
    d, W, R, T = 60, 5, 7, 14
    rng = np.random.default_rng(92)
    o = make("np64", rng.standard_normal(d), W, R, 0.1, 0.9, 0.0, seed=3)
    for t in range(T):
        o.step(rng.standard_normal((W, d)))
    e_bar = o.e.mean(axis=0)
    mean_sq = float((o.e ** 2).sum(axis=1).mean())
    bar_sq = float((e_bar ** 2).sum())
    assert mean_sq > 0 and bar_sq > 0

    def dist(lam):
        return float(((o.detached_points(lam) - o.y()[None, :]) ** 2).sum(axis=1).mean())

    for lam in (0.0, 0.3, 0.7, 1.0):
        assert dist(lam) == pytest.approx(lam * lam * mean_sq - 2 * lam * bar_sq + bar_sq, rel=1e-11)
    lam_star = bar_sq / mean_sq
    assert 0.0 < lam_star < 1.0
    assert dist(lam_star) <= min(dist(lam_star - 1e-3), dist(lam_star + 1e-3))
    assert dist(lam_star) == pytest.approx(bar_sq * (mean_sq - bar_sq) / mean_sq, rel=1e-10)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_diagnostics_against_norms_of_detached_points(dtype):
    """The statistics of Sec. 3.2 computed another way: distances between the
    detached points and y with numpy's norm; lambda*(t) as the vertex of the
    parabola through three of those distances; W = 1 gives lambda* = 1, dist(1) = 0."""
    d, W, R, T = 70, 4, 6, 12
    rng = np.random.default_rng(94)
    o = DefOracle(rng.standard_normal(d), W, R, 0.1, 0.9, 0.0, 5, dtype=dtype)
    for t in range(T):
        o.step(rng.standard_normal((W, d)))
    e64 = o.e.astype(np.float64)
    x64 = o.x.astype(np.float64)
    y64 = x64 - e64.mean(axis=0)

    def dist_by_norm(lam):
        return float(np.mean([np.linalg.norm((x64 - lam * e64[k]) - y64) ** 2 for k in range(W)]))

    for lam in (0.0, 0.3, 1.0):
        dg = o.diagnostics(lam)
        assert dg["dist"] == pytest.approx(dist_by_norm(lam), rel=1e-11)
        assert dg["bar_sq"] == pytest.approx(np.linalg.norm(x64 - y64) ** 2, rel=1e-11)
        assert dg["mean_sq"] == pytest.approx(np.mean(np.linalg.norm(e64, axis=1) ** 2), rel=1e-11)
    d0, d1, d2 = dist_by_norm(0.0), dist_by_norm(1.0), dist_by_norm(2.0)
    a2 = (d2 - 2 * d1 + d0) / 2.0
    a1 = d1 - d0 - a2
    assert o.diagnostics(0.3)["lam_star"] == pytest.approx(-a1 / (2 * a2), rel=1e-9)
    one = DefOracle(rng.standard_normal(d), 1, R, 0.1, 0.9, 0.0, 5, dtype=dtype)
    for t in range(5):
        one.step(rng.standard_normal((1, d)))
    dg = one.diagnostics(1.0)
    assert dg["lam_star"] == pytest.approx(1.0, rel=1e-12) and dg["dist"] == 0.0
    fresh = DefOracle(np.zeros(d), 2, R, 0.1, dtype=dtype).diagnostics(0.3)
    assert fresh == dict(bar_sq=0.0, mean_sq=0.0, lam_star=0.0, dist=0.0)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_per_worker_statistics(dtype):
    """Sec. 3.2 item (1) / Appendix A, first display: lambda*(k,t) = <e_t, e_k>/||e_k||^2
    is the lambda at which worker k's own evaluation point x - lambda*e_k is closest to
    y.  Checked without the formula: worker k's squared distance to y, measured with
    numpy's norm at three lambdas, is a parabola whose vertex must be lambda*(k,t) and
    whose curvature must be ||e_k||^2; the workers' inner products average to
    ||e_t||^2 = ||x - y||^2; one worker alone gives lambda* = 1."""
    d, W, R, T = 70, 4, 6, 12
    rng = np.random.default_rng(95)
    o = DefOracle(rng.standard_normal(d), W, R, 0.1, 0.9, 0.0, 5, dtype=dtype)
    for t in range(T):
        o.step(rng.standard_normal((W, d)))
    e64 = o.e.astype(np.float64)
    x64 = o.x.astype(np.float64)
    y64 = x64 - e64.mean(axis=0)
    pw = o.diagnostics_workers()
    assert pw["norm_sq"].shape == pw["inner"].shape == pw["lam_star"].shape == (W,)

    def dist_k(k, lam):
        return float(np.linalg.norm((x64 - lam * e64[k]) - y64) ** 2)

    for k in range(W):
        d0, d1, d2 = dist_k(k, 0.0), dist_k(k, 1.0), dist_k(k, 2.0)
        a2 = (d2 - 2 * d1 + d0) / 2.0
        a1 = d1 - d0 - a2
        vertex = -a1 / (2 * a2)
        assert pw["lam_star"][k] == pytest.approx(vertex, rel=1e-9), k
        assert pw["norm_sq"][k] == pytest.approx(a2, rel=1e-9), k
        assert pw["norm_sq"][k] == pytest.approx(np.linalg.norm(e64[k]) ** 2, rel=1e-11), k
        assert pw["inner"][k] == pytest.approx(-a1 / 2.0, rel=1e-9), k
        best = dist_k(k, pw["lam_star"][k])
        assert best <= min(dist_k(k, pw["lam_star"][k] - 1e-3), dist_k(k, pw["lam_star"][k] + 1e-3))
    assert len(set(np.round(pw["lam_star"], 12))) == W          # the workers differ
    assert np.mean(pw["inner"]) == pytest.approx(np.linalg.norm(x64 - y64) ** 2, rel=1e-11)
    one = DefOracle(rng.standard_normal(d), 1, R, 0.1, 0.9, 0.0, 5, dtype=dtype)
    for t in range(5):
        one.step(rng.standard_normal((1, d)))
    p1 = one.diagnostics_workers()
    assert p1["lam_star"][0] == pytest.approx(1.0, rel=1e-12) and p1["inner"][0] == p1["norm_sq"][0] > 0
    fresh = DefOracle(np.zeros(d), 2, R, 0.1, dtype=dtype).diagnostics_workers()
    assert not fresh["norm_sq"].any() and not fresh["inner"].any() and not fresh["lam_star"].any()


def test_error_memory_stationary_moments_and_bounds():
    """Gradients g_k = c + noise_k that do not depend on x (mu = 0): an index that
    was last kept `a` steps ago holds e_k = eta*(a*c + sum of a noise terms).  With
    uniform circular starts every index is kept with probability delta = B/d
    independently per step (Assumption 4.2 with equality), so the age is geometric,
    E[a] = (1-delta)/delta and E[a^2] = (1-delta)(2-delta)/delta^2, which gives
      E (1/K) sum_k ||e_k||^2        = eta^2 [sigma^2 E[a] + M^2 E[a^2]]
      E (1/K) sum_k ||e_t - lam e_k||^2 = eta^2 [B1 sigma^2 E[a] + (1-lam)^2 M^2 E[a^2]]
    with sigma^2 = E||noise||^2, M^2 = ||c||^2, B1 = (1/K - lam)^2 + (K-1)/K^2 (the
    constant of Lemma A.2).  Time averages over a long run are checked against these
    values, and against the upper bounds of Lemma A.3 and Lemma A.2 (Appendix A)."""
    d, W, R, eta, T, burn = 240, 4, 8, 0.1, 6000, 300
    delta = block_length(d, R) / d
    rng = np.random.default_rng(20)
    c = rng.standard_normal(d) * 0.05
    sig_g = 0.2
    M2, sigma2 = float(c @ c), d * sig_g ** 2
    Ea, Ea2 = (1 - delta) / delta, (1 - delta) * (2 - delta) / delta ** 2
    lams = (0.0, 0.3, 1.0)
    o = DefOracle(np.zeros(d), W, R, eta, 0.0, 0.0, 77, dtype=np.float64)
    acc = {lam: [] for lam in lams}
    mean_sq, bar_sq = [], []
    for t in range(T):
        o.step(c[None, :] + sig_g * rng.standard_normal((W, d)))
        if t >= burn:
            for lam in lams:
                acc[lam].append(o.diagnostics(lam)["dist"])
            dg = o.diagnostics(0.0)
            mean_sq.append(dg["mean_sq"])
            bar_sq.append(dg["bar_sq"])
    want_mean = eta ** 2 * (sigma2 * Ea + M2 * Ea2)
    assert np.mean(mean_sq) == pytest.approx(want_mean, rel=0.04)
    # Lemma A.3: (1/K) sum_k E||e_k||^2 <= eta^2 (sigma^2 + M^2) / (sqrt(1/(1-delta)) - 1)^2
    assert np.mean(mean_sq) <= eta ** 2 * (sigma2 + M2) / (np.sqrt(1 / (1 - delta)) - 1) ** 2
    for lam in lams:
        B1 = (1.0 / W - lam) ** 2 + (W - 1) / W ** 2
        want = eta ** 2 * (B1 * sigma2 * Ea + (1 - lam) ** 2 * M2 * Ea2)
        assert np.mean(acc[lam]) == pytest.approx(want, rel=0.04), lam
        # Lemma A.2 with L = 0
        cap = eta ** 2 * (B1 * sigma2 + 2 * (1 - lam) ** 2 * M2) / \
            (np.sqrt((1 - delta / 2) / (1 - delta)) - 1) ** 2
        assert np.mean(acc[lam]) <= cap, lam
    # lambda = 0 is error feedback: the distance is ||e_t||^2 itself
    assert np.mean(acc[0.0]) == pytest.approx(np.mean(bar_sq), rel=1e-12)


@pytest.mark.parametrize("kind,tol", [("np64", 1e-12), ("np32", 2e-5), ("c32", 2e-5)])
def test_closed_loop_single_worker_follows_gradient_descent(kind, tol):
    """K = 1, lambda = 1 on f(theta) = 0.5*||theta - c||^2 with the gradient taken at
    the detached point: y_t must be exact gradient descent whatever the compressor
    drops, y_t = c + (1 - eta)^t (y_0 - c)  (Sec. 3.2: for K = 1, lambda = 1 the
    sequence {y_t} is the SGD solution path)."""
    d, R, T, lr = 30, 5, 25, 0.2
    rng = np.random.default_rng(93)
    c = rng.standard_normal(d)
    y0 = rng.standard_normal(d)
    o = make(kind, y0, 1, R, lr, 0.0, 0.0, seed=21)
    y0s = np.asarray(o.x, dtype=np.float64).copy()
    for t in range(T):
        w = np.asarray(o.detached_points(1.0), dtype=np.float64)
        o.step((w - c[None, :]).astype(np.float32 if kind != "np64" else np.float64))
        ref = c + (1 - lr) ** (t + 1) * (y0s - c)
        assert np.allclose(np.asarray(o.y(), dtype=np.float64), ref, rtol=tol, atol=tol), t
    assert np.abs(np.asarray(o.e)).max() > 1e-3      # the compressor did drop something


# --------------------------------------------------------------------------- #
# Integer closed form (follows from Algorithm 1 with g = 1, eta = 1).
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("d,R,W", [(29, 4, 3), (32, 8, 1), (11, 11, 2), (20, 3, 4)])
def test_age_counter_closed_form(kind, d, R, W):
    """P8: g=1, eta=1, mu=0, wd=0, x_0=0: the error memory counts the steps since
    an index was last sent (t if never) and x_t[i] = -(t - age_t(i)).  Only small
    integers occur, so this is exact; it checks indices, wrap, zeroing and the
    update without any rounding."""
    T = 40
    o = make(kind, np.zeros(d), W, R, 1.0, 0.0, 0.0, seed=123)
    age = [0] * d
    xs = [0] * d
    B = block_length(d, R)
    ones = np.ones((W, d), np.float32)
    for t in range(T):
        forced = (d - 1) if t % 7 == 3 else None
        s = o.step(ones, start=forced)
        assert s == (forced if forced is not None else block_start(123, t, d))
        kept = {(s + j) % d for j in range(B)}
        # the averaged block in compact order: entry j belongs to index (s+j) mod d and
        # is 1 + the age that index had before this step
        assert [int(v) for v in np.asarray(o.compact_block())] == [age[(s + j) % d] + 1 for j in range(B)]
        for i in range(d):
            if i in kept:
                xs[i] -= age[i] + 1
                age[i] = 0
            else:
                age[i] += 1
        assert [int(v) for v in np.asarray(o.x)] == xs
        for k in range(W):
            assert [int(v) for v in np.asarray(o.e)[k]] == age
        assert all(xs[i] == -((t + 1) - age[i]) for i in range(d))


# --------------------------------------------------------------------------- #
# Brute force on tiny problems.
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kind", KINDS)
def test_brute_force_every_start_and_ratio(kind):
    """P9: dense per-element evaluation of Algorithm 1 + momentum for d<=16,
    every ratio R in 1..d and every start (all wrap positions), two chained
    steps so that non-zero e and m enter the second one.  Bit-exact."""
    rng = np.random.default_rng(51)
    dt = np.float64 if kind == "np64" else np.float32
    for d, W, mu, wd in [(7, 2, 0.9, 0.0), (12, 3, 0.5, 1e-2), (16, 1, 0.0, 0.0), (5, 4, 0.0, 0.3)]:
        x0 = rng.standard_normal(d).astype(dt)
        g1 = rng.standard_normal((W, d)).astype(np.float32)
        g2 = rng.standard_normal((W, d)).astype(np.float32)
        for R in range(1, d + 1):
            B = block_length(d, R)
            for s1, s2 in itertools.product(range(d), [0, d // 2, d - 1]):
                o = make(kind, x0, W, R, 0.3, mu, wd, seed=0)
                o.step(g1, start=s1)
                o.step(g2, start=s2)
                x, e, m = list(x0), [[dt(0)] * d for _ in range(W)], [[dt(0)] * d for _ in range(W)]
                x, e, m, _ = brute_force_step(x, e, m, g1, s1, B, 0.3, mu, wd, dt)
                x, e, m, cb = brute_force_step(x, e, m, g2, s2, B, 0.3, mu, wd, dt)
                assert np.array_equal(bits(np.asarray(o.x)), bits(np.array(x, dtype=dt)))
                assert np.array_equal(bits(np.asarray(o.e)), bits(np.array(e, dtype=dt)))
                if mu != 0:
                    assert np.array_equal(bits(np.asarray(o.m)), bits(np.array(m, dtype=dt)))
                assert np.array_equal(bits(np.asarray(o.last_cbar_dense)), bits(np.array(cb, dtype=dt)))


@pytest.mark.parametrize("kind", KINDS32)
def test_brute_force_d64_seeded(kind):
    rng = np.random.default_rng(52)
    d, W, R, T = 64, 4, 5, 12
    x0 = rng.standard_normal(d).astype(np.float32)
    o = make(kind, x0, W, R, 0.1, 0.9, 1e-3, seed=99)
    x, e, m = list(x0), [[np.float32(0)] * d for _ in range(W)], [[np.float32(0)] * d for _ in range(W)]
    for t in range(T):
        g = (rng.standard_normal((W, d)) * 0.1).astype(np.float32)
        s = o.step(g)
        x, e, m, _ = brute_force_step(x, e, m, g, s, o.B, 0.1, 0.9, 1e-3)
    assert np.array_equal(bits(np.asarray(o.x)), bits(np.array(x, dtype=np.float32)))
    assert np.array_equal(bits(np.asarray(o.e)), bits(np.array(e, dtype=np.float32)))
    assert np.array_equal(bits(np.asarray(o.m)), bits(np.array(m, dtype=np.float32)))


# --------------------------------------------------------------------------- #
# Column subsets and checkpoints.
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kind", KINDS32)
def test_column_subset_equals_full_run(kind):
    """Columns evolve independently given the blocks, so simulating a subset of
    global indices must reproduce those columns of the full run bit-for-bit."""
    d, W, R, T = 211, 3, 9, 25
    rng = np.random.default_rng(61)
    x0 = rng.standard_normal(d).astype(np.float32)
    cols = np.sort(rng.choice(d, size=40, replace=False))
    cols[0], cols[-1] = 0, d - 1
    full = make(kind, x0, W, R, 0.1, 0.9, 1e-3, seed=5)
    part = make(kind, x0[cols], W, R, 0.1, 0.9, 1e-3, seed=5, d=d, index=cols)
    for t in range(T):
        g = rng.standard_normal((W, d)).astype(np.float32)
        assert full.step(g) == part.step(np.ascontiguousarray(g[:, cols]))
    assert np.array_equal(bits(np.asarray(full.x)[cols]), bits(np.asarray(part.x)))
    assert np.array_equal(bits(np.asarray(full.e)[:, cols]), bits(np.asarray(part.e)))
    assert np.array_equal(bits(np.asarray(full.m)[:, cols]), bits(np.asarray(part.m)))
    assert np.array_equal(bits(np.asarray(full.y())[cols]), bits(np.asarray(part.y())))


@pytest.mark.parametrize("kind", KINDS32)
def test_checkpoint_resume_is_bit_identical(kind):
    """P10: (x, e, m, seed, t, eta) is the whole state."""
    d, W, R, T = 83, 3, 6, 16
    rng = np.random.default_rng(71)
    x0 = rng.standard_normal(d).astype(np.float32)
    G = rng.standard_normal((T, W, d)).astype(np.float32)
    a = make(kind, x0, W, R, 0.1, 0.9, 0.0, seed=8)
    for t in range(T):
        a.step(G[t])
        if t == 6:
            st = a.get_state()
    b = make(kind, np.zeros(d), W, R, 0.7, 0.9, 0.0, seed=1)
    b.set_state(st)
    for t in range(7, T):
        b.step(G[t])
    for n in "xem":
        assert np.array_equal(bits(np.asarray(getattr(a, n))), bits(np.asarray(getattr(b, n))))


def test_numpy_and_c_oracles_agree_bitwise():
    d, W, R, T = 1000, 5, 7, 30
    rng = np.random.default_rng(81)
    x0 = rng.standard_normal(d).astype(np.float32) * 0.05
    a = make("np32", x0, W, R, 0.1, 0.9, 1e-4, seed=6)
    b = make("c32", x0, W, R, 0.1, 0.9, 1e-4, seed=6)
    for t in range(T):
        g = (rng.standard_t(3, size=(W, d)) * 1e-3).astype(np.float32)
        assert a.step(g) == b.step(g)
    for n in "xem":
        assert np.array_equal(bits(np.asarray(getattr(a, n))), bits(np.asarray(getattr(b, n))))
    assert np.array_equal(bits(a.y()), bits(b.y()))
    assert np.array_equal(bits(a.compact_block()), bits(b.compact_block()))
    # detached points, lambda neither 0 nor 1 and W > 1, so that every row and the scale matter
    # (the numpy side is pinned by the special cases, the distance identity and its mutants)
    wa, wb = a.detached_points(0.3), b.detached_points(0.3)
    assert wa.shape == wb.shape == (W, d)
    assert np.array_equal(bits(wa), bits(wb))
    assert len({wa[k].tobytes() for k in range(W)}) == W


def test_tiny_workload_digest_unchanged():
    """The stored digests were written by tests/golden/make_tiny_digest.py from
    the oracle alone; a change to oracle arithmetic or input recipe shows here."""
    import os
    from tests.golden.make_tiny_digest import digest_lines
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_digest.txt")
    assert open(path).read().split("\n")[:-1] == digest_lines()
