"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on identical seeded inputs.  Every test here needs a real MI355X."""
from __future__ import annotations

import numpy as np
import pytest

from oracle.c_oracle import DefOracleC
from oracle.def_oracle import DefOracle
from paper_2004_05298_amd import workloads as wl
from tests.parity import assert_close, bit_equal, bits, in_block_mask

pytestmark = pytest.mark.gpu

# the C ABI takes lambda as a float: the oracle is given the same binary32 value
LAM32 = float(np.float32(0.3))

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    torch.cuda.set_device(0)
    return torch.device("cuda:0")


def _binding():
    from paper_2004_05298_amd import binding
    binding.load_library()          # raises if the HIP library is not built: no fallback
    return binding


def ora_diag(ora, lam):
    """Statistics of the oracle's error memories; the C oracle holds the same arrays,
    so the numpy oracle's routine is applied to them."""
    if hasattr(ora, "diagnostics"):
        return ora.diagnostics(lam)
    return DefOracle.diagnostics(ora, lam)


def fetch_state(ctx, W, d):
    torch.cuda.synchronize()
    e, m, _ = ctx.state_tensors()
    return e.cpu().numpy(), (m.cpu().numpy() if m is not None else None), e.shape[1]


def fetch_avg(ctx):
    torch.cuda.synchronize()
    return ctx.state_tensors()[2].cpu().numpy()


def run_case(dev, w, *, weight_decay=None, momentum=None, T=None, flat_params=True,
             mode="flat", misalign=0, ld=None, oracle="np", check_every_step=True,
             with_y=True, special=None, variant=None, forced=None, detach=None, ldw=None,
             split=False):
    """Run T steps on both sides and compare.  mode: "flat" (one gradient buffer
    [W][ld]) or "tensors" (one allocation per worker and tensor).  split: every
    iteration is def_pack followed by def_apply of the returned sum with divisor W."""
    binding = _binding()
    wd = w.weight_decay if weight_decay is None else weight_decay
    mu = w.momentum if momentum is None else momentum
    T = w.T if T is None else T
    variant = variant or w.variant
    d, W = w.d, w.W
    off = w.tensor_offsets()
    ld = wl.padded_ld(d) if ld is None else ld
    x0 = wl.initial_params(w)
    pool = [g[:, :d] for g in wl.gradient_pool(w, ld=d, threads=4)]
    if special is not None:
        special(pool, x0)

    # device inputs
    if flat_params:
        x_dev = torch.from_numpy(x0).to(dev)
        params, param_tensors = x_dev, None
    else:
        param_tensors = [torch.from_numpy(x0[int(off[l]):int(off[l + 1])].copy()).to(dev)
                         for l in range(w.n_tensors)]
        params = None
    if mode == "flat":
        gdev = []
        for g in pool:
            buf = torch.zeros(W * ld + 8, dtype=torch.float32, device=dev)
            view = buf[misalign:misalign + W * ld].view(W, ld)
            view[:, :d].copy_(torch.from_numpy(np.ascontiguousarray(g)))
            gdev.append((buf, view))
    else:
        gdev = []
        for g in pool:
            tensors = []
            for k in range(W):
                for l in range(w.n_tensors):
                    a, b = int(off[l]), int(off[l + 1])
                    # odd extra offset so that tensors start at every 4-byte alignment
                    pad = (k + l) % 4
                    buf = torch.zeros(b - a + pad, dtype=torch.float32, device=dev)
                    buf[pad:].copy_(torch.from_numpy(np.ascontiguousarray(g[k, a:b])))
                    tensors.append(buf[pad:])
            gdev.append(tensors)
    y_dev = torch.full((d,), float("nan"), dtype=torch.float32, device=dev)
    w_dev = None
    if detach is not None:
        ldw = wl.padded_ld(d) if ldw is None else ldw
        w_dev = torch.full((W, ldw), float("nan"), dtype=torch.float32, device=dev)

    if oracle == "np":
        ora = DefOracle(x0, W, w.R, w.lr, mu, wd, w.seed)
    else:
        ora = DefOracleC(x0, W, w.R, w.lr, mu, wd, w.seed)

    stream = torch.cuda.current_stream().cuda_stream
    ctx = binding.DefContext(d, W, w.R, w.lr, mu, wd, w.seed, params=params,
                             param_tensors=param_tensors, tensor_offsets=off, stream=stream)
    exact = {}
    try:
        e_ptr, m_ptr, a_ptr, ld_state = ctx.state_ptrs()
        assert ld_state >= d and ld_state % 256 == 0
        assert (m_ptr != 0) == (mu != 0)
        if detach is not None:
            ctx.set_detach(w_dev, ldw, detach)
            # the call itself writes the points of the current state: x_0 in every row
            torch.cuda.synchronize()
            assert bit_equal(w_dev.cpu().numpy()[:, :d], ora.detached_points(detach)), "w before the first step"
        for t in range(T):
            g_host = pool[t % w.pool]
            start = (forced or w.forced_start)(t)
            if start is not None:
                ctx.force_next_start(start)
            want_y = with_y and variant != "def_a" and (t == T - 1 or t == T // 2)
            if split:
                if mode == "flat":
                    block = ctx.pack(gdev[t % w.pool][1], ld)
                else:
                    block = ctx.pack_tensors(gdev[t % w.pool])
                assert block == ctx.state_ptrs()[2]
                ctx.apply(block, float(W), y_dev if want_y else None)
            elif mode == "flat":
                view = gdev[t % w.pool][1]
                if variant == "def_a":
                    ctx.a_step(view, ld)
                else:
                    ctx.step(view, ld, y_dev if want_y else None)
            else:
                if variant == "def_a":
                    ctx.a_step_tensors(gdev[t % w.pool])
                else:
                    ctx.step_tensors(gdev[t % w.pool], y_dev if want_y else None)
            s = ora.step(g_host, start=start)
            # integer results: bit-exact
            assert ctx.last_block() == (s, w.B), (t, ctx.last_block(), s, w.B)
            assert ctx.get_step() == t + 1
            if check_every_step or t == T - 1:
                torch.cuda.synchronize()
                avg = fetch_avg(ctx)
                assert_close(f"averaged block t={t}", avg, ora.compact_block())
                exact.setdefault("avg", True)
                exact["avg"] &= bit_equal(avg, ora.compact_block())
                e, m, _ = fetch_state(ctx, W, d)
                mask = in_block_mask(d, s, w.B)
                # error-memory zeroing: literal +0 inside the block, for every worker
                assert (bits(e[:, :d][:, mask]) == 0).all(), f"t={t}: block not zeroed"
                assert not e[:, d:].any(), "padding columns of e must stay zero"
                if detach is not None:
                    wg = w_dev.cpu().numpy()[:, :d]
                    assert_close(f"detached points t={t}", wg, ora.detached_points(detach))
                    exact.setdefault("w", True)
                    exact["w"] &= bit_equal(wg, ora.detached_points(detach))
                if want_y:
                    assert_close(f"y t={t}", y_dev.cpu().numpy(), ora.y())
                    exact.setdefault("y", True)
                    exact["y"] &= bit_equal(y_dev.cpu().numpy(), ora.y())
        torch.cuda.synchronize()
        if mode == "flat":
            reads_x = wd != 0 or detach is not None
            assert ctx.last_path_flat() == (flat_params or not reads_x)
        else:
            assert not ctx.last_path_flat()
        e, m, _ = fetch_state(ctx, W, d)
        if flat_params:
            x = x_dev.cpu().numpy()
        else:
            x = np.concatenate([p.cpu().numpy() for p in param_tensors])
        assert_close("x", x, ora.x)
        assert_close("e", e[:, :d], ora.e)
        assert np.array_equal(e[:, :d] == 0, ora.e == 0), "zero pattern of e differs"
        exact["x"], exact["e"] = bit_equal(x, ora.x), bit_equal(e[:, :d], ora.e)
        if mu != 0:
            assert_close("m", m[:, :d], ora.m)
            assert not m[:, d:].any()
            exact["m"] = bit_equal(m[:, :d], ora.m)
        if variant != "def_a":
            ctx.output(y_dev)
            torch.cuda.synchronize()
            assert_close("y (def_output)", y_dev.cpu().numpy(), ora.y())
        # error-memory statistics of the final state (float64 sums; only the order in which
        # columns are added differs from the oracle, so 1e-10 relative is ample; the
        # distance is formed from the other two and may lose digits to cancellation)
        if not (special is not None):
            diag = torch.full((4,), float("nan"), dtype=torch.float64, device=dev)
            ctx.diagnostics(0.3, diag)
            torch.cuda.synchronize()
            got, ref = diag.cpu().numpy(), ora_diag(ora, LAM32)
            scale = max(ref["mean_sq"], 1e-300)
            assert abs(got[0] - ref["bar_sq"]) <= 1e-10 * scale, (got, ref)
            assert abs(got[1] - ref["mean_sq"]) <= 1e-10 * scale, (got, ref)
            assert abs(got[2] - ref["lam_star"]) <= 1e-9, (got, ref)
            assert abs(got[3] - ref["dist"]) <= 1e-9 * scale, (got, ref)
            # the same per worker (same tolerances: float64 sums in another order)
            pw = torch.full((3 * W,), float("nan"), dtype=torch.float64, device=dev)
            ctx.diagnostics_workers(pw)
            torch.cuda.synchronize()
            pw = pw.cpu().numpy()
            refw = DefOracle.diagnostics_workers(ora)
            assert np.abs(pw[:W] - refw["norm_sq"]).max() <= 1e-10 * scale * W, (pw, refw)
            assert np.abs(pw[W:2 * W] - refw["inner"]).max() <= 1e-10 * scale * W, (pw, refw)
            assert np.abs(pw[2 * W:] - refw["lam_star"]).max() <= 1e-9, (pw, refw)
            assert abs(pw[W:2 * W].mean() - got[0]) <= 1e-10 * scale
        if detach is not None:
            # the stand-alone call, with another lambda, on the final state
            w2 = torch.full((W, d + 3), float("nan"), dtype=torch.float32, device=dev)
            ctx.detach(w2, d + 3, 0.75)
            torch.cuda.synchronize()
            assert_close("def_detach", w2.cpu().numpy()[:, :d], ora.detached_points(0.75))
            assert torch.isnan(w2[:, d:]).all(), "def_detach wrote past column d"
            if ldw > d:
                assert torch.isnan(w_dev[:, d:]).all(), "the step wrote w past column d"
    finally:
        ctx.destroy()
    print(f"[parity] {w.name} mode={mode} misalign={misalign} wd={wd} mu={mu} T={T}: bit-identical {exact}",
          flush=True)
    return exact


# --------------------------------------------------------------------------- #
# The tiny configuration, exactly as specified: d=65,536, W=4, R=16, T=10.
# --------------------------------------------------------------------------- #
def test_tiny_configuration(dev):
    w = wl.tiny()
    assert (w.d, w.W, w.R, w.B, w.T) == (65536, 4, 16, 4096, 10)
    exact = run_case(dev, w)
    assert all(exact.values()), exact


# --------------------------------------------------------------------------- #
# Small relatives of the model-shaped configurations: ragged tensors, d not a
# multiple of 4, several tiles of 4096 elements plus a ragged tail.
# --------------------------------------------------------------------------- #
SHRUNK = [
    ("resnet56_shaped", 53018 + 2, 57, None, 12),
    ("resnet18_shaped", 40009, 62, None, 10),
    ("resnet50_shaped", 45057, 161, None, 10),
    ("vgg16_shaped", 70003, 32, None, 12),
]


@pytest.mark.parametrize("name,d,L,W,T", SHRUNK, ids=[s[0] for s in SHRUNK])
def test_shrunk_model_shaped(dev, name, d, L, W, T):
    base = wl.by_name(name)
    w = wl.shrunk(base, d=d, n_tensors=L, W=W, T=T, pool=min(base.pool, 4))
    exact = run_case(dev, w)
    assert exact["x"] and exact["e"] and exact.get("m", True), exact


@pytest.mark.parametrize("name,d,L,W,T", SHRUNK, ids=[s[0] for s in SHRUNK])
def test_shrunk_tensor_mode(dev, name, d, L, W, T):
    """Per-tensor gradient and parameter allocations through the offset table."""
    base = wl.by_name(name)
    w = wl.shrunk(base, d=d, n_tensors=L, W=min(base.W, 8), T=6, pool=2)
    exact = run_case(dev, w, mode="tensors", flat_params=False)
    assert exact["x"] and exact["e"], exact


@pytest.mark.parametrize("misalign,ld_extra", [(1, 0), (2, 3), (0, 1), (3, 2)])
def test_unaligned_flat_gradients(dev, misalign, ld_extra):
    base = wl.resnet50_shaped()
    w = wl.shrunk(base, d=30011, n_tensors=9, W=5, T=6, pool=2)
    exact = run_case(dev, w, misalign=misalign, ld=w.d + ld_extra)
    assert exact["x"] and exact["e"] and exact["m"], exact


def test_flat_gradients_with_tensor_params(dev):
    base = wl.resnet18_shaped()
    w = wl.shrunk(base, d=25003, n_tensors=11, W=6, T=6, pool=2)
    for wd in (0.0, 1e-3):
        exact = run_case(dev, w, flat_params=False, weight_decay=wd, variant="def")
        assert exact["x"] and exact["e"], exact


# --------------------------------------------------------------------------- #
# Degenerate shapes and hyper-parameters.
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("d,W,R", [
    (1, 1, 1), (3, 2, 3), (4, 3, 1), (5, 1, 2), (63, 4, 63), (64, 2, 64), (257, 33, 5),
    (4096, 17, 4096), (4097, 16, 1), (8191, 3, 2), (16384, 1, 7), (12289, 40, 3),
    (2000, 300, 7), (256, 2, 1), (512, 3, 2), (768, 5, 3),
])
def test_degenerate_shapes(dev, d, W, R):
    base = wl.tiny()
    w = wl.shrunk(base, d=d, n_tensors=min(3, d), W=W, R=R, T=5, pool=3)
    # steps 1 and 3: blocks that start exactly on a 256-index tile edge (if there is one)
    edge = 256 if d > 256 else 0
    exact = run_case(dev, w, weight_decay=1e-3, forced=lambda t: {1: edge, 3: (d - w.B) % d}.get(t))
    assert all(exact.values()), exact


@pytest.mark.parametrize("mu,wd", [(0.0, 0.0), (0.0, 1e-2), (0.9, 0.0), (0.5, 5e-4)])
@pytest.mark.parametrize("mode", ["flat", "tensors"])
def test_hyperparameter_paths(dev, mu, wd, mode):
    base = wl.resnet56_shaped()
    w = wl.shrunk(base, d=20001, n_tensors=7, W=3, T=8, pool=3)
    exact = run_case(dev, w, momentum=mu, weight_decay=wd, mode=mode,
                     flat_params=(mode == "flat"))
    assert exact["x"] and exact["e"], exact


@pytest.mark.parametrize("d,W,R", [(300, 3, 1), (1000, 40, 1), (5000, 2, 2), (66000, 9, 3), (257, 1, 257)])
def test_large_blocks_and_many_workers(dev, d, W, R):
    """Blocks that cover the whole vector (R = 1: every wave keeps all its elements, every
    step wraps) or a large part of it, more workers than the averaging kernel stages at a
    time, and a one-element block."""
    w = wl.shrunk(wl.tiny(), d=d, n_tensors=3 if d > 300 else 1, W=W, R=R, T=6, pool=3)
    exact = run_case(dev, w, momentum=0.9, weight_decay=1e-3, forced=lambda t: {2: d - 1, 3: d // 2}.get(t))
    assert all(exact.values()), exact


# --------------------------------------------------------------------------- #
# Detached evaluation points written in the same pass (Algorithm 1, "detach" line).
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("name,d,L,lam,mode,kw", [
    ("resnet50_shaped", 45057, 21, 0.3, "flat", {}),
    ("resnet18_shaped", 40009, 9, 0.3, "flat", {}),
    ("resnet56_shaped", 20001, 7, 1.0, "flat", dict(momentum=0.0)),
    ("vgg16_shaped", 30003, 5, 0.0, "flat", {}),
    ("resnet50_shaped", 30011, 9, 0.3, "flat", dict(misalign=1)),
    ("resnet50_shaped", 30011, 9, 0.5, "flat", dict(ldw=30011)),
    ("resnet18_shaped", 25003, 11, 0.3, "tensors", dict(flat_params=False)),
    ("resnet50_shaped", 25003, 11, 0.3, "tensors", dict(flat_params=False)),
], ids=["wd", "no-wd", "no-momentum-lam1", "lam0", "misaligned-g", "odd-ldw", "tensors", "tensors-wd"])
def test_detached_points_in_the_same_pass(dev, name, d, L, lam, mode, kw):
    base = wl.by_name(name)
    w = wl.shrunk(base, d=d, n_tensors=L, W=min(base.W, 6), T=8, pool=2)
    exact = run_case(dev, w, mode=mode, detach=lam, forced=lambda t: {2: d - 5, 5: 0}.get(t), **kw)
    assert exact["w"] and exact["x"] and exact["e"], exact


def test_detach_rejects_bad_arguments(dev):
    binding = _binding()
    d, W = 1000, 2
    x = torch.zeros(d, device=dev)
    wbuf = torch.zeros(W, 1024, device=dev)
    ctx = binding.DefContext(d, W, 4, 0.1, 0.9, 0.0, 1, params=x,
                             stream=torch.cuda.current_stream().cuda_stream)
    for call in (lambda: ctx.set_detach(wbuf, 999, 0.3), lambda: ctx.set_detach(wbuf, 1024, 1.5),
                 lambda: ctx.set_detach(wbuf, 1024, -0.1), lambda: ctx.set_detach(wbuf, 1024, float("nan")),
                 lambda: ctx.detach(None, 1024, 0.3), lambda: ctx.detach(wbuf.data_ptr() + 2, 1024, 0.3)):
        with pytest.raises(binding.DefError) as ei:
            call()
        assert ei.value.status == binding.DEF_EINVAL
    ctx.set_detach(wbuf, 1024, 0.3)
    ctx.set_detach(None)
    # not between the two halves of a split iteration
    g = torch.zeros(W, 1024, device=dev)
    block = ctx.pack(g, 1024)
    with pytest.raises(binding.DefError) as ei:
        ctx.set_detach(wbuf, 1024, 0.3)
    assert ei.value.status == binding.DEF_EINVAL
    ctx.apply(block, float(W))
    ctx.set_detach(wbuf, 1024, 0.3)
    ctx.destroy()


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for q in range(n):
        d = int(rng.choice([rng.integers(1, 300), rng.integers(300, 5000), rng.integers(5000, 40000)]))
        W = int(rng.integers(1, 20))
        R = int(rng.integers(1, min(d, 300) + 1))
        mu = float(rng.choice([0.0, 0.5, 0.9]))
        wd = float(rng.choice([0.0, 1e-3]))
        mode = str(rng.choice(["flat", "flat", "tensors"]))
        misalign = int(rng.choice([0, 0, 1, 2, 3])) if mode == "flat" else 0
        detach = [None, 0.3, 1.0][int(rng.integers(0, 3))]
        L = int(rng.integers(1, min(d, 9) + 1))
        cases.append((q, d, W, R, mu, wd, mode, misalign, detach, L))
    return cases


@pytest.mark.parametrize("q,d,W,R,mu,wd,mode,misalign,detach,L", _random_cases(24, 20040529),
                         ids=lambda v: str(v))
def test_seeded_random_shapes(dev, q, d, W, R, mu, wd, mode, misalign, detach, L):
    """A seeded draw of shapes and options: sizes around and below one tile, odd
    worker counts, every gradient alignment, both modes, with and without the
    detached points."""
    w = wl.shrunk(wl.tiny(), d=d, n_tensors=L, W=W, R=R, T=5, pool=3)
    starts = {1: d - 1, 3: max(0, d - w.B)}               # a wrapped block and one ending at d-1
    exact = run_case(dev, w, momentum=mu, weight_decay=wd, mode=mode, misalign=misalign,
                     flat_params=(mode == "flat"), detach=detach, forced=lambda t: starts.get(t))
    assert exact["x"] and exact["e"], exact


def test_every_wrap_position_small(dev):
    """Force each start of a small problem in turn (all wrap positions)."""
    base = wl.tiny()
    w = wl.shrunk(base, d=37, n_tensors=3, W=3, R=5, T=37, pool=4)

    exact = run_case(dev, w, forced=lambda t: t)
    assert all(exact.values()), exact


def _plant_specials(pool, x0):
    g = pool[0]
    g[0, 0:8] = [np.nan, np.inf, -np.inf, -0.0, 1e-45, -1e-45, 3e-39, 1e38]
    g[1, 100:104] = [-0.0, -0.0, 1e-42, -1e-42]
    pool[1][0, 5] = np.float32(1e-40)


def test_special_values_and_denormals(dev):
    """NaN, infinities, signed zeros and denormal gradients: the block must still
    be the literal +0 and denormals must not be flushed."""
    base = wl.tiny()
    w = wl.shrunk(base, d=5000, n_tensors=2, W=2, R=4, T=4, pool=2)
    forced = lambda t: {0: 0, 1: 4990}.get(t)   # the planted values sit inside these blocks
    # run_case compares with the tolerance rule, which requires identical NaN and
    # infinity patterns; NaN payload bits are not compared
    run_case(dev, w, special=_plant_specials, momentum=0.0, weight_decay=0.0, forced=forced)
    run_case(dev, w, special=_plant_specials, forced=forced)


def test_set_seed_lr_step_and_resume(dev):
    """Seed, learning-rate and step-counter changes mid-run, and a resume from a
    checkpoint of (x, e, m, seed, t, eta) in a fresh context, follow the oracle."""
    binding = _binding()
    base = wl.resnet56_shaped()
    w = wl.shrunk(base, d=9001, n_tensors=4, W=3, T=12, pool=4)
    d, W = w.d, w.W
    ld = wl.padded_ld(d)
    x0 = wl.initial_params(w)
    pool = wl.gradient_pool(w, ld=ld, threads=1)
    gdev = [torch.from_numpy(g).to(dev) for g in pool]
    ora = DefOracle(x0, W, w.R, w.lr, w.momentum, 0.0, w.seed)
    x_dev = torch.from_numpy(x0).to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    ctx = binding.DefContext(d, W, w.R, w.lr, w.momentum, 0.0, w.seed, params=x_dev, stream=stream)
    for t in range(6):
        if t == 2:
            ctx.set_lr(0.01); ora.set_lr(0.01)
        if t == 4:
            ctx.set_seed(777); ora.set_seed(777)
        ctx.step(gdev[t % 4], ld)
        assert ctx.last_block()[0] == ora.step(pool[t % 4][:, :d])
    torch.cuda.synchronize()
    e, m, lds = fetch_state(ctx, W, d)
    x_ck = x_dev.clone()
    ctx.destroy()
    # fresh context, restore, continue
    x2 = x_ck.clone()
    ctx2 = binding.DefContext(d, W, w.R, 0.01, w.momentum, 0.0, 777, params=x2, stream=stream)
    e_view, m_view, _ = ctx2.state_tensors()
    assert e_view.shape[1] == lds
    e_view.copy_(torch.from_numpy(e).to(dev))
    m_view.copy_(torch.from_numpy(m).to(dev))
    ctx2.set_step(6)
    for t in range(6, 12):
        ctx2.step(gdev[t % 4], ld)
        assert ctx2.last_block()[0] == ora.step(pool[t % 4][:, :d])
    torch.cuda.synchronize()
    e2, m2, _ = fetch_state(ctx2, W, d)
    ctx2.destroy()
    assert bit_equal(x2.cpu().numpy(), ora.x)
    assert bit_equal(e2[:, :d], ora.e) and bit_equal(m2[:, :d], ora.m)


def test_tensor_mode_with_an_unchanged_pointer_table(dev):
    """The same gradient tensors every step: the device copy of the pointer table is
    uploaded once and reused."""
    base = wl.resnet56_shaped()
    w = wl.shrunk(base, d=9001, n_tensors=5, W=3, T=5, pool=1)
    exact = run_case(dev, w, mode="tensors", flat_params=False)
    assert exact["x"] and exact["e"], exact


def test_tensor_mode_cycling_through_more_tables_than_are_cached(dev):
    """Six distinct gradient sets with four device slots: tables are evicted and
    uploaded again while steps are in flight."""
    base = wl.resnet56_shaped()
    w = wl.shrunk(base, d=7001, n_tensors=6, W=3, T=14, pool=6)
    exact = run_case(dev, w, mode="tensors", flat_params=False, check_every_step=False)
    assert exact["x"] and exact["e"], exact


def test_a_problem_that_does_not_fit_reports_out_of_memory(dev):
    """hipMalloc failure surfaces as DEF_ENOMEM, leaves no context behind, and the
    library keeps working afterwards."""
    binding = _binding()
    x = torch.zeros(16, device=dev)
    with pytest.raises(binding.DefError) as ei:
        binding.DefContext(2**36, 2, 4, 0.1, 0.9, 0.0, 1, params=x,          # 512 GiB per state buffer
                           stream=torch.cuda.current_stream().cuda_stream)
    assert ei.value.status == binding.DEF_ENOMEM
    w = wl.shrunk(wl.tiny(), d=999, n_tensors=2, W=2, T=3, pool=2)
    exact = run_case(dev, w)
    assert all(exact.values()), exact


def test_invalid_arguments_change_nothing(dev):
    binding = _binding()
    d, W = 1000, 2
    x = torch.zeros(d, device=dev)
    g = torch.ones(W, 1024, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    ctx = binding.DefContext(d, W, 4, 0.1, 0.9, 0.0, 1, params=x, stream=stream)
    for call in (lambda: ctx.step(None, 1024), lambda: ctx.step(g, 999),
                 lambda: ctx.step(g.data_ptr() + 2, 1024), lambda: ctx.force_next_start(d),
                 lambda: ctx.output(None), lambda: ctx.last_block()):
        with pytest.raises(binding.DefError) as ei:
            call()
        assert ei.value.status == binding.DEF_EINVAL
    assert ctx.get_step() == 0
    ctx.step(g, 1024)
    torch.cuda.synchronize()
    assert ctx.get_step() == 1
    ctx.destroy()


# --------------------------------------------------------------------------- #
# The iteration in two halves (workers spread over several GPUs)
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("mode,flat_params,wd,mu,detach", [
    ("flat", True, 1e-4, 0.9, None),
    ("flat", True, 0.0, 0.0, LAM32),
    ("flat", True, 1e-3, 0.9, LAM32),
    ("tensors", False, 1e-4, 0.9, None),
])
def test_pack_then_apply_is_the_step(dev, mode, flat_params, wd, mu, detach):
    """def_pack + def_apply(own sum, divisor W) must equal def_step, hence the oracle, bit for bit."""
    w = wl.shrunk(wl.by_name("resnet56_shaped"), 30011, 9, T=8)
    exact = run_case(dev, w, weight_decay=wd, momentum=mu, T=8, mode=mode, flat_params=flat_params,
                     detach=detach, split=True)
    assert all(exact.values()), exact


@pytest.mark.parametrize("groups,per_group,wd", [(2, 1, 0.0), (2, 1, 1e-3), (2, 4, 0.0), (3, 2, 1e-3)])
def test_worker_groups_with_a_summed_block_match_the_full_oracle(dev, groups, per_group, wd):
    """The deployment of Sec. 5 on one device: `groups` contexts stand for GPUs, each with
    `per_group` workers and its own replica of x; the blocks def_pack returns are added
    (the stand-in for the all-reduce) and every context applies the sum with divisor
    W = groups*per_group.  The oracle runs all W workers in one place.  With one worker per
    group and two groups the sum a + b is the oracle's own ((+0 + a) + b): bit-identical;
    otherwise the groups' partial sums associate differently and the 1e-6 tolerance applies."""
    binding = _binding()
    W = groups * per_group
    base = wl.shrunk(wl.by_name("resnet56_shaped"), 20021, 7)
    d, ld, R, T = base.d, wl.padded_ld(base.d), base.R, 10
    rng = np.random.default_rng(1234)
    x0 = wl.initial_params(base)
    grads = [(rng.standard_normal((W, d)) * 1e-2).astype(np.float32) for _ in range(3)]
    ora = DefOracle(x0, W, R, base.lr, 0.9, wd, base.seed)
    stream = torch.cuda.current_stream().cuda_stream
    xs = [torch.from_numpy(x0).to(dev) for _ in range(groups)]
    ctxs = [binding.DefContext(d, per_group, R, base.lr, 0.9, wd, base.seed, params=xs[q], stream=stream)
            for q in range(groups)]
    gdev = []
    for g in grads:
        per = []
        for q in range(groups):
            buf = torch.zeros(per_group, ld, dtype=torch.float32, device=dev)
            buf[:, :d].copy_(torch.from_numpy(g[q * per_group:(q + 1) * per_group]))
            per.append(buf)
        gdev.append(per)
    try:
        for t in range(T):
            views = [ctxs[q].block_view(ctxs[q].pack(gdev[t % 3][q], ld)) for q in range(groups)]
            total = views[0].clone()
            for v in views[1:]:
                total = total + v
            for q in range(groups):
                ctxs[q].apply(total, float(W))
            s = ora.step(grads[t % 3])
            assert all(c.last_block() == (s, base.B) for c in ctxs)
        torch.cuda.synchronize()
        exact = groups == 2 and per_group == 1
        xg = [x.cpu().numpy() for x in xs]
        for q in range(1, groups):
            assert bit_equal(xg[q], xg[0])                 # replicas never diverge
        e = np.concatenate([c.state_tensors()[0].cpu().numpy()[:, :d] for c in ctxs])
        m = np.concatenate([c.state_tensors()[1].cpu().numpy()[:, :d] for c in ctxs])
        avg = ctxs[0].state_tensors()[2].cpu().numpy()
        assert_close("x", xg[0], ora.x)
        assert_close("e", e, ora.e)
        assert_close("m", m, ora.m)
        assert_close("averaged block", avg, ora.compact_block())
        mask = in_block_mask(d, ora.last_start, base.B)
        assert (bits(e[:, mask]) == 0).all()
        # DEF's output over all workers = the average of the groups' outputs (same x, equal group sizes)
        ys = []
        for c in ctxs:
            yq = torch.empty(d, dtype=torch.float32, device=dev)
            c.output(yq)
            ys.append(yq)
        torch.cuda.synchronize()
        y_all = (torch.stack(ys).double().mean(dim=0)).float().cpu().numpy()
        assert_close("y", y_all, ora.y())
        if exact or wd == 0.0:
            assert bit_equal(e, ora.e) and bit_equal(m, ora.m)   # x never enters e or m without decay
        if exact:
            assert bit_equal(xg[0], ora.x) and bit_equal(avg, ora.compact_block())
        print(f"[parity] {groups} groups x {per_group} workers wd={wd}: bit-identical x={bit_equal(xg[0], ora.x)} "
              f"e={bit_equal(e, ora.e)} m={bit_equal(m, ora.m)}", flush=True)
    finally:
        for c in ctxs:
            c.destroy()


def test_split_iteration_call_order_is_enforced(dev):
    binding = _binding()
    d, W = 1000, 2
    x = torch.zeros(d, device=dev)
    g = torch.ones(W, 1024, device=dev)
    ctx = binding.DefContext(d, W, 4, 0.1, 0.9, 0.0, 1, params=x, stream=torch.cuda.current_stream().cuda_stream)
    try:
        with pytest.raises(binding.DefError):
            ctx.apply(x, 2.0)                              # nothing packed
        block = ctx.pack(g, 1024)
        for call in (lambda: ctx.step(g, 1024), lambda: ctx.pack(g, 1024), lambda: ctx.a_step(g, 1024),
                     lambda: ctx.apply(block, 0.0), lambda: ctx.apply(None, 2.0)):
            with pytest.raises(binding.DefError) as ei:
                call()
            assert ei.value.status == binding.DEF_EINVAL
        assert ctx.get_step() == 1
        ctx.apply(block, 2.0)
        ctx.step(g, 1024)
        torch.cuda.synchronize()
        assert ctx.get_step() == 2
    finally:
        ctx.destroy()
