"""GPU parity at the full sizes of the model-shaped configurations, in the launch
configuration the benchmark times (flat gradients, padded row stride).

The ResNet-56-, ResNet-18- and ResNet-50-shaped configurations (the last is the
one the benchmark is quoted on) are compared buffer for buffer with the plain C
oracle.  For the VGG-16-shaped one, whose oracle state alone would be 53 GB (and
17.7 GB per gradient set on the host), the oracle simulates a sample of columns
exactly (each column of (x, e, m) evolves independently once the block of every
step is known): random columns plus every tensor boundary, the ends of the
vector, and the edges of every step's block; whole-buffer properties (zeroing of
the last block, zero padding) are checked on the device.  The sampled check is
kept for the ResNet-50-shaped configuration as well.

The kernel instantiations that only large problems select (non-temporal accesses
and the residency cap, several super-tiles of the blocked order) are compared with
the oracle for every way of calling the step: per-tensor pointers, detached points
with and without momentum, the stand-alone detach kernel, and the two-halves form.
"""
from __future__ import annotations

import numpy as np
import pytest

from oracle.c_oracle import DefOracleC
from oracle.philox import block_start
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


def _ctx(w, x_dev):
    from paper_2004_05298_amd import binding
    binding.load_library()
    return binding.DefContext(w.d, w.W, w.R, w.lr, w.momentum, w.weight_decay, w.seed,
                              params=x_dev, tensor_offsets=w.tensor_offsets(),
                              stream=torch.cuda.current_stream().cuda_stream)


def _gpu_step(ctx, w, t, g, ld, y):
    start = w.forced_start(t)
    if start is not None:
        ctx.force_next_start(start)
    use_a = w.variant == "def_a" or (w.variant == "both" and t % 2 == 1)
    if use_a:
        ctx.a_step(g, ld)
    else:
        ctx.step(g, ld, y)
    return start


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["resnet56_shaped", "resnet18_shaped", "resnet50_shaped"])
def test_whole_buffers_against_c_oracle(dev, name):
    w = wl.by_name(name)
    print(f"[fullsize] {name}: whole buffers, T={w.T}", flush=True)
    d, W, ld = w.d, w.W, wl.padded_ld(w.d)
    x0 = wl.initial_params(w)
    host_pool = wl.gradient_pool(w, ld=ld, threads=16)
    dev_pool = [torch.from_numpy(g).to(dev) for g in host_pool]
    x = torch.from_numpy(x0).to(dev)
    y = torch.empty(d, dtype=torch.float32, device=dev)
    ora = DefOracleC(x0, W, w.R, w.lr, w.momentum, w.weight_decay, w.seed)
    ctx = _ctx(w, x)
    try:
        for t in range(w.T):
            last = t == w.T - 1
            start = _gpu_step(ctx, w, t, dev_pool[t % w.pool], ld, y if last else None)
            s = ora.step(host_pool[t % w.pool], start=start)
            assert ctx.last_block() == (s, w.B)
        torch.cuda.synchronize()
        assert ctx.last_path_flat()
        if name != "resnet56_shaped":
            # large state: the non-temporal, residency-capped instantiation
            assert "nt=1" in ctx.last_kernel() and "lds=8960" in ctx.last_kernel(), ctx.last_kernel()
        e, m, avg = ctx.state_tensors()
        e, m, avg = e.cpu().numpy(), m.cpu().numpy(), avg.cpu().numpy()
        xg = x.cpu().numpy()
        assert_close("x", xg, ora.x)
        assert_close("e", e[:, :d], ora.e)
        assert_close("m", m[:, :d], ora.m)
        assert_close("averaged block", avg, ora.compact_block())
        mask = in_block_mask(d, ora.last_start, w.B)
        assert (bits(e[:, :d][:, mask]) == 0).all()
        assert np.array_equal(e[:, :d] == 0, ora.e == 0)
        assert not e[:, d:].any() and not m[:, d:].any()
        if w.variant != "def_a":
            assert_close("y", y.cpu().numpy(), ora.y())
        else:
            ctx.output(y)
            torch.cuda.synchronize()
            assert_close("y", y.cpu().numpy(), ora.y())
        from oracle.def_oracle import DefOracle
        diag = torch.zeros(4, dtype=torch.float64, device=dev)
        ctx.diagnostics(0.3, diag)
        torch.cuda.synchronize()
        got, ref = diag.cpu().numpy(), DefOracle.diagnostics(ora, LAM32)
        assert abs(got[0] - ref["bar_sq"]) <= 1e-10 * ref["mean_sq"], (got, ref)
        assert abs(got[1] - ref["mean_sq"]) <= 1e-10 * ref["mean_sq"], (got, ref)
        assert abs(got[2] - ref["lam_star"]) <= 1e-9 and abs(got[3] - ref["dist"]) <= 1e-9 * ref["mean_sq"]
        print(f"[fullsize] {name}: lambda*(t)={got[2]:.4f} EF distance/DEF distance at 0.3 = {got[0] / got[3]:.3f}",
              flush=True)
        print(f"[fullsize] {name}: bit-identical x={bit_equal(xg, ora.x)} e={bit_equal(e[:, :d], ora.e)} "
              f"m={bit_equal(m[:, :d], ora.m)} avg={bit_equal(avg, ora.compact_block())}", flush=True)
        assert bit_equal(e[:, :d], ora.e) and bit_equal(m[:, :d], ora.m)
    finally:
        ctx.destroy()


@pytest.mark.timeout(600)
def test_thousand_steps_stay_bit_identical(dev):
    """A long run at the ResNet-56-shaped size: 1000 iterations cycling the gradient
    pool, with a learning-rate drop, a seed change, a forced wrap and a y output on the
    way; the state is compared with the C oracle's at the end and at three checkpoints."""
    w = wl.by_name("resnet56_shaped")
    d, W, ld = w.d, w.W, wl.padded_ld(w.d)
    x0 = wl.initial_params(w)
    host_pool = wl.gradient_pool(w, ld=ld, threads=16)
    dev_pool = [torch.from_numpy(g).to(dev) for g in host_pool]
    x = torch.from_numpy(x0).to(dev)
    y = torch.empty(d, dtype=torch.float32, device=dev)
    ora = DefOracleC(x0, W, w.R, w.lr, w.momentum, w.weight_decay, w.seed)
    ctx = _ctx(w, x)
    try:
        for t in range(1000):
            if t == 400:
                ctx.set_lr(0.01)
                ora.set_lr(0.01)
            if t == 600:
                ctx.set_seed(77)
                ora.set_seed(77)
            start = None
            if t % 97 == 5:
                start = d - w.B // 3                      # block crosses the end
                ctx.force_next_start(start)
            ctx.step(dev_pool[t % w.pool], ld, y if t % 250 == 249 else None)
            s = ora.step(host_pool[t % w.pool], start=start)
            assert ctx.last_block() == (s, w.B)
            if t % 250 == 249:
                torch.cuda.synchronize()
                e, m, _ = ctx.state_tensors()
                assert bit_equal(x.cpu().numpy(), ora.x), t
                assert bit_equal(e.cpu().numpy()[:, :d], ora.e), t
                assert bit_equal(m.cpu().numpy()[:, :d], ora.m), t
                assert bit_equal(y.cpu().numpy(), ora.y()), t
        print("[fullsize] resnet56_shaped: 1000 steps bit-identical (x, e, m, y at t = 250, 500, 750, 1000)",
              flush=True)
    finally:
        ctx.destroy()


def _sample_columns(w, starts, n_random):
    d, B = w.d, w.B
    rng = np.random.default_rng([w.seed, 99])
    picks = [rng.integers(0, d, size=n_random), np.arange(0, min(d, 64)), np.arange(max(0, d - 64), d)]
    off = w.tensor_offsets().astype(np.int64)
    for delta in range(-2, 3):
        picks.append(np.clip(off + delta, 0, d - 1))
    for s in starts:
        for edge in (s, s + B):
            picks.append((edge + np.arange(-4, 5)) % d)
    return np.unique(np.concatenate(picks).astype(np.int64))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["resnet50_shaped", "vgg16_shaped"])
def test_sampled_columns_at_full_size(dev, name):
    w = wl.by_name(name)
    d, W, ld = w.d, w.W, wl.padded_ld(w.d)
    print(f"[fullsize] {name}: generating {w.pool} gradient sets of {W}x{d}", flush=True)
    dev_pool = wl.device_gradient_pool(w, ld, device=dev)
    x0 = wl.initial_params(w)
    starts = [w.forced_start(t) if w.forced_start(t) is not None else block_start(w.seed, t, d)
              for t in range(w.T)]
    cols = _sample_columns(w, starts, 1_000_000)
    cols_dev = torch.from_numpy(cols).to(dev)
    host_cols = [g.index_select(1, cols_dev).cpu().numpy() for g in dev_pool]
    ora = DefOracleC(x0[cols], W, w.R, w.lr, w.momentum, w.weight_decay, w.seed, d=d, index=cols)
    x = torch.from_numpy(x0).to(dev)
    y = torch.empty(d, dtype=torch.float32, device=dev)
    ctx = _ctx(w, x)
    try:
        for t in range(w.T):
            last = t == w.T - 1
            start = _gpu_step(ctx, w, t, dev_pool[t % w.pool], ld, y if last else None)
            s = ora.step(host_cols[t % w.pool], start=start)
            assert ctx.last_block() == (s, w.B) and s == starts[t]
        torch.cuda.synchronize()
        assert ctx.last_path_flat()
        e, m, avg = ctx.state_tensors()
        xg = x.index_select(0, cols_dev).cpu().numpy()
        eg = e.index_select(1, cols_dev).cpu().numpy()
        mg = m.index_select(1, cols_dev).cpu().numpy()
        assert_close("x[cols]", xg, ora.x)
        assert_close("e[cols]", eg, ora.e)
        assert_close("m[cols]", mg, ora.m)
        assert np.array_equal(eg == 0, ora.e == 0)
        # the averaged block at the sampled positions that fall inside the last block
        s_last = starts[-1]
        j = (cols - s_last) % d
        inside = j < w.B
        avg_g = avg.index_select(0, torch.from_numpy(j[inside]).to(dev)).cpu().numpy()
        assert_close("averaged block[cols]", avg_g, ora.last_cbar_dense[inside])
        # y is produced on the steps that take def_step; recompute it for the final state
        ctx.output(y)
        torch.cuda.synchronize()
        assert_close("y[cols]", y.index_select(0, cols_dev).cpu().numpy(), ora.y())
        # whole-buffer properties, on the device
        first = min(w.B, d - s_last)
        assert not e[:, s_last:s_last + first].any() and not e[:, :w.B - first].any(), "last block not zero"
        assert not e[:, d:].any() and not m[:, d:].any(), "padding touched"
        assert torch.isfinite(x).all()
        print(f"[fullsize] {name}: {cols.size} columns, bit-identical x={bit_equal(xg, ora.x)} "
              f"e={bit_equal(eg, ora.e)} m={bit_equal(mg, ora.m)}", flush=True)
        assert bit_equal(eg, ora.e) and bit_equal(mg, ora.m)
    finally:
        ctx.destroy()


# --------------------------------------------------------------------------- #
# The instantiations that only large problems select, for every way of calling the
# step.  Shape: the ResNet-18-shaped model (11.7 M parameters in 62 tensors, 16
# workers, 748 MB per state buffer: non-temporal accesses, residency cap, three
# super-tiles of the blocked order), here with weight decay on so that x is read.
# --------------------------------------------------------------------------- #
def _large(wd=1e-4, mu=0.9):
    w = wl.by_name("resnet18_shaped").replace(weight_decay=wd, momentum=mu, T=6, pool=2, variant="def")
    assert w.d > 3 * 16384 * 256 // 2          # more than one super-tile of 16384 tiles of 256
    return w


def _per_tensor_storage(w, x0, host_pool, dev):
    """One device range per tensor, each starting at an odd multiple of 4 bytes past a
    256-byte boundary (pad = l mod 4 floats), for the parameters and for every worker's
    gradients of every set."""
    off = [int(v) for v in w.tensor_offsets()]
    starts, pos = [], 0
    for l in range(w.n_tensors):
        pos = -(-pos // 64) * 64 + (l % 4)
        starts.append(pos)
        pos += off[l + 1] - off[l]
    total = pos
    xbuf = torch.zeros(total, dtype=torch.float32, device=dev)
    x_host = torch.from_numpy(x0)
    params = []
    for l in range(w.n_tensors):
        view = xbuf[starts[l]:starts[l] + off[l + 1] - off[l]]
        view.copy_(x_host[off[l]:off[l + 1]])
        params.append(view)
    tables = []
    for g in host_pool:
        gbuf = torch.zeros((w.W, total), dtype=torch.float32, device=dev)
        g_dev = torch.from_numpy(g).to(dev)
        table = []
        for k in range(w.W):
            for l in range(w.n_tensors):
                view = gbuf[k, starts[l]:starts[l] + off[l + 1] - off[l]]
                view.copy_(g_dev[k, off[l]:off[l + 1]])
                table.append(view)
        del g_dev
        tables.append((gbuf, table))
    return xbuf, params, tables


def _compare_whole_state(ctx, w, x_flat, ora, what):
    d = w.d
    e, m, avg = ctx.state_tensors()
    eg = e.cpu().numpy()
    assert_close(f"{what}: x", x_flat, ora.x)
    assert_close(f"{what}: e", eg[:, :d], ora.e)
    assert np.array_equal(eg[:, :d] == 0, ora.e == 0), f"{what}: zero pattern of e"
    assert not eg[:, d:].any(), f"{what}: padding of e touched"
    same = dict(x=bit_equal(x_flat, ora.x), e=bit_equal(eg[:, :d], ora.e))
    if m is not None:
        mg = m.cpu().numpy()
        assert_close(f"{what}: m", mg[:, :d], ora.m)
        assert not mg[:, d:].any(), f"{what}: padding of m touched"
        same["m"] = bit_equal(mg[:, :d], ora.m)
    avg = avg.cpu().numpy()
    assert_close(f"{what}: averaged block", avg, ora.compact_block())
    same["avg"] = bit_equal(avg, ora.compact_block())
    mask = in_block_mask(d, ora.last_start, w.B)
    assert (bits(eg[:, :d][:, mask]) == 0).all(), f"{what}: last block not zeroed"
    print(f"[fullsize] {what}: bit-identical {same}", flush=True)
    assert same["e"] and same.get("m", True), same
    return same


@pytest.mark.timeout(600)
def test_large_per_tensor_gradients_and_parameters(dev):
    """def_step_tensors with per-tensor parameters at a size that selects the non-temporal
    instantiation with pointer tables (Sec. 1: the model is a list of layer tensors, the
    block runs over their concatenation)."""
    from paper_2004_05298_amd import binding
    binding.load_library()
    w = _large()
    d, W = w.d, w.W
    print(f"[fullsize] per-tensor: d={d} W={W} L={w.n_tensors}", flush=True)
    x0 = wl.initial_params(w)
    host_pool = wl.gradient_pool(w, ld=d, threads=16)
    xbuf, params, tables = _per_tensor_storage(w, x0, host_pool, dev)
    y = torch.empty(d, dtype=torch.float32, device=dev)
    ora = DefOracleC(x0, W, w.R, w.lr, w.momentum, w.weight_decay, w.seed)
    ctx = binding.DefContext(d, W, w.R, w.lr, w.momentum, w.weight_decay, w.seed,
                             param_tensors=params, tensor_offsets=w.tensor_offsets(),
                             stream=torch.cuda.current_stream().cuda_stream)
    try:
        forced = {2: d - w.B // 3}                                     # one block across the end
        for t in range(w.T):
            if t in forced:
                ctx.force_next_start(forced[t])
            ctx.step_tensors(tables[t % w.pool][1], y if t == w.T - 1 else None)
            s = ora.step(host_pool[t % w.pool], start=forced.get(t))
            assert ctx.last_block() == (s, w.B)
        torch.cuda.synchronize()
        name = ctx.last_kernel()
        assert not ctx.last_path_flat()
        assert "tables=1" in name and "nt=1" in name and "lds=8960" in name and "wd=1" in name, name
        x_flat = np.concatenate([p.cpu().numpy() for p in params])
        _compare_whole_state(ctx, w, x_flat, ora, "per-tensor")
        assert_close("per-tensor: y", y.cpu().numpy(), ora.y())
    finally:
        ctx.destroy()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("mu", [0.9, 0.0])
def test_large_detached_points(dev, mu):
    """def_set_detach(lambda = 0.3) in the same pass, with and without momentum, and the
    stand-alone def_detach with another lambda, at a size that selects the non-temporal,
    residency-capped instantiations and several super-tiles (Algorithm 1, "detach" line)."""
    w = _large(mu=mu)
    d, W, ld = w.d, w.W, wl.padded_ld(w.d)
    print(f"[fullsize] detach: d={d} W={W} mu={mu}", flush=True)
    x0 = wl.initial_params(w)
    host_pool = wl.gradient_pool(w, ld=ld, threads=16)
    dev_pool = [torch.from_numpy(g).to(dev) for g in host_pool]
    x = torch.from_numpy(x0).to(dev)
    wbuf = torch.full((W, ld), float("nan"), dtype=torch.float32, device=dev)
    ora = DefOracleC(x0, W, w.R, w.lr, w.momentum, w.weight_decay, w.seed)
    ctx = _ctx(w, x)
    try:
        ctx.set_detach(wbuf, ld, 0.3)
        torch.cuda.synchronize()
        assert bit_equal(wbuf[:, :d].cpu().numpy(), ora.detached_points(LAM32)), "w before the first step"
        forced = {3: d - w.B // 2}
        for t in range(w.T):
            if t in forced:
                ctx.force_next_start(forced[t])
            ctx.step(dev_pool[t % w.pool], ld, None)
            s = ora.step(host_pool[t % w.pool], start=forced.get(t))
            assert ctx.last_block() == (s, w.B)
            if t in (0, 3, w.T - 1):
                torch.cuda.synchronize()
                wg = wbuf[:, :d].cpu().numpy()
                ref = ora.detached_points(LAM32)
                assert_close(f"w t={t}", wg, ref)
                assert bit_equal(wg, ref), f"w t={t} not bit-identical"
        name = ctx.last_kernel()
        want_lds = "lds=11520" if mu != 0 else "lds=7680"
        assert "detach=1" in name and "nt=1" in name and want_lds in name and f"mu={int(mu != 0)}" in name, name
        assert torch.isnan(wbuf[:, d:]).all(), "the step wrote w past column d"
        _compare_whole_state(ctx, w, x.cpu().numpy(), ora, f"detach mu={mu}")
        # stand-alone kernel, another lambda, odd row stride
        w2 = torch.full((W, d + 3), float("nan"), dtype=torch.float32, device=dev)
        ctx.detach(w2, d + 3, 0.75)
        torch.cuda.synchronize()
        assert bit_equal(w2[:, :d].cpu().numpy(), ora.detached_points(0.75)), "def_detach"
        assert torch.isnan(w2[:, d:]).all(), "def_detach wrote past column d"
    finally:
        ctx.destroy()


@pytest.mark.timeout(600)
def test_large_pack_then_apply(dev):
    """The two-halves form (def_pack, then def_apply of the local sum with divisor W) at
    the ResNet-50-shaped size: the same state as def_step, compared with the oracle
    (Algorithm 1, all-reduce and update lines)."""
    w = wl.by_name("resnet50_shaped").replace(T=6)
    d, W, ld = w.d, w.W, wl.padded_ld(w.d)
    print(f"[fullsize] pack+apply: d={d} W={W}", flush=True)
    x0 = wl.initial_params(w)
    host_pool = wl.gradient_pool(w, ld=ld, threads=16)
    dev_pool = [torch.from_numpy(g).to(dev) for g in host_pool]
    x = torch.from_numpy(x0).to(dev)
    y = torch.empty(d, dtype=torch.float32, device=dev)
    ora = DefOracleC(x0, W, w.R, w.lr, w.momentum, w.weight_decay, w.seed)
    ctx = _ctx(w, x)
    try:
        for t in range(w.T):
            block = ctx.pack(dev_pool[t % w.pool], ld)
            assert block == ctx.state_ptrs()[2]
            ctx.apply(block, float(W), y if t == w.T - 1 else None)
            s = ora.step(host_pool[t % w.pool])
            assert ctx.last_block() == (s, w.B)
        torch.cuda.synchronize()
        name = ctx.last_kernel()
        assert "nt=1" in name and "lds=8960" in name, name
        _compare_whole_state(ctx, w, x.cpu().numpy(), ora, "pack+apply")
        assert_close("pack+apply: y", y.cpu().numpy(), ora.y())
    finally:
        ctx.destroy()


@pytest.mark.timeout(600)
def test_large_unaligned_gradient_rows(dev):
    """Gradient rows that are only 4-byte aligned (buffer offset by one float, odd row stride)
    at a size that selects the non-temporal instantiation: g is then read with dword-aligned
    dwordx4 loads while the library's own rows stay on 1 KiB boundaries."""
    w = _large()
    d, W = w.d, w.W
    ld = d + 3
    print(f"[fullsize] unaligned rows: d={d} W={W} ld={ld}", flush=True)
    x0 = wl.initial_params(w)
    host_pool = wl.gradient_pool(w, ld=d, threads=16)
    dev_pool = []
    for g in host_pool:
        buf = torch.zeros(W * ld + 8, dtype=torch.float32, device=dev)
        view = buf[1:1 + W * ld].view(W, ld)
        view[:, :d].copy_(torch.from_numpy(g))
        assert view.data_ptr() % 16 == 4
        dev_pool.append((buf, view))
    x = torch.from_numpy(x0).to(dev)
    y = torch.empty(d, dtype=torch.float32, device=dev)
    ora = DefOracleC(x0, W, w.R, w.lr, w.momentum, w.weight_decay, w.seed)
    ctx = _ctx(w, x)
    try:
        e_ptr, m_ptr, _, ld_state = ctx.state_ptrs()
        # the library's own layout: rows on tile boundaries, e and m apart in their low address bits
        assert ld_state % 256 == 0 and e_ptr % 16384 == 8192 and m_ptr % 16384 == 4096
        for t in range(w.T):
            ctx.step(dev_pool[t % w.pool][1], ld, y if t == w.T - 1 else None)
            s = ora.step(host_pool[t % w.pool])
            assert ctx.last_block() == (s, w.B)
        torch.cuda.synchronize()
        name = ctx.last_kernel()
        assert "nt=1" in name and "tables=0" in name, name
        _compare_whole_state(ctx, w, x.cpu().numpy(), ora, "unaligned rows")
        assert_close("unaligned rows: y", y.cpu().numpy(), ora.y())
    finally:
        ctx.destroy()
