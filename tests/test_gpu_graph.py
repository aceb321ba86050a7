"""Device-side block draw and HIP-graph replay of captured steps, against the CPU
oracle.  Each replay is followed by a synchronisation and checked on its own, with
eager work (the copy of the next gradients) between replays."""
from __future__ import annotations

import numpy as np
import pytest

from oracle.def_oracle import DefOracle
from paper_2004_05298_amd import workloads as wl
from tests.parity import bit_equal

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    torch.cuda.set_device(0)
    return torch.device("cuda:0")


def _setup(dev, stream, d=30011, W=5, R=9, T=12, wd=1e-4, L=7):
    from paper_2004_05298_amd import binding
    binding.load_library()
    w = wl.shrunk(wl.resnet50_shaped(), d=d, n_tensors=L, W=W, R=R, T=T, pool=4)
    ld = wl.padded_ld(w.d)
    x0 = wl.initial_params(w)
    pool = wl.gradient_pool(w, ld=ld, threads=1)
    with torch.cuda.stream(stream):
        x = torch.from_numpy(x0).to(dev)
        gdev = [torch.from_numpy(g).to(dev) for g in pool]
    stream.synchronize()
    ora = DefOracle(x0, w.W, w.R, w.lr, w.momentum, wd, w.seed)
    ctx = binding.DefContext(w.d, w.W, w.R, w.lr, w.momentum, wd, w.seed, params=x,
                             tensor_offsets=w.tensor_offsets(), stream=stream.cuda_stream)
    return w, ld, pool, gdev, x, ora, ctx


def _check_state(ctx, x, ora, d, where):
    e, m, _ = ctx.state_tensors()
    assert bit_equal(x.cpu().numpy(), ora.x), f"{where}: x"
    assert bit_equal(e.cpu().numpy()[:, :d], ora.e), f"{where}: e"
    assert bit_equal(m.cpu().numpy()[:, :d], ora.m), f"{where}: m"


def test_device_draw_matches_host_draw_and_oracle(dev):
    stream = torch.cuda.Stream()
    w, ld, pool, gdev, x, ora, ctx = _setup(dev, stream)
    try:
        ctx.set_device_draw(True)
        for t in range(w.T):
            if t == 3:
                ctx.force_next_start(w.d - 2)
            if t == 5:
                ctx.set_seed(4242); ora.set_seed(4242)
            if t == 8:
                ctx.set_step(100); ora.set_step(100)
            if t == 10:
                ctx.set_device_draw(False)          # host draw again; the host's counter is current
            ctx.step(gdev[t % w.pool], ld)
            s = ora.step(pool[t % w.pool][:, :w.d], start=(w.d - 2 if t == 3 else None))
            ctx.sync_step()
            assert ctx.last_block() == (s, w.B), t
            assert ctx.get_step() == ora.t
        stream.synchronize()
        _check_state(ctx, x, ora, w.d, "device draw")
    finally:
        ctx.destroy()


@pytest.mark.parametrize("steps_per_graph,split", [(1, False), (3, False), (2, True)])
def test_graph_replays_follow_the_oracle(dev, steps_per_graph, split):
    """split: every captured iteration is def_pack + def_apply of the local sum (the two
    halves a multi-GPU caller would put a collective between)."""
    stream = torch.cuda.Stream()
    w, ld, pool, gdev, x, ora, ctx = _setup(dev, stream)
    n = steps_per_graph
    try:
        with torch.cuda.stream(stream):
            static = [torch.zeros_like(gdev[0]) for _ in range(n)]
            y = torch.zeros(w.d, dtype=torch.float32, device=dev)
        ctx.set_device_draw(True)
        # two eager steps first (they also warm the kernels up), then capture
        for t in range(2):
            ctx.step(gdev[t % w.pool], ld)
            ora.step(pool[t % w.pool][:, :w.d])
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for q in range(n):
                if split:
                    ctx.apply(ctx.pack(static[q], ld), float(w.W), y if q == n - 1 else None)
                else:
                    ctx.step(static[q], ld, y if q == n - 1 else None)
        stream.synchronize()
        _check_state(ctx, x, ora, w.d, "capture must not execute anything")
        t = 2
        for replay in range(5):
            with torch.cuda.stream(stream):
                for q in range(n):                   # eager work between replays
                    static[q].copy_(gdev[(t + q) % w.pool])
                graph.replay()
            stream.synchronize()
            for q in range(n):
                s = ora.step(pool[(t + q) % w.pool][:, :w.d])
            t += n
            _check_state(ctx, x, ora, w.d, f"replay {replay}")
            assert bit_equal(y.cpu().numpy(), ora.y()), f"replay {replay}: y"
            ctx.sync_step()
            assert ctx.get_step() == t and ctx.last_block() == (s, w.B)
        # eager steps after the replays continue the same sequence
        for _ in range(2):
            ctx.step(gdev[t % w.pool], ld)
            ora.step(pool[t % w.pool][:, :w.d])
            t += 1
        stream.synchronize()
        _check_state(ctx, x, ora, w.d, "eager after replays")
    finally:
        ctx.destroy()


def test_captured_pointer_table_survives_other_tables(dev):
    """A captured def_step_tensors reads its gradient pointer table from device memory on
    every replay.  The table must already be on the device when the capture starts (a new
    one would need a copy, which cannot be captured: DEF_EINVAL), and it must not be
    replaced when more tables than the library caches pass through afterwards."""
    from paper_2004_05298_amd import binding
    stream = torch.cuda.Stream()
    w, ld, pool, gdev, x, ora, ctx = _setup(dev, stream, T=20)
    off = [int(v) for v in w.tensor_offsets()]

    def table(buf):
        return [buf[k, off[l]:off[l + 1]] for k in range(w.W) for l in range(w.n_tensors)]

    try:
        with torch.cuda.stream(stream):
            static = torch.zeros_like(gdev[0])
            others = [g.clone() for g in gdev] + [gdev[0].clone(), gdev[1].clone()]    # six more tables
        ctx.set_device_draw(True)
        t = 0
        with torch.cuda.stream(stream):
            static.copy_(gdev[0])
        ctx.step_tensors(table(static))                      # eager: the table goes to the device
        ora.step(pool[0][:, :w.d]); t += 1
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        refused = None
        with torch.cuda.graph(graph, stream=stream):
            try:
                ctx.step_tensors(table(others[0]))           # never seen: cannot be uploaded now
            except binding.DefError as err:
                refused = err.status
            ctx.step_tensors(table(static))
        assert refused == binding.DEF_EINVAL
        stream.synchronize()
        _check_state(ctx, x, ora, w.d, "capture must not execute anything")
        for replay in range(3):
            # six other tables eagerly in between: more than the library keeps
            for q, buf in enumerate(others):
                src = (t + q) % w.pool
                with torch.cuda.stream(stream):
                    buf.copy_(gdev[src])
                ctx.step_tensors(table(buf))
                ora.step(pool[src][:, :w.d])
            t += len(others)
            with torch.cuda.stream(stream):
                static.copy_(gdev[t % w.pool])
                graph.replay()
            stream.synchronize()
            ora.step(pool[t % w.pool][:, :w.d]); t += 1
            _check_state(ctx, x, ora, w.d, f"replay {replay}")
            ctx.sync_step()
            assert ctx.get_step() == t
    finally:
        ctx.destroy()


def test_captured_iteration_with_detached_points_and_statistics(dev):
    """Everything a training iteration may enqueue besides the step is captured with it: the
    step writes the detached points, then come def_output, the stand-alone def_detach with
    another lambda, both sets of error-memory statistics and the statistics entry point that
    allocates nothing.  A call that allocated, copied or synchronised would break the capture;
    each replay's outputs are compared with the oracle."""
    from paper_2004_05298_amd import binding
    stream = torch.cuda.Stream()
    w, ld, pool, gdev, x, ora, ctx = _setup(dev, stream, d=41003, W=19, R=7, T=12, wd=1e-4, L=5)
    W, d = w.W, w.d
    lam = float(np.float32(0.3))
    lam2 = float(np.float32(0.75))
    try:
        with torch.cuda.stream(stream):
            static = torch.zeros_like(gdev[0])
            y = torch.zeros(d, dtype=torch.float32, device=dev)
            pts = torch.zeros((W, ld), dtype=torch.float32, device=dev)
            pts2 = torch.zeros((W, ld), dtype=torch.float32, device=dev)
            diag = torch.zeros(4, dtype=torch.float64, device=dev)
            diag_static = torch.zeros(4, dtype=torch.float64, device=dev)
            per_worker = torch.zeros(3 * W, dtype=torch.float64, device=dev)
        ctx.set_device_draw(True)
        ctx.set_detach(pts, ld, lam)
        ctx.step(gdev[0], ld)                       # one eager step (also warms the kernels up)
        ora.step(pool[0][:, :d])
        e, _, _ = ctx.state_tensors()
        ld_state = e.stride(0)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            ctx.step(static, ld)
            ctx.output(y)
            ctx.detach(pts2, ld, lam2)
            ctx.diagnostics(lam, diag)
            ctx.diagnostics_workers(per_worker)
            binding.diagnostics_static(e.data_ptr(), ld_state, d, W, lam, diag_static, stream.cuda_stream)
        stream.synchronize()
        _check_state(ctx, x, ora, d, "capture must not execute anything")
        t = 1
        for replay in range(4):
            with torch.cuda.stream(stream):
                static.copy_(gdev[t % w.pool])       # eager work between replays
                graph.replay()
            stream.synchronize()
            ora.step(pool[t % w.pool][:, :d])
            t += 1
            where = f"replay {replay}"
            _check_state(ctx, x, ora, d, where)
            assert bit_equal(y.cpu().numpy(), ora.y()), f"{where}: y"
            assert bit_equal(pts.cpu().numpy()[:, :d], ora.detached_points(lam)), f"{where}: w of the step"
            assert bit_equal(pts2.cpu().numpy()[:, :d], ora.detached_points(lam2)), f"{where}: def_detach"
            got, ref = diag.cpu().numpy(), ora.diagnostics(lam)
            scale = ref["mean_sq"]
            assert abs(got[0] - ref["bar_sq"]) <= 1e-10 * scale and abs(got[1] - ref["mean_sq"]) <= 1e-10 * scale
            assert abs(got[2] - ref["lam_star"]) <= 1e-9 and abs(got[3] - ref["dist"]) <= 1e-9 * scale
            assert np.array_equal(diag_static.cpu().numpy(), got), f"{where}: static statistics differ"
            pw, refw = per_worker.cpu().numpy(), ora.diagnostics_workers()
            assert np.abs(pw[:W] - refw["norm_sq"]).max() <= 1e-10 * scale * W
            assert np.abs(pw[W:2 * W] - refw["inner"]).max() <= 1e-10 * scale * W
            assert np.abs(pw[2 * W:] - refw["lam_star"]).max() <= 1e-9
    finally:
        ctx.destroy()
