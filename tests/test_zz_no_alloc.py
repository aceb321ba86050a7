"""def_diagnostics_static, the entry point that allocates nothing (its partial sums live
in a fixed array inside the library's device image), against def_diagnostics on the same
error memories and against the CPU oracle: two calls in a row on one GPU, the second on
a smaller problem, then the first again."""
from __future__ import annotations

import numpy as np
import pytest

from oracle.def_oracle import DefOracle
from paper_2004_05298_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

LAM = 0.3
LAM32 = float(np.float32(LAM))


def _run(dev, d, W, R, T):
    """A context and an oracle after T steps on the same seeded gradients."""
    from paper_2004_05298_amd import binding
    binding.load_library()
    w = wl.shrunk(wl.resnet18_shaped(), d=d, n_tensors=5, W=W, R=R, T=T, pool=3)
    ld = wl.padded_ld(d)
    x0 = wl.initial_params(w)
    pool = wl.gradient_pool(w, ld=ld, threads=4)
    x = torch.from_numpy(x0).to(dev)
    gdev = [torch.from_numpy(g).to(dev) for g in pool]
    ora = DefOracle(x0, W, R, w.lr, w.momentum, 0.0, w.seed)
    ctx = binding.DefContext(d, W, R, w.lr, w.momentum, 0.0, w.seed, params=x,
                             stream=torch.cuda.current_stream().cuda_stream)
    for t in range(T):
        ctx.step(gdev[t % w.pool], ld)
        ora.step(pool[t % w.pool][:, :d])
    torch.cuda.synchronize()
    return ctx, ora, x


def _check(binding, dev, ctx, ora, d, W, what):
    stream = torch.cuda.current_stream().cuda_stream
    e_ptr, _, _, ld = ctx.state_ptrs()
    want = torch.full((4,), float("nan"), dtype=torch.float64, device=dev)
    got = torch.full((4,), float("nan"), dtype=torch.float64, device=dev)
    ctx.diagnostics(LAM, want)
    binding.diagnostics_static(e_ptr, ld, d, W, LAM, got, stream)
    torch.cuda.synchronize()
    want, got = want.cpu().numpy(), got.cpu().numpy()
    assert np.array_equal(got.view(np.uint64), want.view(np.uint64)), (what, got, want)
    # and to the oracle, with the tolerances of the other statistics tests (float64 sums in
    # another order; the distance is formed from the two norms)
    ref = ora.diagnostics(LAM32)
    scale = max(ref["mean_sq"], 1e-300)
    assert abs(got[0] - ref["bar_sq"]) <= 1e-10 * scale, (what, got, ref)
    assert abs(got[1] - ref["mean_sq"]) <= 1e-10 * scale, (what, got, ref)
    assert abs(got[2] - ref["lam_star"]) <= 1e-9, (what, got, ref)
    assert abs(got[3] - ref["dist"]) <= 1e-9 * scale, (what, got, ref)
    assert ref["mean_sq"] > 0
    # a caller-held copy with the tightest row stride and rubbish in the padding columns
    ld4 = -(-d // 4) * 4
    e_view = ctx.state_tensors()[0]
    copy = torch.full((W, ld4), float("nan"), dtype=torch.float32, device=dev)
    copy[:, :d] = e_view[:, :d]
    again = torch.full((4,), float("nan"), dtype=torch.float64, device=dev)
    binding.diagnostics_static(copy, ld4, d, W, LAM, again, stream)
    torch.cuda.synchronize()
    assert np.array_equal(again.cpu().numpy().view(np.uint64), want.view(np.uint64)), (what, "copy")
    return got


def test_static_scratch_statistics_match_the_allocating_entry_point():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2004_05298_amd import binding
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    big = _run(dev, d=300011, W=5, R=9, T=6)
    small = _run(dev, d=5003, W=3, R=4, T=5)
    try:
        first = _check(binding, dev, big[0], big[1], 300011, 5, "first call")
        second = _check(binding, dev, small[0], small[1], 5003, 3, "second call, smaller input")
        third = _check(binding, dev, big[0], big[1], 300011, 5, "first input again")
        assert np.array_equal(first, third) and not np.array_equal(first, second)
        # beyond the fixed limit: refused with its own status, nothing run
        out = torch.zeros(4, dtype=torch.float64, device=dev)
        e_ptr, _, _, ld = big[0].state_ptrs()
        with pytest.raises(binding.DefError) as ei:
            binding.diagnostics_static(e_ptr, binding.DEF_STATIC_MAX_D + 4, binding.DEF_STATIC_MAX_D + 1, 1,
                                       LAM, out, torch.cuda.current_stream().cuda_stream)
        assert ei.value.status == binding.DEF_ELIMIT
    finally:
        big[0].destroy()
        small[0].destroy()
