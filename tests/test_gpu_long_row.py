"""GPU parity for a parameter vector longer than 2^32: column indices, block
positions and row strides that need more than 32 bits.

d = 2^32 + 1029 (not a multiple of 4), one worker, momentum and weight decay on,
so the pass reads x in the blocked order over 1025 super-tiles.  The oracle's whole
state would be 4 x 17 GB on the host, so, as for the VGG-16-shaped workload, it
simulates a sample of columns exactly: random ones, the two ends of the vector, the
neighbourhoods of 2^31 and 2^32, and the edges of every step's block.  The blocks
are forced across the end of the vector, across index 2^32 and across index 2^31.
Inputs are drawn on the device by torch's seeded generator (the host generators
would take minutes at this length); the oracle is given the sampled columns of the
same tensors.  Whole-buffer properties are checked on the device.
"""
from __future__ import annotations

import numpy as np
import pytest

from oracle.c_oracle import DefOracleC
from oracle.philox import block_start
from paper_2004_05298_amd import workloads as wl
from tests.parity import assert_close, bit_equal

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

D = (1 << 32) + 1029
NEED_BYTES = 135 << 30        # x, y, w, two gradient sets, e, m: seven rows of 17.2 GB, plus slack


def _normal_rows(shape, std, gen, dev):
    """A float32 tensor of the given shape filled with N(0, std^2), drawn in pieces of 2^28."""
    out = torch.empty(shape, dtype=torch.float32, device=dev)
    flat = out.view(-1)
    piece = 1 << 28
    for lo in range(0, flat.numel(), piece):
        flat[lo:lo + piece].normal_(0.0, std, generator=gen)
    return out


@pytest.mark.timeout(900)
def test_row_longer_than_2_32_columns():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    torch.cuda.empty_cache()              # what earlier tests left in torch's cache counts as used
    free, _ = torch.cuda.mem_get_info()
    if free < NEED_BYTES:
        pytest.skip(f"needs {NEED_BYTES >> 30} GiB of free device memory, {free >> 30} GiB free")
    from paper_2004_05298_amd import binding
    binding.load_library()

    d, W, R, lr, mu, wd, seed = D, 1, 1024, 0.1, 0.9, 1e-4, 200405298 + 32
    B = -(-d // R)
    ld = wl.padded_ld(d)
    print(f"[long row] d={d} B={B} ld={ld}: drawing inputs on the device", flush=True)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    x = _normal_rows((d,), 0.05, gen, dev)
    pool = [_normal_rows((W, ld), 1e-3, gen, dev) for _ in range(2)]

    forced = {1: d - B // 2,              # across the end of the vector
              2: (1 << 32) - B // 2,      # across index 2^32
              3: (1 << 31) - 5}           # across index 2^31
    T = 5
    starts = [forced.get(t, block_start(seed, t, d)) for t in range(T)]
    rng = np.random.default_rng([seed, 7])
    picks = [rng.integers(0, d, size=300_000), np.arange(0, 64), np.arange(d - 64, d),
             (1 << 31) + np.arange(-40, 40), (1 << 32) + np.arange(-40, 40)]
    for s in starts:
        for edge in (s, s + B):
            picks.append((edge + np.arange(-6, 7)) % d)
        picks.append((s + rng.integers(0, B, size=20_000)) % d)       # inside every block
    cols = np.unique(np.concatenate(picks).astype(np.int64))
    cols_dev = torch.from_numpy(cols).to(dev)
    x0_cols = x.index_select(0, cols_dev).cpu().numpy()
    host_cols = [g.index_select(1, cols_dev).cpu().numpy() for g in pool]
    ora = DefOracleC(x0_cols, W, R, lr, mu, wd, seed, d=d, index=cols)

    y = torch.empty(d, dtype=torch.float32, device=dev)
    ctx = binding.DefContext(d, W, R, lr, mu, wd, seed, params=x,
                             stream=torch.cuda.current_stream().cuda_stream)
    try:
        assert ctx.block_length() == B
        for t in range(T):
            if t in forced:
                ctx.force_next_start(forced[t])
            print(f"[long row] step {t}: start {starts[t]}", flush=True)
            ctx.step(pool[t % 2], ld, y if t == T - 1 else None)
            s = ora.step(host_cols[t % 2], start=forced.get(t))
            assert ctx.last_block() == (s, B) and s == starts[t]
        torch.cuda.synchronize()
        assert ctx.last_path_flat()
        assert "wd=1" in ctx.last_kernel() and "nt=1" in ctx.last_kernel(), ctx.last_kernel()
        e, m, avg = ctx.state_tensors()
        xg = x.index_select(0, cols_dev).cpu().numpy()
        eg = e.index_select(1, cols_dev).cpu().numpy()
        mg = m.index_select(1, cols_dev).cpu().numpy()
        assert_close("x[cols]", xg, ora.x)
        assert_close("e[cols]", eg, ora.e)
        assert_close("m[cols]", mg, ora.m)
        assert np.array_equal(eg == 0, ora.e == 0)
        assert_close("y[cols]", y.index_select(0, cols_dev).cpu().numpy(), ora.y())
        s_last = starts[-1]
        j = (cols - s_last) % d
        inside = j < B
        assert inside.sum() > 10_000
        avg_g = avg.index_select(0, torch.from_numpy(j[inside]).to(dev)).cpu().numpy()
        assert_close("averaged block[cols]", avg_g, ora.last_cbar_dense[inside])
        # whole-buffer properties, on the device
        first = min(B, d - s_last)
        assert not e[:, s_last:s_last + first].any() and not e[:, :B - first].any(), "last block not zero"
        assert not e[:, d:].any() and not m[:, d:].any(), "padding touched"
        # the stand-alone detached points at this length
        lam = float(np.float32(0.75))
        w = torch.empty((W, ld), dtype=torch.float32, device=dev)
        ctx.detach(w, ld, lam)
        torch.cuda.synchronize()
        wg = w.index_select(1, cols_dev).cpu().numpy()
        assert_close("w[cols]", wg, ora.detached_points(lam))
        # one worker: e_t is e_0, so both norms are the same sum and lambda*(t) is exactly 1
        diag = torch.zeros(4, dtype=torch.float64, device=dev)
        ctx.diagnostics(lam, diag)
        per_worker = torch.zeros(3 * W, dtype=torch.float64, device=dev)
        ctx.diagnostics_workers(per_worker)
        torch.cuda.synchronize()
        got, pw = diag.cpu().numpy(), per_worker.cpu().numpy()
        assert got[0] == got[1] and got[2] == 1.0, got
        assert pw[2] == 1.0 and abs(pw[0] - got[0]) <= 1e-10 * got[0], (pw, got)
        print(f"[long row] {cols.size} columns, bit-identical x={bit_equal(xg, ora.x)} e={bit_equal(eg, ora.e)} "
              f"m={bit_equal(mg, ora.m)} w={bit_equal(wg, ora.detached_points(lam))}", flush=True)
        assert bit_equal(eg, ora.e) and bit_equal(mg, ora.m)
    finally:
        ctx.destroy()
        del x, y, pool
        torch.cuda.empty_cache()
