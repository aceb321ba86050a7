"""The plain streaming probes (include/def_probe.h) do what their names say, in every
launch shape offered: the benchmark prices the DEF step against them, so a probe that
skipped part of its buffer would flatter or slander the step."""
from __future__ import annotations

import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SHAPES = [(64, 1, 0), (64, 1, 10240), (64, 2, 0), (64, 4, 0), (256, 1, 0), (256, 2, 0), (256, 4, 0)]


@pytest.mark.parametrize("threads,quads,lds", SHAPES)
def test_probes_touch_exactly_their_buffers(threads, quads, lds):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2004_05298_amd import binding
    binding.load_library()
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream
    n = 256 * 4099                                    # not a multiple of any workgroup's 4096 floats
    guard = 64
    src = torch.arange(n, dtype=torch.float32, device="cuda") * 0.5 - 1000.0
    buf = torch.full((n + 2 * guard,), -7.0, dtype=torch.float32, device="cuda")
    dst = buf[guard:guard + n]
    assert dst.data_ptr() % 16 == 0
    args = dict(threads=threads, quads=quads, lds_reserve=lds, stream=stream)

    binding.probe_stream(binding.PROBE_READ, src, None, n, **args)            # reads only
    binding.probe_stream(binding.PROBE_WRITE, None, dst, n, 3.25, **args)
    torch.cuda.synchronize()
    assert bool((dst == 3.25).all())
    binding.probe_stream(binding.PROBE_COPY, src, dst, n, **args)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    binding.probe_stream(binding.PROBE_UPDATE, None, dst, n, 2.0, **args)
    torch.cuda.synchronize()
    assert torch.equal(dst, src * 2.0)
    assert bool((buf[:guard] == -7.0).all()) and bool((buf[guard + n:] == -7.0).all())
    assert torch.equal(src, torch.arange(n, dtype=torch.float32, device="cuda") * 0.5 - 1000.0)
