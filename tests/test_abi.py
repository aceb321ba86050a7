"""CPU-only checks of the C ABI: the built library exports every symbol that
include/def.h declares, the binding covers them all, argument validation rejects
bad problem statements before touching the GPU, and the shared block draw equals
the oracle's for every (seed, step, d) tried.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

from oracle.philox import block_start as oracle_block_start
from paper_2004_05298_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", name) for name in sorted(os.listdir(os.path.join(ROOT, "include")))
           if name.endswith(".h")]


def declared_functions():
    names = set()
    for header in HEADERS:
        text = open(header).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(def_[a-z_]+)\s*\(", text))
    return sorted(names)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding._build.library_path()):
        binding._build.build_library()
    return binding.load_library()


def test_header_declares_the_required_entry_points():
    names = declared_functions()
    for required in ("def_init", "def_step", "def_a_step", "def_set_seed"):
        assert required in names


def test_library_exports_every_declared_symbol(lib):
    raw = ctypes.CDLL(binding._build.library_path())
    for name in declared_functions():
        assert hasattr(raw, name), f"{name} declared in def.h but not exported"


def test_binding_covers_every_declared_symbol():
    assert sorted(binding.SIGNATURES) == declared_functions()


def test_config_struct_layout_matches_header():
    # uint64, 2x uint32, 3x float (+4 pad), uint64, ptr, uint32 (+4 pad), ptr, ptr, ptr
    assert ctypes.sizeof(binding.DefConfig) == 8 + 8 + 12 + 4 + 8 + 8 + 8 + 8 + 8 + 8
    assert binding.DefConfig.seed.offset == 32
    assert binding.DefConfig.params.offset == 56
    assert binding.DefConfig.stream.offset == 72


def test_block_start_equals_oracle_draw(lib):
    for seed in (0, 1, 200405298, 200405301, 2**63 + 5, 2**64 - 1):
        for d in (1, 2, 37, 65536, 853018, 25557032, 138357544, 2**39 + 7):
            for t in list(range(20)) + [10**6, 2**40 + 3, 2**64 - 1]:
                assert binding.block_start(seed, t, d) == oracle_block_start(seed, t, d)


def test_block_start_rejects_bad_arguments(lib):
    out = ctypes.c_uint64()
    assert lib.def_block_start(1, 1, 0, ctypes.byref(out)) == binding.DEF_EINVAL
    assert lib.def_block_start(1, 1, 5, None) == binding.DEF_EINVAL


def _cfg(**kw):
    c = binding.DefConfig()
    c.d, c.W, c.R, c.lr, c.momentum, c.weight_decay, c.seed = 100, 2, 4, 0.1, 0.9, 0.0, 1
    c.tensor_offsets, c.n_tensors, c.params, c.param_ptrs, c.stream = None, 1, 4096, None, None
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def _offsets(vals):
    arr = (ctypes.c_uint64 * len(vals))(*vals)
    return ctypes.cast(arr, ctypes.POINTER(ctypes.c_uint64)), arr


@pytest.mark.parametrize("bad", [
    dict(d=0), dict(W=0), dict(R=0), dict(R=101), dict(d=2**40), dict(params=None),
    dict(params=4098), dict(lr=float("nan")), dict(momentum=float("nan")),
])
def test_init_rejects_bad_problem_statements(lib, bad):
    h = ctypes.c_void_p()
    assert lib.def_init(ctypes.byref(h), ctypes.byref(_cfg(**bad))) == binding.DEF_EINVAL
    assert not h.value


@pytest.mark.parametrize("vals", [[0, 50, 50, 100], [0, 60, 40, 100], [1, 50, 100], [0, 50, 99],
                                   [0, 50, 101]])
def test_init_rejects_bad_offset_tables(lib, vals):
    ptr, keep = _offsets(vals)
    h = ctypes.c_void_p()
    cfg = _cfg(tensor_offsets=ptr, n_tensors=len(vals) - 1)
    assert lib.def_init(ctypes.byref(h), ctypes.byref(cfg)) == binding.DEF_EINVAL
    del keep


def test_null_handles_are_rejected(lib):
    assert lib.def_init(None, ctypes.byref(_cfg())) == binding.DEF_EINVAL
    assert lib.def_init(ctypes.byref(ctypes.c_void_p()), None) == binding.DEF_EINVAL
    assert lib.def_step(None, 4096, 100, None) == binding.DEF_EINVAL
    assert lib.def_a_step(None, 4096, 100) == binding.DEF_EINVAL
    assert lib.def_set_seed(None, 1) == binding.DEF_EINVAL
    assert lib.def_destroy(None) == binding.DEF_EINVAL
    assert lib.def_output(None, 4096) == binding.DEF_EINVAL
    assert lib.def_strerror(binding.DEF_EINVAL) == b"invalid argument"


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library(str(tmp_path / "libdef_hip.so"))


def test_init_rejects_problems_whose_grid_would_not_fit(lib):
    """W * ceil(d/256) must stay below 2^31; refused before anything is allocated."""
    h = ctypes.c_void_p()
    assert lib.def_init(ctypes.byref(h), ctypes.byref(_cfg(d=2**39, W=64))) == binding.DEF_EINVAL
    assert not h.value


def test_binding_checks_table_lengths_before_calling_the_library(lib):
    """The C side reads n_tensors+1 offsets, n_tensors parameter pointers and
    W*n_tensors gradient pointers from host arrays whose length it cannot see;
    the binding refuses lists of any other length."""
    with pytest.raises(ValueError, match="param_tensors has 2 entries for 3 tensors"):
        binding.DefContext(30, 2, 2, 0.1, param_tensors=[4096, 8192], tensor_offsets=[0, 10, 20, 30])
    with pytest.raises(ValueError, match="at least two entries"):
        binding.DefContext(30, 2, 2, 0.1, params=4096, tensor_offsets=[0])
    with pytest.raises(ValueError, match="params .* or param_tensors"):
        binding.DefContext(30, 2, 2, 0.1)
    ctx = binding.DefContext.__new__(binding.DefContext)      # no library context behind it
    ctx.W, ctx.n_tensors, ctx._h = 2, 3, ctypes.c_void_p()
    with pytest.raises(ValueError, match="5 gradient tensors given, W\\*n_tensors = 6"):
        ctx._gtable([4096] * 5)
    assert len(ctx._gtable([4096] * 6)) == 6


def test_static_entry_point_checks_sizes_before_touching_the_gpu(lib):
    """def_diagnostics_static validates its arguments, and refuses problems beyond the
    size its fixed scratch array covers, before any HIP call."""
    big = binding.DEF_STATIC_MAX_D
    call = lib.def_diagnostics_static
    assert call(4096, big + 4, big + 1, 1, 0.3, 8192, None) == binding.DEF_ELIMIT
    assert lib.def_strerror(binding.DEF_ELIMIT) == b"problem larger than the fixed limit of this entry point"
    for args in [(None, 128, 100, 2, 0.3, 8192, None),        # no error memories
                 (4096, 128, 100, 2, 0.3, None, None),         # no output
                 (4096, 128, 0, 2, 0.3, 8192, None),           # d = 0
                 (4096, 128, 100, 0, 0.3, 8192, None),         # W = 0
                 (4096, 96, 100, 2, 0.3, 8192, None),          # ld < d
                 (4096, 102, 100, 2, 0.3, 8192, None),         # ld not a multiple of 4
                 (4100, 128, 100, 2, 0.3, 8192, None),         # rows not 16-byte aligned
                 (4096, 128, 100, 2, 0.3, 8196, None),         # output not 8-byte aligned
                 (4096, 128, 100, 2, 1.5, 8192, None)]:        # lambda outside [0, 1]
        assert call(*args) == binding.DEF_EINVAL, args


def test_probe_rejects_bad_arguments_before_launching(lib):
    call = lib.def_probe_stream
    assert call(7, 4096, 8192, 1024, 1.0, 64, 1, 10240, None) == binding.DEF_EINVAL      # unknown kind
    assert call(2, 4096, 8192, 1000, 1.0, 64, 1, 10240, None) == binding.DEF_EINVAL      # n not a multiple of 256
    assert call(2, 4096, 8192, 0, 1.0, 64, 1, 10240, None) == binding.DEF_EINVAL
    assert call(2, None, 8192, 1024, 1.0, 64, 1, 10240, None) == binding.DEF_EINVAL      # copy without a source
    assert call(1, None, None, 1024, 1.0, 64, 1, 10240, None) == binding.DEF_EINVAL      # write without a destination
    assert call(2, 4100, 8192, 1024, 1.0, 64, 1, 10240, None) == binding.DEF_EINVAL      # misaligned
    assert call(2, 4096, 8192, 1024, 1.0, 64, 1, 70000, None) == binding.DEF_EINVAL      # LDS reservation too large
    assert call(2, 4096, 8192, 1024, 1.0, 128, 1, 0, None) == binding.DEF_EINVAL         # shape not offered
    assert call(2, 4096, 8192, 1024, 1.0, 64, 3, 0, None) == binding.DEF_EINVAL
