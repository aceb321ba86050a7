"""Mutation check of the oracle pins (CPU only).

Each case plants one plausible mistake in a private copy of the numpy oracle's
source (a dropped term, a wrong sign, a missing wrap, ...) and asserts that at
least one pin of tests/test_oracle_pins.py fails on it.  The unmodified copy must
pass the same pins.  Nothing here touches the GPU.
"""
import os
import types

import numpy as np
import pytest

import oracle.def_oracle as real_module
import oracle.philox as real_philox
from tests import test_oracle_pins as pins

_SRC = open(real_module.__file__.replace(".pyc", ".py")).read()
_PHILOX_SRC = open(real_philox.__file__.replace(".pyc", ".py")).read()

# The pins a mutant is run through (numpy kinds only: the copy is a numpy oracle).
def _pin_calls():
    calls = []
    for kind in ("np32", "np64"):
        calls.append(lambda k=kind: pins.test_start_is_pure_function_of_seed_and_step(k))
        calls.append(lambda k=kind: pins.test_compressor_expectation_and_contraction(k, 13, 3))
        calls.append(lambda k=kind: pins.test_age_counter_closed_form(k, 29, 4, 3))
        calls.append(lambda k=kind: pins.test_age_counter_closed_form(k, 20, 3, 4))
        calls.append(lambda k=kind: pins.test_brute_force_every_start_and_ratio(k))
    calls.append(lambda: pins.test_split_is_exact_and_block_is_literal_zero("np32"))
    calls.append(lambda: pins.test_allreduce_compatibility_whole_iteration("np64"))
    for mu, wd in [(0.9, 0.0), (0.9, 5e-4), (0.0, 1e-2)]:
        calls.append(lambda mu=mu, wd=wd: pins.test_ratio_one_is_momentum_sgd("np64", 1e-12, mu, wd))
    calls.append(lambda: pins.test_y_follows_uncompressed_momentum_path("np64", 1e-12, 61, 3, 7))
    calls.append(lambda: pins.test_single_worker_lemma_x_chases_sgd_path())
    calls.append(lambda: pins.test_block_length_is_the_ceiling())
    for kind in ("np32", "np64"):
        calls.append(lambda k=kind: pins.test_detached_points_special_cases(k))
    calls.append(lambda: pins.test_detached_points_distance_identity())
    calls.append(lambda: pins.test_closed_loop_single_worker_follows_gradient_descent("np64", 1e-12))
    calls.append(lambda: _diag_pin(np.float64))
    calls.append(lambda: _diag_pin(np.float64, pins.test_per_worker_statistics))
    return calls


def _diag_pin(dtype, pin=None):
    saved = pins.DefOracle
    pins.DefOracle = pins.NUMPY_ORACLE
    try:
        (pin or pins.test_diagnostics_against_norms_of_detached_points)(dtype)
    finally:
        pins.DefOracle = saved


def _load(src, philox_src=None):
    ph = real_philox
    if philox_src is not None:
        ph = types.ModuleType("mutant_philox")
        exec(compile(philox_src, "mutant_philox", "exec"), ph.__dict__)
    mod = types.ModuleType("mutant_oracle")
    mod.__dict__["__name__"] = "mutant_oracle"
    code = src.replace("from .philox import block_start", "")
    mod.__dict__["block_start"] = ph.block_start
    exec(compile(code, "mutant_oracle", "exec"), mod.__dict__)
    return mod, ph


def _run_pins(mod, ph):
    """Returns the number of pins that fail with the given oracle module."""
    saved = (pins.NUMPY_ORACLE, pins.block_length, pins.in_block, pins.block_start)
    pins.NUMPY_ORACLE = mod.DefOracle
    pins.block_length, pins.in_block, pins.block_start = mod.block_length, mod.in_block, ph.block_start
    failed = 0
    try:
        for call in _pin_calls():
            try:
                call()
            except (AssertionError, IndexError, ValueError, ZeroDivisionError):
                failed += 1
        try:
            pins.test_block_start_is_library_draw_mod_d()
        except AssertionError:
            failed += 1
    finally:
        pins.NUMPY_ORACLE, pins.block_length, pins.in_block, pins.block_start = saved
    return failed


MUTANTS = [
    ("momentum term dropped", "mk = self.mu * self.m[k] + gk", "mk = gk + 0 * self.m[k]"),
    ("momentum sign", "mk = self.mu * self.m[k] + gk", "mk = self.mu * self.m[k] - gk"),
    ("lr on the wrong operand", "p = self.lr * mk + self.e[k]", "p = mk + self.lr * self.e[k]"),
    ("error feedback dropped", "p = self.lr * mk + self.e[k]", "p = self.lr * mk"),
    ("update sign", "self.x = self.x - cbar", "self.x = self.x + cbar"),
    ("sum instead of mean", "cbar = acc / ft(self.W)", "cbar = acc"),
    ("block not zeroed", "self.e[k] = np.where(mask, zero, p)", "self.e[k] = p"),
    ("residual dropped", "self.e[k] = np.where(mask, zero, p)", "self.e[k] = np.where(mask, zero, zero)"),
    ("mask inverted", "cp = np.where(mask, p, zero)", "cp = np.where(mask, zero, p)"),
    ("no circular wrap", "return ((index - np.int64(s)) % np.int64(d)) < np.int64(B)",
     "return ((index - np.int64(s)) >= 0) & ((index - np.int64(s)) < np.int64(B))"),
    ("block one too long", ") < np.int64(B)", ") <= np.int64(B)"),
    ("block starts one late", "((index - np.int64(s)) %", "((index - np.int64(s) - 1) %"),
    ("floor instead of ceil", "return -(-d // R)", "return max(1, d // R)"),
    ("decay at the wrong sign", "gk = gk + self.wd * self.x", "gk = gk - self.wd * self.x"),
    ("decay dropped", "gk = gk + self.wd * self.x", "gk = gk + 0 * self.x"),
    ("y sign", "return self.x - acc / self.dtype.type(self.W)", "return self.x + acc / self.dtype.type(self.W)"),
    ("y not averaged", "return self.x - acc / self.dtype.type(self.W)", "return self.x - acc"),
    ("step counter stuck", "self.t += 1", "self.t += 0"),
    ("detach sign", "out[k] = self.x - lam * self.e[k]", "out[k] = self.x + lam * self.e[k]"),
    ("detach ignores lambda", "out[k] = self.x - lam * self.e[k]", "out[k] = self.x - self.e[k]"),
    ("detach uses momentum", "out[k] = self.x - lam * self.e[k]", "out[k] = self.x - lam * self.m[k]"),
    ("detach uses worker 0", "out[k] = self.x - lam * self.e[k]", "out[k] = self.x - lam * self.e[0]"),
    ("compact block starts one late",
     "j = (np.int64(self.last_start) + np.arange(self.B, dtype=np.int64)) % np.int64(self.d)",
     "j = (np.int64(self.last_start) + 1 + np.arange(self.B, dtype=np.int64)) % np.int64(self.d)"),
    ("diagnostics: mean error not divided", "e_bar = acc / np.float64(self.W)", "e_bar = acc"),
    ("diagnostics: mean_sq is a sum", "for k in range(self.W)) / self.W)\n        dist", "for k in range(self.W)))\n        dist"),
    ("diagnostics: lambda* inverted", "lam_star=(bar_sq / mean_sq if", "lam_star=(mean_sq / bar_sq if"),
    ("diagnostics: distance sign", "(e_bar - np.float64(lam) * e[k]) ** 2", "(e_bar + np.float64(lam) * e[k]) ** 2"),
    ("per worker: inner product with worker 0", "np.sum(mean_e * e[k]) for k", "np.sum(mean_e * e[0]) for k"),
    ("per worker: norm of worker 0", "np.sum(e[k] * e[k]) for k in range(self.W)], dtype", "np.sum(e[0] * e[0]) for k in range(self.W)], dtype"),
    ("per worker: mean error not divided", "mean_e = acc / np.float64(self.W)", "mean_e = acc"),
    ("per worker: lambda* inverted", "inner[k] / norm_sq[k] if norm_sq[k] > 0", "norm_sq[k] / inner[k] if norm_sq[k] > 0"),
    ("per worker: inner product with itself", "np.sum(mean_e * e[k]) for k", "np.sum(e[k] * e[k]) for k"),
]

PHILOX_MUTANTS = [
    ("seed and step swapped", "philox4x64_10((int(t) & _MASK, 0, 0, 0), (int(seed) & _MASK, 0))",
     "philox4x64_10((int(seed) & _MASK, 0, 0, 0), (int(t) & _MASK, 0))"),
    ("nine rounds", "for _ in range(10):", "for _ in range(9):"),
    ("products swapped", "((prod_b >> 64) ^ c1 ^ k0, prod_b & _MASK,\n                          (prod_a >> 64) ^ c3 ^ k1, prod_a & _MASK)",
     "((prod_a >> 64) ^ c1 ^ k0, prod_a & _MASK,\n                          (prod_b >> 64) ^ c3 ^ k1, prod_b & _MASK)"),
    ("second output word", ")[0] % int(d)", ")[1] % int(d)"),
]


def test_unmodified_copy_passes_every_pin():
    mod, ph = _load(_SRC, _PHILOX_SRC)
    assert _run_pins(mod, ph) == 0


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new):
    assert _SRC.count(old) == 1, f"mutation target not unique/present: {old!r}"
    mod, ph = _load(_SRC.replace(old, new))
    assert _run_pins(mod, ph) >= 1, f"no pin noticed: {name}"


@pytest.mark.parametrize("name,old,new", PHILOX_MUTANTS, ids=[m[0] for m in PHILOX_MUTANTS])
def test_planted_generator_mistake_is_caught(name, old, new):
    assert _PHILOX_SRC.count(old) == 1, f"mutation target not unique/present: {old!r}"
    mod, ph = _load(_SRC, _PHILOX_SRC.replace(old, new))
    assert _run_pins(mod, ph) >= 1, f"no pin noticed: {name}"


# --------------------------------------------------------------------------- #
# The plain C oracle: planted mistakes in a private build of def_oracle.c must
# break its bit-agreement with the (mutant-pinned) numpy oracle.
# --------------------------------------------------------------------------- #
_C_SRC_PATH = os.path.join(os.path.dirname(real_module.__file__), "def_oracle.c")
_C_SRC = open(_C_SRC_PATH).read()

C_MUTANTS = [
    ("detach reads worker 0's error", "float scaled = lambda * e[(size_t)k * (size_t)n + (size_t)c];",
     "float scaled = lambda * e[(size_t)c];"),
    ("detach writes worker 0's row", "w[(size_t)k * (size_t)n + (size_t)c] = x[c] - scaled;",
     "w[(size_t)c] = x[c] - scaled;"),
    ("detach sign", "w[(size_t)k * (size_t)n + (size_t)c] = x[c] - scaled;",
     "w[(size_t)k * (size_t)n + (size_t)c] = x[c] + scaled;"),
    ("detach ignores lambda", "float scaled = lambda * e[(size_t)k * (size_t)n + (size_t)c];",
     "float scaled = e[(size_t)k * (size_t)n + (size_t)c];"),
    ("momentum dropped", "mk = carried + gk; ", "mk = gk;           "),
    ("block not zeroed", "ek[c] = 0.0f;                       /* ... and the residual there is +0  */",
     "ek[c] = p;"),
    ("no wrap", "if (j < 0) j += d;", ""),
    ("y not averaged", "y[c] = x[c] - acc / (float)W;", "y[c] = x[c] - acc;"),
    ("sum instead of mean", "cbar[c] = cbar[c] / (float)W;", ""),
]


def _c_agreement(library):
    saved = pins.DefOracleC
    if library is not None:
        pins.DefOracleC = lambda *a, **kw: saved(*a, library=library, **kw)
    try:
        pins.test_numpy_and_c_oracles_agree_bitwise()
    finally:
        pins.DefOracleC = saved


def _build_c(src, tmp_path, tag):
    import subprocess
    from oracle import c_oracle
    c_file = tmp_path / f"oracle_{tag}.c"
    so_file = tmp_path / f"liboracle_{tag}.so"
    c_file.write_text(src)
    subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                           "-o", str(so_file), str(c_file)])
    return c_oracle.load(str(so_file))


def test_unmodified_c_build_agrees(tmp_path):
    _c_agreement(_build_c(_C_SRC, tmp_path, "clean"))


@pytest.mark.parametrize("name,old,new", C_MUTANTS, ids=[m[0] for m in C_MUTANTS])
def test_planted_c_mistake_is_caught(tmp_path, name, old, new):
    assert _C_SRC.count(old) == 1, f"mutation target not unique/present: {old!r}"
    library = _build_c(_C_SRC.replace(old, new), tmp_path, "mutant")
    with pytest.raises(AssertionError):
        _c_agreement(library)
