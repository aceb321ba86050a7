"""Thin ctypes binding of the C ABI in include/def.h.

Argument marshalling only: every step of the method runs in the HIP kernels of
libdef_hip.so.  torch supplies device memory (tensor.data_ptr()) and the stream
handle, nothing else.  There is no CPU fallback: if the library has not been
built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

from . import build as _build

DEF_OK, DEF_EINVAL, DEF_ENOMEM, DEF_EHIP, DEF_ELIMIT = 0, -1, -2, -3, -4
DEF_STATIC_MAX_D = 268435456

_u64, _u32, _i64, _f32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int64, ctypes.c_float
_vp = ctypes.c_void_p


class DefConfig(ctypes.Structure):
    """Mirror of `def_config`."""
    _fields_ = [
        ("d", _u64), ("W", _u32), ("R", _u32),
        ("lr", _f32), ("momentum", _f32), ("weight_decay", _f32),
        ("seed", _u64),
        ("tensor_offsets", ctypes.POINTER(_u64)), ("n_tensors", _u32),
        ("params", _vp), ("param_ptrs", ctypes.POINTER(_vp)),
        ("stream", _vp),
    ]


# name -> (restype, argtypes); every symbol include/def.h declares
SIGNATURES = {
    "def_init": (ctypes.c_int, [ctypes.POINTER(_vp), ctypes.POINTER(DefConfig)]),
    "def_destroy": (ctypes.c_int, [_vp]),
    "def_step": (ctypes.c_int, [_vp, _vp, _u64, _vp]),
    "def_a_step": (ctypes.c_int, [_vp, _vp, _u64]),
    "def_step_tensors": (ctypes.c_int, [_vp, ctypes.POINTER(_vp), _vp]),
    "def_a_step_tensors": (ctypes.c_int, [_vp, ctypes.POINTER(_vp)]),
    "def_pack": (ctypes.c_int, [_vp, _vp, _u64, ctypes.POINTER(_vp)]),
    "def_pack_tensors": (ctypes.c_int, [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp)]),
    "def_apply": (ctypes.c_int, [_vp, _vp, _f32, _vp]),
    "def_output": (ctypes.c_int, [_vp, _vp]),
    "def_set_detach": (ctypes.c_int, [_vp, _vp, _u64, _f32]),
    "def_detach": (ctypes.c_int, [_vp, _vp, _u64, _f32]),
    "def_diagnostics": (ctypes.c_int, [_vp, _f32, _vp]),
    "def_diagnostics_static": (ctypes.c_int, [_vp, _u64, _u64, _u32, _f32, _vp, _vp]),
    "def_diagnostics_workers": (ctypes.c_int, [_vp, _vp]),
    "def_block_length": (ctypes.c_int, [_vp, ctypes.POINTER(_u64)]),
    "def_set_seed": (ctypes.c_int, [_vp, _u64]),
    "def_set_device_draw": (ctypes.c_int, [_vp, ctypes.c_int]),
    "def_sync_step": (ctypes.c_int, [_vp]),
    "def_set_lr": (ctypes.c_int, [_vp, _f32]),
    "def_set_step": (ctypes.c_int, [_vp, _u64]),
    "def_get_step": (ctypes.c_int, [_vp, ctypes.POINTER(_u64)]),
    "def_force_next_start": (ctypes.c_int, [_vp, _i64]),
    "def_last_block": (ctypes.c_int, [_vp, ctypes.POINTER(_u64), ctypes.POINTER(_u64)]),
    "def_block_start": (ctypes.c_int, [_u64, _u64, _u64, ctypes.POINTER(_u64)]),
    "def_state_ptrs": (ctypes.c_int, [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp),
                                      ctypes.POINTER(_vp), ctypes.POINTER(_u64)]),
    "def_last_path": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_int)]),
    "def_last_kernel": (ctypes.c_char_p, [_vp]),
    "def_profile_begin": (ctypes.c_int, [_vp, _u32]),
    "def_profile_end": (ctypes.c_int, [_vp, ctypes.POINTER(_f32), _u32, ctypes.POINTER(_u32)]),
    "def_probe_stream": (ctypes.c_int, [ctypes.c_int, _vp, _vp, _u64, _f32, _u32, _u32, _u32, _vp]),
    "def_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "def_last_hip_error": (ctypes.c_int, []),
}

_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libdef_hip.so (building nothing).  Raises if it is missing."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    # torch ships its own HIP runtime; importing it first makes the dynamic loader
    # resolve this library's libamdhip64 dependency to that same copy, so that
    # torch's streams and allocations are valid handles inside the library.
    import torch  # noqa: F401
    path = path or _build.library_path()
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} not found: build the HIP library first "
            "(python -c 'import __graft_entry__ as g; g.build()'); there is no CPU fallback")
    lib = ctypes.CDLL(path)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


class DefError(RuntimeError):
    def __init__(self, status: int, where: str):
        lib = load_library()
        msg = lib.def_strerror(status).decode()
        if status == DEF_EHIP:
            msg += f" (hip error {lib.def_last_hip_error()})"
        super().__init__(f"{where}: {msg}")
        self.status = status


def _check(status: int, where: str) -> None:
    if status != DEF_OK:
        raise DefError(status, where)


def block_start(seed: int, t: int, d: int) -> int:
    out = _u64()
    _check(load_library().def_block_start(seed, t, d, ctypes.byref(out)), "def_block_start")
    return out.value


def diagnostics_static(e, ld: int, d: int, W: int, lam: float, out, stream: int = 0) -> None:
    """def_diagnostics_static: e is a device tensor (or address) [W][ld], out 4 float64 on the device."""
    _check(load_library().def_diagnostics_static(_ptr(e), ld, d, W, lam, _ptr(out), stream),
           "def_diagnostics_static")


PROBE_READ, PROBE_WRITE, PROBE_COPY, PROBE_UPDATE = 0, 1, 2, 3


def probe_stream(kind: int, src, dst, n: int, value: float = 1.0, threads: int = 64, quads: int = 1,
                 lds_reserve: int = 10240, stream: int = 0) -> None:
    """def_probe_stream (include/def_probe.h): one streaming launch of known traffic."""
    _check(load_library().def_probe_stream(kind, _ptr(src), _ptr(dst), n, value, threads, quads,
                                           lds_reserve, stream), "def_probe_stream")


def _ptr(t) -> int:
    """Device address of a torch tensor (or a raw integer address)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return t.data_ptr()


class _DeviceArray:
    """Minimal __cuda_array_interface__ holder so that torch can view library-owned memory."""

    def __init__(self, ptr: int, shape, strides_bytes=None):
        self.__cuda_array_interface__ = {
            "shape": tuple(int(v) for v in shape), "typestr": "<f4", "data": (int(ptr), False),
            "version": 2, "strides": strides_bytes,
        }


def device_view(ptr: int, shape):
    """Zero-copy float32 torch tensor over device memory at `ptr` (row-major)."""
    import torch
    return torch.as_tensor(_DeviceArray(ptr, shape), device="cuda")


class DefContext:
    """Owner of one `def_ctx`.  Method names follow the C entry points."""

    def __init__(self, d: int, W: int, R: int, lr: float, momentum: float = 0.0,
                 weight_decay: float = 0.0, seed: int = 0, params=None,
                 param_tensors: Optional[Sequence] = None,
                 tensor_offsets: Optional[Sequence[int]] = None, stream: int = 0):
        self._lib = load_library()
        self._h = _vp()
        cfg = DefConfig()
        cfg.d, cfg.W, cfg.R = d, W, R
        cfg.lr, cfg.momentum, cfg.weight_decay = lr, momentum, weight_decay
        cfg.seed = seed
        self._keep: List[object] = [params, param_tensors]
        # the C side reads n_tensors+1 offsets and n_tensors pointers: lengths are checked here
        n_tensors = 1 if tensor_offsets is None else len(tensor_offsets) - 1
        if n_tensors < 1:
            raise ValueError("tensor_offsets needs at least two entries")
        if param_tensors is not None and len(param_tensors) != n_tensors:
            raise ValueError(f"param_tensors has {len(param_tensors)} entries for {n_tensors} tensors")
        if params is None and param_tensors is None:
            raise ValueError("give params (one flat vector) or param_tensors")
        if tensor_offsets is not None:
            arr = (_u64 * len(tensor_offsets))(*[int(v) for v in tensor_offsets])
            cfg.tensor_offsets = ctypes.cast(arr, ctypes.POINTER(_u64))
            cfg.n_tensors = len(tensor_offsets) - 1
        else:
            cfg.tensor_offsets = None
            cfg.n_tensors = 1
        cfg.params = _ptr(params)
        if param_tensors is not None:
            parr = (_vp * len(param_tensors))(*[_ptr(p) for p in param_tensors])
            cfg.param_ptrs = ctypes.cast(parr, ctypes.POINTER(_vp))
        else:
            cfg.param_ptrs = None
        cfg.stream = stream
        self.d, self.W, self.R = d, W, R
        self.n_tensors = cfg.n_tensors
        _check(self._lib.def_init(ctypes.byref(self._h), ctypes.byref(cfg)), "def_init")

    # -- lifetime -------------------------------------------------------------
    def destroy(self) -> None:
        if self._h:
            h, self._h = self._h, _vp()
            _check(self._lib.def_destroy(h), "def_destroy")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()

    # -- steps ----------------------------------------------------------------
    def step(self, grads, ld: int, y_out=None) -> None:
        _check(self._lib.def_step(self._h, _ptr(grads), ld, _ptr(y_out)), "def_step")

    def a_step(self, grads, ld: int) -> None:
        _check(self._lib.def_a_step(self._h, _ptr(grads), ld), "def_a_step")

    def _gtable(self, grad_tensors):
        flat = [_ptr(g) for g in grad_tensors]
        if len(flat) != self.W * self.n_tensors:      # the C side reads exactly W*n_tensors entries
            raise ValueError(f"{len(flat)} gradient tensors given, W*n_tensors = {self.W * self.n_tensors}")
        return (_vp * len(flat))(*flat)

    def step_tensors(self, grad_tensors: Sequence, y_out=None) -> None:
        """grad_tensors: W*n_tensors tensors, worker-major."""
        tbl = self._gtable(grad_tensors)
        _check(self._lib.def_step_tensors(self._h, ctypes.cast(tbl, ctypes.POINTER(_vp)), _ptr(y_out)),
               "def_step_tensors")

    def a_step_tensors(self, grad_tensors: Sequence) -> None:
        tbl = self._gtable(grad_tensors)
        _check(self._lib.def_a_step_tensors(self._h, ctypes.cast(tbl, ctypes.POINTER(_vp))),
               "def_a_step_tensors")

    def pack(self, grads, ld: int) -> int:
        """First half of a split iteration; returns the device address of the B-float sum
        of the local workers' kept blocks (see block_view)."""
        out = _vp()
        _check(self._lib.def_pack(self._h, _ptr(grads), ld, ctypes.byref(out)), "def_pack")
        return out.value or 0

    def pack_tensors(self, grad_tensors: Sequence) -> int:
        tbl = self._gtable(grad_tensors)
        out = _vp()
        _check(self._lib.def_pack_tensors(self._h, ctypes.cast(tbl, ctypes.POINTER(_vp)), ctypes.byref(out)),
               "def_pack_tensors")
        return out.value or 0

    def block_length(self) -> int:
        n = _u64()
        _check(self._lib.def_block_length(self._h, ctypes.byref(n)), "def_block_length")
        return n.value

    def block_view(self, ptr: int):
        """torch view [B] of the vector def_pack returned (what a collective would reduce)."""
        return device_view(ptr, (self.block_length(),))

    def apply(self, block, divisor: float, y_out=None) -> None:
        _check(self._lib.def_apply(self._h, _ptr(block), divisor, _ptr(y_out)), "def_apply")

    def output(self, y_out) -> None:
        _check(self._lib.def_output(self._h, _ptr(y_out)), "def_output")

    def set_detach(self, w_out, ldw: int = 0, lam: float = 0.0) -> None:
        self._detach_out = w_out                      # keep the tensor alive while it is set
        _check(self._lib.def_set_detach(self._h, _ptr(w_out), ldw, lam), "def_set_detach")

    def detach(self, w_out, ldw: int, lam: float) -> None:
        _check(self._lib.def_detach(self._h, _ptr(w_out), ldw, lam), "def_detach")

    def diagnostics(self, lam: float, out) -> None:
        """out: float64 device tensor with 4 entries (see def_diagnostics)."""
        _check(self._lib.def_diagnostics(self._h, lam, _ptr(out)), "def_diagnostics")

    def diagnostics_workers(self, out) -> None:
        """out: float64 device tensor with 3*W entries (see def_diagnostics_workers)."""
        _check(self._lib.def_diagnostics_workers(self._h, _ptr(out)), "def_diagnostics_workers")

    # -- knobs ----------------------------------------------------------------
    def set_seed(self, seed: int) -> None:
        _check(self._lib.def_set_seed(self._h, seed), "def_set_seed")

    def set_device_draw(self, on: bool) -> None:
        _check(self._lib.def_set_device_draw(self._h, 1 if on else 0), "def_set_device_draw")

    def sync_step(self) -> None:
        _check(self._lib.def_sync_step(self._h), "def_sync_step")

    def set_lr(self, lr: float) -> None:
        _check(self._lib.def_set_lr(self._h, lr), "def_set_lr")

    def set_step(self, t: int) -> None:
        _check(self._lib.def_set_step(self._h, t), "def_set_step")

    def get_step(self) -> int:
        t = _u64()
        _check(self._lib.def_get_step(self._h, ctypes.byref(t)), "def_get_step")
        return t.value

    def force_next_start(self, s: int) -> None:
        _check(self._lib.def_force_next_start(self._h, s), "def_force_next_start")

    def last_block(self):
        s, n = _u64(), _u64()
        _check(self._lib.def_last_block(self._h, ctypes.byref(s), ctypes.byref(n)), "def_last_block")
        return s.value, n.value

    def last_path_flat(self) -> bool:
        v = ctypes.c_int()
        _check(self._lib.def_last_path(self._h, ctypes.byref(v)), "def_last_path")
        return bool(v.value)

    def last_kernel(self) -> Optional[str]:
        name = self._lib.def_last_kernel(self._h)
        return name.decode() if name else None

    def state_ptrs(self):
        """(e_ptr, m_ptr, avg_block_ptr, ld_state) as integers."""
        e, m, a, ld = _vp(), _vp(), _vp(), _u64()
        _check(self._lib.def_state_ptrs(self._h, ctypes.byref(e), ctypes.byref(m), ctypes.byref(a),
                                        ctypes.byref(ld)), "def_state_ptrs")
        return e.value or 0, m.value or 0, a.value or 0, ld.value

    def state_tensors(self):
        """(e, m, avg_block) as torch views of the library-owned buffers: e and m
        are [W][ld_state] (m is None without momentum), avg_block is [B]."""
        e, m, a, ld = self.state_ptrs()
        return (device_view(e, (self.W, ld)), device_view(m, (self.W, ld)) if m else None,
                device_view(a, (self.block_length(),)))

    # -- timing ---------------------------------------------------------------
    def profile_begin(self, max_steps: int) -> None:
        _check(self._lib.def_profile_begin(self._h, max_steps), "def_profile_begin")

    def profile_end(self, cap: int) -> List[float]:
        buf = (_f32 * max(cap, 1))()
        n = _u32()
        _check(self._lib.def_profile_end(self._h, buf, cap, ctypes.byref(n)), "def_profile_end")
        return [buf[i] for i in range(min(cap, n.value))]
