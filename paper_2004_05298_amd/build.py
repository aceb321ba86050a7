"""Builds the HIP library (libdef_hip.so) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
_CSRC = os.path.join(_PKG, "csrc")
_LIB = os.path.join(_PKG, "libdef_hip.so")

SOURCES = [os.path.join(_CSRC, "def_api.hip"), os.path.join(_CSRC, "def_kernels.hip"),
           os.path.join(_CSRC, "def_probe.hip")]
HEADERS = [os.path.join(_CSRC, "def_internal.h"), os.path.join(_ROOT, "include", "def.h"),
           os.path.join(_ROOT, "include", "def_probe.h")]

# -ffp-contract=off: every multiply and add rounds separately (results must not
#   depend on whether the compiler fuses them).
# -packed-fp32-ops disabled: packed fp32 instructions are kept out of the device code.
HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
    "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def library_path() -> str:
    """The in-tree library, or the build named by DEF_HIP_LIBRARY (to compare two builds)."""
    return os.environ.get("DEF_HIP_LIBRARY") or _LIB


def is_built() -> bool:
    return os.path.exists(_LIB)


def build_library(verbose: bool = False) -> str:
    """Compile unconditionally; returns the path of the shared library."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(_ROOT, "include"), "-I", _CSRC,
                                  "-o", _LIB] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose and res.stderr.strip():
        print(res.stderr)
    return _LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
