"""CPU checker for the kernel sources (test helper, not collected by pytest).

Builds paper_1811_00778_amd/csrc/hcnn.cpp with -DHCNN_HOSTEMU (g++, no HIP): the same
kernel phase bodies and the same host orchestration run as loops over blocks and
threads on host memory.  Lets the CPU test-suite compare kernel indexing and
arithmetic with the oracle before anything runs on a GPU.  The product binding never
loads this library.
"""
import ctypes
import os
import subprocess

import numpy as np

from paper_1811_00778_amd import _capi
from paper_1811_00778_amd._ops import OpsMixin

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_SRC_DIR = os.path.join(_ROOT, "paper_1811_00778_amd", "csrc")
_OUT_DIR = os.path.join(_ROOT, "tests", "_build")
# HCNN_EMU_SANITIZE=1: build and load the checker with AddressSanitizer and UndefinedBehaviorSanitizer (host code
# only: this is the one build in which the kernels' indexing runs under a bounds checker).  The sanitizer runtime
# has to be in the process before Python starts, so run it as
#     HCNN_EMU_SANITIZE=1 LD_PRELOAD=$(g++ -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
#         python -m pytest tests/test_emu_parity.py -q
SANITIZE = os.environ.get("HCNN_EMU_SANITIZE", "") not in ("", "0")
_OUT = os.path.join(_OUT_DIR, "libhcnn_emu_san.so" if SANITIZE else "libhcnn_emu.so")
_lib = None


def build() -> str:
    os.makedirs(_OUT_DIR, exist_ok=True)
    srcs = [os.path.join(_SRC_DIR, f) for f in os.listdir(_SRC_DIR)] + [os.path.join(_ROOT, "include", "hcnn.h")]
    if os.path.exists(_OUT) and all(os.path.getmtime(s) <= os.path.getmtime(_OUT) for s in srcs):
        return _OUT
    tmp = _OUT + ".tmp.%d" % os.getpid()
    extra = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] \
        if SANITIZE else ["-O2"]
    subprocess.check_call(["g++", "-std=c++17"] + extra + ["-DHCNN_HOSTEMU", "-fPIC", "-shared", "-Wall", "-Wextra",
                           "-Wno-unused-parameter", "-Wno-unknown-pragmas", "-o", tmp,
                           os.path.join(_SRC_DIR, "hcnn.cpp")])
    os.replace(tmp, _OUT)
    return _OUT


def lib():
    global _lib
    if _lib is None:
        _lib = _capi.declare(ctypes.CDLL(build()))
    return _lib


class EmuContext(OpsMixin):
    def __init__(self, n, q, p, t):
        self.raw = _capi.RawContext(lib(), n, q, p, t, 0)

    def _ptr(self, x):
        return ctypes.c_void_p(x.ctypes.data)

    _NP = {"u32": np.uint32, "i32": np.int32, "u64": np.uint64}

    def _empty(self, shape, dtype_name):
        return np.empty(shape, dtype=self._NP[dtype_name])

    def _check(self, x, dtype_name):
        want = self._NP[dtype_name]
        if not isinstance(x, np.ndarray) or x.dtype != want or not x.flags["C_CONTIGUOUS"]:
            raise TypeError("expected contiguous %s ndarray" % want.__name__)
        if x.ctypes.data % 16:
            raise TypeError("array not 16-byte aligned")


def aligned(a):
    """Copy of a in 16-byte aligned storage (numpy gives 16-byte alignment for fresh allocations)."""
    out = np.empty(a.shape, dtype=a.dtype)
    assert out.ctypes.data % 16 == 0
    out[...] = a
    return out
