"""Compile the oracle's C loops with gcc (TEST INFRASTRUCTURE ONLY).

Run as `python -m oracle.build`, or call `build()`; `load()` builds on first
use when the shared object is missing or older than its source.
"""
import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "ckernels.c")
OUT_DIR = os.path.join(_HERE, "_build")
OUT = os.path.join(OUT_DIR, "liboracle.so")


def build(force: bool = True) -> str:
    os.makedirs(OUT_DIR, exist_ok=True)
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    tmp = OUT + ".tmp.%d" % os.getpid()
    subprocess.check_call(
        ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", tmp, SRC]
    )
    os.replace(tmp, OUT)
    return OUT


_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build(force=False))
    return _lib


if __name__ == "__main__":
    print(build())
