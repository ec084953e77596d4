"""Builds and loads the oracle's C sources with gcc (test infrastructure)."""
from __future__ import annotations

import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("draft_oracle.c", "accept_oracle.c")]
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build_oracle_lib(force: bool = False) -> str:
    """Compile the oracle's C files (plain -O2; the oracle is never tuned)."""
    stale = (not os.path.exists(_SO)) or any(os.path.getmtime(_SO) < os.path.getmtime(s) for s in _SRCS)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", _SO] + _SRCS + ["-lm"])
    return _SO


def load():
    global _lib
    if _lib is None:
        build_oracle_lib()
        lib = ctypes.CDLL(_SO)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.draft_oracle.argtypes = [i32p, ctypes.c_int64, ctypes.c_int32, i32p, ctypes.c_int32,
                                     ctypes.c_int32, ctypes.c_int32, i32p, i32p, i32p, i64p]
        lib.draft_oracle.restype = None
        lib.draft_oracle_batch.argtypes = [i32p, i64p, i64p, ctypes.c_int32, i32p, i32p, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           i32p, i32p, i32p, i64p]
        lib.draft_oracle_batch.restype = None
        lib.accept_oracle.argtypes = [f32p, i32p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                      i32p, i32p, i32p]
        lib.accept_oracle.restype = None
        _lib = lib
    return _lib


def ptr(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))
