"""Builds and loads the multi-threaded feature-table writer (wl_fill.c)."""
import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wl_fill.c")
_LIB = os.path.join(_HERE, "libwl_fill.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def load() -> ctypes.CDLL:
    lib = ctypes.CDLL(build())
    lib.wl_fill_store.restype = None
    return lib
