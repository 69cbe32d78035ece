"""Build and load liboracle.so (plain C, gcc)."""
import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRC = os.path.join(_HERE, "oracle.c")
_lib = None

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force=True):
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _SO, _SRC, "-lm"])
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)   # also when the source is newer than the library
        _lib = ctypes.CDLL(_SO)
        _lib.orc_bf16_round_scalar.restype = ctypes.c_float
        _lib.orc_bf16_round_scalar.argtypes = [ctypes.c_float]
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib
