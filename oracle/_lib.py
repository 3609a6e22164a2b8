"""Builds and loads the C core of the oracle (attention_oracle.c) with gcc.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path imports this package.
"""
import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention_oracle.c")
_SO = os.path.join(_HERE, "liboracle_attention.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile attention_oracle.c into a shared object next to it."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _SO + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _SO)
    return _SO


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        vp, i64, i32, f64 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double
        L.oracle_attention.restype = i32
        L.oracle_attention.argtypes = [i32, vp, i64, vp, vp, i64, vp, vp, i64, vp,
                                       i32, i32, i32, f64, vp, vp]
        L.oracle_attention_rows.restype = i32
        L.oracle_attention_rows.argtypes = [i32, vp, i64, vp, vp, i64, vp, vp, i64, vp,
                                            i32, i32, i32, f64, vp, i64, vp, vp]
        L.oracle_num_threads.restype = i32
        L.oracle_num_threads.argtypes = []
        _lib = L
    return _lib
