"""Loader for the oracle's plain-C ring primitives (ring.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's cpu_baseline leg
import anything under oracle/.  Nothing here knows about the HIP library.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ring.c")
_LIB = os.path.join(_HERE, "_ring.so")


def build(force=False):
    """Compile ring.c with gcc (OpenMP over limbs is the only parallelism)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


_u64p = C.POINTER(C.c_uint64)
_i64p = C.POINTER(C.c_int64)


def _load():
    lib = C.CDLL(build())
    u64, i32 = C.c_uint64, C.c_int
    sig = {
        "orc_mulmod": ([u64, u64, u64], u64),
        "orc_powmod": ([u64, u64, u64], u64),
        "orc_ntt": ([_u64p, i32, i32, _u64p, _u64p], None),
        "orc_intt": ([_u64p, i32, i32, _u64p, _u64p], None),
        "orc_add": ([_u64p, _u64p, _u64p, i32, i32, _u64p], None),
        "orc_sub": ([_u64p, _u64p, _u64p, i32, i32, _u64p], None),
        "orc_mul": ([_u64p, _u64p, _u64p, i32, i32, _u64p], None),
        "orc_mac": ([_u64p, _u64p, _u64p, i32, i32, _u64p], None),
        "orc_mul_scalar": ([_u64p, _u64p, _u64p, i32, i32, _u64p], None),
        "orc_automorphism": ([_u64p, _u64p, i32, i32, _u64p, u64], None),
        "orc_reduce_i64": ([_u64p, _i64p, i32, i32, _u64p], None),
        "orc_reduce_u64": ([_u64p, _u64p, i32, i32, _u64p], None),
        "orc_base_conv": ([_u64p, _u64p, i32, i32, i32, _u64p, _u64p, _u64p, _u64p], None),
        "orc_rng_key": ([u64, u64], u64),
        "orc_rng_draw": ([u64, u64, u64], u64),
        "orc_sample_uniform": ([_u64p, i32, u64, u64, u64], None),
        "orc_sample_gauss": ([_i64p, i32, _u64p, i32, u64, u64], None),
    }
    for name, (args, res) in sig.items():
        f = getattr(lib, name)
        f.argtypes, f.restype = args, res
    return lib


lib = _load()


def u64(a):
    """Contiguous uint64 view/copy of an array-like."""
    return np.ascontiguousarray(a, dtype=np.uint64)


def p(a):
    assert a.dtype == np.uint64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_u64p)


def pi(a):
    assert a.dtype == np.int64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_i64p)
