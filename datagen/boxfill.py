"""ctypes front end of datagen/boxfill.c (compiled on first use with gcc)."""
import ctypes as C
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libboxfill.so")
_lib = None


def build(force=False):
    src = [os.path.join(HERE, "boxfill.c"), os.path.join(HERE, "pattern.h")]
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(s) for s in src):
        subprocess.run(["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", LIB, src[0]], check=True)
    return LIB


def fill_box(seed, kind, tensor, shape, lo, ext, out):
    """Write the pattern words of box [lo, lo+ext) of `tensor` into `out` (uint16/uint32 array)."""
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.vps_pattern_fill_box.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.POINTER(C.c_int32),
                                              C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_void_p]
        _lib.vps_pattern_fill_box.restype = None
    n = int(np.prod([int(e) for e in ext]))
    assert out.size == n and out.dtype == (np.uint16 if kind == 0 else np.uint32) and out.flags.c_contiguous
    arr = lambda v: (C.c_int32 * 4)(*[int(x) for x in v])
    _lib.vps_pattern_fill_box(seed, kind, tensor, arr(shape), arr(lo), arr(ext), out.ctypes.data)
    return out
