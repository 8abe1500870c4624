"""Loader for the C narrowing oracle (rne.c).  Test infrastructure only."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_rne.so")
_lib = None


def build(force=False):
    src = os.path.join(_HERE, "rne.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-o", tmp, src, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_narrow_rne.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t]
        lib.oracle_narrow_rne.restype = None
        _lib = lib
    return _lib


def narrow(bits_u32):
    """uint32 fp32 bit patterns -> uint16 bf16 bit patterns, same shape."""
    a = np.ascontiguousarray(bits_u32, dtype=np.uint32)
    out = np.empty(a.shape, dtype=np.uint16)
    if a.size:
        _load().oracle_narrow_rne(a.ctypes.data, out.ctypes.data, a.size)
    return out


def convert(bits, src_dtype, dst_dtype):
    """Element-wise storage conversion between the two dtypes of the path."""
    if src_dtype == dst_dtype:
        return np.array(bits, copy=True)
    if src_dtype == "f32" and dst_dtype == "bf16":
        return narrow(bits)
    raise ValueError("unsupported conversion %s -> %s" % (src_dtype, dst_dtype))
