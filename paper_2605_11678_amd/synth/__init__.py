"""Seeded synthetic inputs (weights, tokens) — input generation only.

A thin ctypes wrapper over ``synth.c``.  Element i of a stream depends only on
(seed, stream, i).  This module holds none of the method's arithmetic and is
the one piece of code that both the HIP path's callers and the oracle's
callers use.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libsynth.so")
        if not os.path.exists(path):
            from .. import build
            build.build_synth()
        lib = ctypes.CDLL(path)
        for name, ptr in (("synth_normal_bf16", ctypes.c_void_p), ("synth_normal_bf16_as_f32", ctypes.c_void_p)):
            f = getattr(lib, name)
            f.restype = None
            f.argtypes = [ptr, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                          ctypes.c_float, ctypes.c_float]
        _LIB = lib
    return _LIB


def normal_bf16(n, seed, stream, mean=0.0, std=1.0, first=0, out=None):
    """uint16 array of BF16 bit patterns, value = bf16(mean + std * N(0,1))."""
    if out is None:
        out = np.empty(int(n), dtype=np.uint16)
    assert out.dtype == np.uint16 and out.flags.c_contiguous and out.size == n
    _lib().synth_normal_bf16(out.ctypes.data, first, n, seed, stream, mean, std)
    return out


def normal_bf16_as_f32(n, seed, stream, mean=0.0, std=1.0, first=0):
    """float32 array whose every value is exactly BF16-representable."""
    out = np.empty(int(n), dtype=np.float32)
    _lib().synth_normal_bf16_as_f32(out.ctypes.data, first, n, seed, stream, mean, std)
    return out


def bf16_bits_to_f32(bits):
    """Exact widening of BF16 bit patterns (uint16) to float32."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
