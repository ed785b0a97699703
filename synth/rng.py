"""ctypes front end of rng.c (built with gcc on first use if the library is absent)."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "rng.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, vp = ctypes.c_uint64, ctypes.c_void_p
        lib.synth_normal_f32.argtypes = [u64, u64, u64, u64, ctypes.c_double, vp]
        lib.synth_normal_bf16.argtypes = [u64, u64, u64, u64, ctypes.c_double, vp]
        lib.synth_uniform_i32.argtypes = [u64, u64, u64, u64, ctypes.c_int32, ctypes.c_int32, vp]
        lib.synth_uniform_f64.argtypes = [u64, u64, u64, u64, vp]
        for f in (lib.synth_normal_f32, lib.synth_normal_bf16, lib.synth_uniform_i32, lib.synth_uniform_f64):
            f.restype = None
        _lib = lib
    return _lib


def normal_f32(seed, stream, n, scale=1.0, offset=0, out=None):
    """n values of scale*N(0,1) as float32; value i depends only on (seed, stream, offset+i)."""
    if out is None:
        out = np.empty(n, dtype=np.float32)
    assert out.dtype == np.float32 and out.size == n and out.flags.c_contiguous
    _load().synth_normal_f32(seed, stream, offset, n, float(scale), out.ctypes.data)
    return out


def normal_bf16(seed, stream, n, scale=1.0, offset=0, out=None):
    """Same values as normal_f32 rounded to nearest-even bfloat16, returned as uint16 bit patterns."""
    if out is None:
        out = np.empty(n, dtype=np.uint16)
    assert out.dtype == np.uint16 and out.size == n and out.flags.c_contiguous
    _load().synth_normal_bf16(seed, stream, offset, n, float(scale), out.ctypes.data)
    return out


def uniform_i32(seed, stream, n, lo, hi, offset=0):
    """n integers uniform in [lo, hi)."""
    out = np.empty(n, dtype=np.int32)
    _load().synth_uniform_i32(seed, stream, offset, n, int(lo), int(hi), out.ctypes.data)
    return out


def uniform_f64(seed, stream, n, offset=0):
    """n doubles uniform in [0, 1)."""
    out = np.empty(n, dtype=np.float64)
    _load().synth_uniform_f64(seed, stream, offset, n, out.ctypes.data)
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to the float32 values they denote."""
    return (bits.astype(np.uint32) << 16).view(np.float32)
