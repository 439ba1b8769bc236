"""ctypes front end of gen.c (counter-based integer generator)."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libdgen.so")
_MASK64 = (1 << 64) - 1


def build(force=False):
    """Compile gen.c with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64 = ctypes.c_uint64
        lib.dgen_mix64.restype = u64
        lib.dgen_mix64.argtypes = [u64]
        lib.dgen_normal_f32.argtypes = [u64, u64, u64, ctypes.c_double, ctypes.c_void_p]
        lib.dgen_normal_bf16.argtypes = [u64, u64, u64, ctypes.c_double, ctypes.c_void_p]
        lib.dgen_uniform_i32.argtypes = [u64, u64, u64, ctypes.c_uint32, ctypes.c_void_p]
        lib.dgen_bits.argtypes = [u64, u64, u64, ctypes.c_void_p]
        for f in (lib.dgen_normal_f32, lib.dgen_normal_bf16, lib.dgen_uniform_i32, lib.dgen_bits):
            f.restype = None
        _lib = lib
    return _lib


def mix64(x):
    """SplitMix64 output function of a 64-bit integer."""
    return int(_load().dgen_mix64(x & _MASK64))


def stream_key(seed, tensor_id, layer=0, expert=0):
    """64-bit key of one value stream: distinct per (seed, tensor, layer, expert)."""
    tag = ((tensor_id & 0xFFFF) << 40) | ((layer & 0xFFFF) << 24) | (expert & 0xFFFFFF)
    return mix64((seed & _MASK64) ^ mix64(tag))


def normal(key, shape, std, dtype, first=0):
    """Approximately N(0, std^2) values; dtype 'f32' -> float32 array, 'bf16' -> uint16 bit patterns."""
    n = int(np.prod(shape))
    if dtype == "f32":
        out = np.empty(n, dtype=np.float32)
        _load().dgen_normal_f32(key, first, n, float(std), out.ctypes.data)
    elif dtype == "bf16":
        out = np.empty(n, dtype=np.uint16)
        _load().dgen_normal_bf16(key, first, n, float(std), out.ctypes.data)
    else:
        raise ValueError(dtype)
    return out.reshape(shape)


def uniform_ids(key, count, bound, first=0):
    """Uniform int32 on [0, bound)."""
    out = np.empty(int(count), dtype=np.int32)
    _load().dgen_uniform_i32(key, first, int(count), int(bound), out.ctypes.data)
    return out


def bernoulli_bits(key, count, first=0):
    """Bernoulli(1/2) as uint8 0/1."""
    out = np.empty(int(count), dtype=np.uint8)
    _load().dgen_bits(key, first, int(count), out.ctypes.data)
    return out
