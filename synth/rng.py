"""ctypes front end of gen.c: counter-based draws addressed by (seed, stream, index)."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libheisd_synth.so")
_lib = None


def build_native(force: bool = False) -> str:
    """Compile gen.c into libheisd_synth.so next to it (gcc, OpenMP)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-o", tmp, src, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build_native()
        lib = ctypes.CDLL(_SO)
        u64, dbl, i32, vp = ctypes.c_uint64, ctypes.c_double, ctypes.c_int32, ctypes.c_void_p
        for name in ("synth_normal_f64", "synth_normal_f32", "synth_normal_bf16"):
            getattr(lib, name).argtypes = [u64, u64, u64, u64, dbl, dbl, vp]
            getattr(lib, name).restype = None
        lib.synth_uniform_i32.argtypes = [u64, u64, u64, u64, i32, i32, vp]
        lib.synth_uniform_i32.restype = None
        lib.synth_uniform_f64.argtypes = [u64, u64, u64, u64, vp]
        lib.synth_uniform_f64.restype = None
        _lib = lib
    return _lib


def stream_id(name: str) -> int:
    """Stable 64-bit id of a tensor name (FNV-1a)."""
    h = 0xCBF29CE484222325
    for b in name.encode():
        h = ((h ^ b) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def _sid(stream) -> int:
    return stream_id(stream) if isinstance(stream, str) else int(stream) & 0xFFFFFFFFFFFFFFFF


def _normal(fn, dtype, seed, stream, n, mean, std, first):
    out = np.empty(int(n), dtype=dtype)
    getattr(_load(), fn)(int(seed), _sid(stream), int(first), int(n), float(mean), float(std),
                          out.ctypes.data)
    return out


def normal_f64(seed, stream, n, mean=0.0, std=1.0, first=0):
    return _normal("synth_normal_f64", np.float64, seed, stream, n, mean, std, first)


def normal_f32(seed, stream, n, mean=0.0, std=1.0, first=0):
    return _normal("synth_normal_f32", np.float32, seed, stream, n, mean, std, first)


def normal_bf16(seed, stream, n, mean=0.0, std=1.0, first=0):
    """N(mean, std) rounded once (nearest-even) to bf16; returns the uint16 bit patterns."""
    return _normal("synth_normal_bf16", np.uint16, seed, stream, n, mean, std, first)


def uniform_i32(seed, stream, n, lo, hi, first=0):
    out = np.empty(int(n), dtype=np.int32)
    _load().synth_uniform_i32(int(seed), _sid(stream), int(first), int(n), int(lo), int(hi),
                              out.ctypes.data)
    return out


def uniform_f64(seed, stream, n, first=0):
    out = np.empty(int(n), dtype=np.float64)
    _load().synth_uniform_f64(int(seed), _sid(stream), int(first), int(n), out.ctypes.data)
    return out
