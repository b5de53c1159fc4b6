"""numpy-facing wrapper of the CPU oracle (oracle/libtinykg_ref.so).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.
All arrays are host numpy arrays; every function returns fresh arrays.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _declare(_lib)
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _declare(L):
    u8p, f32p, u32p = C.POINTER(C.c_uint8), C.POINTER(C.c_float), C.POINTER(C.c_uint32)
    L.tinykg_ref_philox4x32_10.argtypes = [u32p, u32p, u32p]
    L.tinykg_ref_philox4x32_10.restype = None
    L.tinykg_ref_noise16.argtypes = [C.c_uint64, C.c_uint64]
    L.tinykg_ref_noise16.restype = C.c_uint32
    L.tinykg_ref_pack.argtypes = [u8p, C.c_int64, C.c_int, u8p]
    L.tinykg_ref_unpack.argtypes = [u8p, C.c_int64, C.c_int, u8p]
    L.tinykg_ref_quantize_codes.argtypes = [f32p, C.c_int64, C.c_int, C.c_int, C.c_uint64,
                                            C.c_uint64, C.c_int, u8p, f32p, f32p]
    L.tinykg_ref_quantize.argtypes = [f32p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64,
                                      C.c_uint64, C.c_int, u8p, f32p, f32p]
    L.tinykg_ref_dequantize.argtypes = [u8p, f32p, f32p, C.c_int64, C.c_int64, C.c_int, C.c_int,
                                        f32p]


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid arguments")


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    assert ctr.shape == (4,) and key.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    lib().tinykg_ref_philox4x32_10(_p(ctr, C.c_uint32), _p(key, C.c_uint32), _p(out, C.c_uint32))
    return out


def noise16(seed, index):
    return int(lib().tinykg_ref_noise16(C.c_uint64(seed), C.c_uint64(index)))


def pack(codes, bits):
    codes = np.ascontiguousarray(codes, dtype=np.uint8).ravel()
    out = np.empty(codes.size * bits // 8, dtype=np.uint8)
    _check(lib().tinykg_ref_pack(_p(codes, C.c_uint8), codes.size, bits, _p(out, C.c_uint8)), "pack")
    return out


def unpack(packed, n, bits):
    packed = np.ascontiguousarray(packed, dtype=np.uint8).ravel()
    assert packed.size * 8 >= n * bits
    out = np.empty(n, dtype=np.uint8)
    _check(lib().tinykg_ref_unpack(_p(packed, C.c_uint8), n, bits, _p(out, C.c_uint8)), "unpack")
    return out


def quantize_codes(act, bits, group, seed, first_index=0, rounding=0):
    """Unpacked codes (uint8, one per element), gmin, gscale."""
    act = np.ascontiguousarray(act, dtype=np.float32)
    n = act.size
    if group <= 0 or n % group:
        raise ValueError("oracle quantize: size not a multiple of the group")
    codes = np.empty(n, dtype=np.uint8)
    gmin = np.empty(n // group, dtype=np.float32)
    gscale = np.empty(n // group, dtype=np.float32)
    _check(lib().tinykg_ref_quantize_codes(_p(act, C.c_float), n, bits, group, C.c_uint64(seed),
                                           C.c_uint64(first_index), rounding, _p(codes, C.c_uint8),
                                           _p(gmin, C.c_float), _p(gscale, C.c_float)),
           "quantize_codes")
    return codes, gmin, gscale


def quantize(act, bits, group, seed, first_index=0, rounding=0):
    """Packed bit-stream (uint8), gmin, gscale for a 2-D (or flat) fp32 array."""
    act = np.ascontiguousarray(act, dtype=np.float32)
    rows, dim = (act.shape if act.ndim == 2 else (1, act.size))
    n = act.size
    if group <= 0 or n % group:
        raise ValueError("oracle quantize: size not a multiple of the group")
    packed = np.empty(n * bits // 8, dtype=np.uint8)
    gmin = np.empty(n // group, dtype=np.float32)
    gscale = np.empty(n // group, dtype=np.float32)
    _check(lib().tinykg_ref_quantize(_p(act, C.c_float), rows, dim, bits, group, C.c_uint64(seed),
                                     C.c_uint64(first_index), rounding, _p(packed, C.c_uint8),
                                     _p(gmin, C.c_float), _p(gscale, C.c_float)), "quantize")
    return packed, gmin, gscale


def dequantize(packed, gmin, gscale, rows, dim, bits, group):
    packed = np.ascontiguousarray(packed, dtype=np.uint8).ravel()
    gmin = np.ascontiguousarray(gmin, dtype=np.float32)
    gscale = np.ascontiguousarray(gscale, dtype=np.float32)
    n = rows * dim
    assert packed.size == n * bits // 8 and gmin.size == n // group == gscale.size
    out = np.empty((rows, dim), dtype=np.float32)
    _check(lib().tinykg_ref_dequantize(_p(packed, C.c_uint8), _p(gmin, C.c_float),
                                       _p(gscale, C.c_float), rows, dim, bits, group,
                                       _p(out, C.c_float)), "dequantize")
    return out
