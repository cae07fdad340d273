"""ctypes access to the format-variant reference codec in ``splitzip_variants_oracle.c``.

TEST INFRASTRUCTURE, like the package it sits in: imported by the tests and by
the benchmark's cpu_baseline leg only; imports nothing from the product.
Only argument marshalling happens here.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

BF16, E5M2, E4M3 = 0, 1, 2
ESC_POS, ESC_SENTINEL, ESC_ABS32 = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "splitzip_variants_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_splitzip_variants.so")
_lib = None


class Variant(C.Structure):
    _fields_ = [("dtype", C.c_uint32), ("code_bits", C.c_uint32), ("k", C.c_uint32),
                ("escape_mode", C.c_uint32), ("chunk", C.c_uint32), ("value_bits", C.c_uint32)]

    def __repr__(self):
        return (f"Variant(dtype={self.dtype}, code_bits={self.code_bits}, k={self.k}, "
                f"escape_mode={self.escape_mode}, chunk={self.chunk}, value_bits={self.value_bits})")


def variant(dtype, code_bits=4, k=16, escape_mode=ESC_POS, chunk=1024, value_bits=0) -> Variant:
    return Variant(dtype, code_bits, k, escape_mode, chunk, value_bits)


def build(force: bool = False) -> str:
    return _build(force=force, src=_SRC, out=_LIB)


def load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        vp = C.POINTER(Variant)
        u8p = C.POINTER(C.c_uint8)
        u64p = C.POINTER(C.c_uint64)
        lib.oracle_v_valid.restype = C.c_int
        lib.oracle_v_valid.argtypes = [vp]
        for f in (lib.oracle_v_payload_bytes, lib.oracle_v_total_bytes):
            f.restype = C.c_uint64
            f.argtypes = [C.c_uint64, C.c_uint64, vp]
        lib.oracle_v_calibrate.restype = C.c_int
        lib.oracle_v_calibrate.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, u8p, u64p]
        lib.oracle_v_compress.restype = C.c_int
        lib.oracle_v_compress.argtypes = [C.c_void_p, C.c_uint64, vp, u8p, C.c_void_p, C.c_uint64, u64p, u64p]
        lib.oracle_v_decompress.restype = C.c_int
        lib.oracle_v_decompress.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, vp, u8p, C.c_void_p]
        _lib = lib
    return _lib


def _u8(a):
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def _words(x: np.ndarray, dtype: int) -> np.ndarray:
    want = np.uint16 if dtype == BF16 else np.uint8
    x = np.ascontiguousarray(x)
    if x.dtype != want:
        raise TypeError(f"expected {want} words, got {x.dtype}")
    return x.reshape(-1)


def valid(v: Variant) -> bool:
    return bool(load().oracle_v_valid(C.byref(v)))


def payload_bytes(n: int, m: int, v: Variant) -> int:
    return int(load().oracle_v_payload_bytes(n, m, C.byref(v)))


def total_bytes(n: int, m: int, v: Variant) -> int:
    return int(load().oracle_v_total_bytes(n, m, C.byref(v)))


def calibrate(sample: np.ndarray, dtype: int, k: int):
    """Returns (dec[16] with the k most frequent exponents first, histogram[256])."""
    x = _words(sample, dtype)
    dec = np.zeros(16, np.uint8)
    hist = np.zeros(256, np.uint64)
    rc = load().oracle_v_calibrate(x.ctypes.data, x.size, dtype, k, _u8(dec),
                                   hist.ctypes.data_as(C.POINTER(C.c_uint64)))
    if rc:
        raise RuntimeError(f"oracle_v_calibrate failed: {rc}")
    return dec, hist


def compress(x: np.ndarray, v: Variant, dec, capacity: int | None = None):
    """Returns (blob of exactly total bytes, n_escapes)."""
    x = _words(x, v.dtype)
    dec = np.ascontiguousarray(dec, dtype=np.uint8)
    lib = load()
    tot, m = C.c_uint64(0), C.c_uint64(0)
    rc = lib.oracle_v_compress(x.ctypes.data, x.size, C.byref(v), _u8(dec), None, 0, C.byref(tot), C.byref(m))
    if rc != -2:
        raise RuntimeError(f"oracle_v_compress sizing failed: {rc}")
    cap = tot.value if capacity is None else capacity
    out = np.full(max(cap, 1), 0xA5, np.uint8)  # poison: every byte must be written by the codec
    rc = lib.oracle_v_compress(x.ctypes.data, x.size, C.byref(v), _u8(dec), out.ctypes.data, cap,
                               C.byref(tot), C.byref(m))
    if rc:
        raise RuntimeError(f"oracle_v_compress failed: {rc}")
    return out[: tot.value], int(m.value)


def decompress(blob: np.ndarray, n: int, v: Variant, dec) -> np.ndarray:
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    dec = np.ascontiguousarray(dec, dtype=np.uint8)
    out = np.zeros(n, np.uint16 if v.dtype == BF16 else np.uint8)
    rc = load().oracle_v_decompress(blob.ctypes.data, blob.size, n, C.byref(v), _u8(dec),
                                    out.ctypes.data if n else None)
    if rc:
        raise ValueError(f"oracle_v_decompress failed: {rc}")
    return out
