"""ctypes access to the plain C reference codec in ``splitzip_oracle.c``.

TEST INFRASTRUCTURE: imported by the tests, by the smoke check and by the
benchmark's cpu_baseline leg only.  The product package never imports this
module and this module imports nothing from the product package.

All functions take and return numpy arrays / Python ints; nothing here does any
codec arithmetic, it only marshals arguments for the C functions.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

BF16 = 0
E5M2 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "splitzip_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_splitzip.so")

_lib = None


def build(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the C oracle with gcc (-O2, no threads)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", src, "-o", out]
        )
    return out


def _bind(lib):
    u8p = C.POINTER(C.c_uint8)
    u64p = C.POINTER(C.c_uint64)
    lib.oracle_bf16_exponent.restype = C.c_uint8
    lib.oracle_bf16_exponent.argtypes = [C.c_uint16]
    lib.oracle_bf16_signmant.restype = C.c_uint8
    lib.oracle_bf16_signmant.argtypes = [C.c_uint16]
    lib.oracle_bf16_combine.restype = C.c_uint16
    lib.oracle_bf16_combine.argtypes = [C.c_uint8, C.c_uint8]
    lib.oracle_e5m2_exponent.restype = C.c_uint8
    lib.oracle_e5m2_exponent.argtypes = [C.c_uint8]
    lib.oracle_e5m2_signmant.restype = C.c_uint8
    lib.oracle_e5m2_signmant.argtypes = [C.c_uint8]
    lib.oracle_e5m2_combine.restype = C.c_uint8
    lib.oracle_e5m2_combine.argtypes = [C.c_uint8, C.c_uint8]
    for f in (lib.oracle_sm_bytes,):
        f.restype = C.c_uint64
        f.argtypes = [C.c_uint64, C.c_int]
    for f in (lib.oracle_payload_bytes, lib.oracle_total_bytes):
        f.restype = C.c_uint64
        f.argtypes = [C.c_uint64, C.c_uint64, C.c_int]
    lib.oracle_calibrate.restype = C.c_int
    lib.oracle_calibrate.argtypes = [C.c_void_p, C.c_uint64, C.c_int, u8p, u8p, u8p, u64p]
    lib.oracle_tables_from_dec.restype = C.c_int
    lib.oracle_tables_from_dec.argtypes = [u8p, C.c_int, u8p, u8p]
    lib.oracle_count_escapes.restype = C.c_uint64
    lib.oracle_count_escapes.argtypes = [C.c_void_p, C.c_uint64, C.c_int, u8p]
    lib.oracle_compress.restype = C.c_int
    lib.oracle_compress.argtypes = [C.c_void_p, C.c_uint64, C.c_int, u8p, u8p, u8p, C.c_void_p,
                                    C.c_uint64, u64p, u64p]
    lib.oracle_decompress.restype = C.c_int
    lib.oracle_decompress.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int, u8p, C.c_void_p]
    return lib


def load(path: str | None = None):
    """Load (building first if needed) the oracle library."""
    global _lib
    if path is not None:
        return _bind(C.CDLL(path))
    if _lib is None:
        _lib = _bind(C.CDLL(build()))
    return _lib


def _u8(a):
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def _words(x: np.ndarray, dtype: int) -> np.ndarray:
    want = np.uint16 if dtype == BF16 else np.uint8
    x = np.ascontiguousarray(x)
    if x.dtype != want:
        raise TypeError(f"expected {want} words, got {x.dtype}")
    return x.reshape(-1)


class Codebook:
    """The three calibration tables (decoding, encoding, membership)."""

    def __init__(self, dec, enc, member, dtype, hist=None):
        self.dec = np.ascontiguousarray(dec, dtype=np.uint8)
        self.enc = np.ascontiguousarray(enc, dtype=np.uint8)
        self.member = np.ascontiguousarray(member, dtype=np.uint8)
        self.dtype = int(dtype)
        self.hist = hist


def calibrate(sample: np.ndarray, dtype: int) -> Codebook:
    x = _words(sample, dtype)
    dec = np.zeros(16, np.uint8)
    enc = np.zeros(256, np.uint8)
    member = np.zeros(256, np.uint8)
    hist = np.zeros(256, np.uint64)
    rc = load().oracle_calibrate(x.ctypes.data, x.size, dtype, _u8(dec), _u8(enc), _u8(member),
                                 hist.ctypes.data_as(C.POINTER(C.c_uint64)))
    if rc:
        raise RuntimeError(f"oracle_calibrate failed: {rc}")
    return Codebook(dec, enc, member, dtype, hist)


def codebook_from_dec(dec, dtype: int) -> Codebook:
    dec = np.ascontiguousarray(dec, dtype=np.uint8)
    assert dec.size == 16
    enc = np.zeros(256, np.uint8)
    member = np.zeros(256, np.uint8)
    rc = load().oracle_tables_from_dec(_u8(dec), dtype, _u8(enc), _u8(member))
    if rc:
        raise ValueError(f"oracle_tables_from_dec failed: {rc}")
    return Codebook(dec, enc, member, dtype)


def count_escapes(x: np.ndarray, cb: Codebook) -> int:
    x = _words(x, cb.dtype)
    return int(load().oracle_count_escapes(x.ctypes.data, x.size, cb.dtype, _u8(cb.member)))


def sm_bytes(n: int, dtype: int) -> int:
    return int(load().oracle_sm_bytes(n, dtype))


def payload_bytes(n: int, m: int, dtype: int) -> int:
    return int(load().oracle_payload_bytes(n, m, dtype))


def total_bytes(n: int, m: int, dtype: int) -> int:
    return int(load().oracle_total_bytes(n, m, dtype))


def compress(x: np.ndarray, cb: Codebook, capacity: int | None = None):
    """Returns (blob uint8 array of exactly total bytes, n_escapes)."""
    x = _words(x, cb.dtype)
    lib = load()
    tot = C.c_uint64(0)
    m = C.c_uint64(0)
    # first call sizes the stream (capacity 0 reports the sizes and writes nothing)
    rc = lib.oracle_compress(x.ctypes.data, x.size, cb.dtype, _u8(cb.dec), _u8(cb.enc),
                             _u8(cb.member), None, 0, C.byref(tot), C.byref(m))
    if rc != -2:
        raise RuntimeError(f"oracle_compress sizing failed: {rc}")
    cap = tot.value if capacity is None else capacity
    out = np.full(max(cap, 1), 0xA5, np.uint8)  # poison: every byte must be written by the codec
    rc = lib.oracle_compress(x.ctypes.data, x.size, cb.dtype, _u8(cb.dec), _u8(cb.enc),
                             _u8(cb.member), out.ctypes.data, cap, C.byref(tot), C.byref(m))
    if rc:
        raise RuntimeError(f"oracle_compress failed: {rc}")
    return out[: tot.value], int(m.value)


def decompress(blob: np.ndarray, n: int, cb: Codebook) -> np.ndarray:
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    out = np.zeros(n, np.uint16 if cb.dtype == BF16 else np.uint8)
    rc = load().oracle_decompress(blob.ctypes.data, blob.size, n, cb.dtype, _u8(cb.dec),
                                  out.ctypes.data if n else None)
    if rc:
        raise ValueError(f"oracle_decompress failed: {rc}")
    return out
