"""ctypes front end of the CPU oracle (oracle/taco_ref.cpp).  Test infrastructure only.

All arrays are numpy host arrays.  bf16 tensors travel as uint16 bit patterns.
The functions mirror Algorithm 1 of the TACO paper: compress (sender side),
decompress (receiver side) and decompress_sum (receiver side followed by the local
reduction of Section 4.4.2).
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        # TACO_REF_LIB: load another build of the oracle instead (the mutation test plants mistakes in copies of it)
        path = os.environ.get("TACO_REF_LIB") or _build.LIB
        if path == _build.LIB and (not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC)):
            _build.build(force=True)
        L = ctypes.CDLL(path)
        c = ctypes
        L.taco_ref_threads.restype = c.c_int
        L.taco_ref_threads.argtypes = []
        L.taco_ref_set_threads.restype = c.c_int
        L.taco_ref_set_threads.argtypes = [c.c_int]
        L.taco_ref_e4m3_decode.restype = c.c_double
        L.taco_ref_e4m3_decode.argtypes = [c.c_uint8]
        L.taco_ref_e4m3_encode.restype = c.c_uint8
        L.taco_ref_e4m3_encode.argtypes = [c.c_double]
        L.taco_ref_format_decode.restype = c.c_double
        L.taco_ref_format_decode.argtypes = [c.c_int32, c.c_uint8]
        L.taco_ref_format_encode.restype = c.c_uint8
        L.taco_ref_format_encode.argtypes = [c.c_int32, c.c_double]
        L.taco_ref_float_to_bf16.restype = c.c_uint16
        L.taco_ref_float_to_bf16.argtypes = [c.c_float]
        L.taco_ref_hadamard_matrix.restype = c.c_int
        L.taco_ref_hadamard_matrix.argtypes = [c.c_int32, c.c_void_p]
        L.taco_ref_rotate.restype = c.c_int
        L.taco_ref_rotate.argtypes = [c.c_void_p, c.c_int32, c.c_void_p]
        L.taco_ref_compress.restype = c.c_int
        L.taco_ref_compress.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_float, c.c_float,
                                        c.c_void_p, c.c_void_p, c.c_void_p]
        L.taco_ref_compress_ex.restype = c.c_int
        L.taco_ref_compress_ex.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_float, c.c_float, c.c_int32, c.c_int32,
                                           c.c_void_p, c.c_void_p, c.c_void_p]
        L.taco_ref_decompress_sum_ex.restype = c.c_int
        L.taco_ref_decompress_sum_ex.argtypes = [c.c_void_p, c.c_void_p, c.c_int32, c.c_int64, c.c_int32, c.c_int32,
                                                 c.c_int32, c.c_void_p, c.c_void_p]
        L.taco_ref_decompress_sum.restype = c.c_int
        L.taco_ref_decompress_sum.argtypes = [c.c_void_p, c.c_void_p, c.c_int32, c.c_int64,
                                              c.c_int32, c.c_void_p, c.c_void_p]
        L.taco_ref_decompress.restype = c.c_int
        L.taco_ref_decompress.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int32,
                                          c.c_void_p, c.c_void_p]
        _LIB = L
    return _LIB


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(lib().taco_ref_threads())


def set_threads(threads: int) -> int:
    """Threads the block loops use from now on (results do not depend on it); returns the number in effect."""
    return int(lib().taco_ref_set_threads(int(threads)))


def e4m3_decode(code: int) -> float:
    return lib().taco_ref_e4m3_decode(int(code) & 0xFF)


def e4m3_encode(v: float) -> int:
    return int(lib().taco_ref_e4m3_encode(float(v)))


FORMAT_E4M3, FORMAT_E5M2, FORMAT_INT8 = 0, 1, 2
MODE_RESCALE, MODE_ROTATE, MODE_POSTSCALE, MODE_FULL = 1, 2, 4, 7


def format_decode(fmt: int, code: int) -> float:
    return lib().taco_ref_format_decode(int(fmt), int(code) & 0xFF)


def format_encode(fmt: int, v: float) -> int:
    return int(lib().taco_ref_format_encode(int(fmt), float(v)))


def float_to_bf16(f: float) -> int:
    return int(lib().taco_ref_float_to_bf16(float(f)))


def hadamard_matrix(block: int) -> np.ndarray:
    H = np.empty((block, block), dtype=np.float64)
    rc = lib().taco_ref_hadamard_matrix(block, _ptr(H))
    if rc != 0:
        raise ValueError(f"taco_ref_hadamard_matrix({block}) -> {rc}")
    return H


def rotate(x: np.ndarray) -> np.ndarray:
    """(1/sqrt(B)) H_B x for one block, B = len(x)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    rc = lib().taco_ref_rotate(_ptr(x), x.size, _ptr(y))
    if rc != 0:
        raise ValueError(f"taco_ref_rotate(B={x.size}) -> {rc}")
    return y


def n_blocks(n: int, block: int) -> int:
    return (n + block - 1) // block


def compress(x_bf16: np.ndarray, block: int = 128, tau: float = 1.0, eps: float = 1e-12,
             want_z: bool = False, mode: int = MODE_FULL, fmt: int = FORMAT_E4M3):
    """x_bf16: uint16 array (any shape, flattened row-major).
    Returns (payload uint8[M*B], scales float32[M,2] = {alpha, s}) and, if want_z,
    the rotated values Z (float64[M*B]) before quantisation."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16).reshape(-1)
    n = x.size
    M = n_blocks(n, block)
    payload = np.empty(M * block, dtype=np.uint8)
    scales = np.empty((M, 2), dtype=np.float32)
    z = np.empty(M * block, dtype=np.float64) if want_z else None
    rc = lib().taco_ref_compress_ex(_ptr(x), n, block, float(np.float32(tau)), float(np.float32(eps)), mode, fmt,
                                    _ptr(payload), _ptr(scales), _ptr(z) if want_z else None)
    if rc != 0:
        raise ValueError(f"taco_ref_compress(n={n}, B={block}) -> {rc}")
    return (payload, scales, z) if want_z else (payload, scales)


def decompress_sum(payloads, scales, n: int, block: int = 128, want_sum: bool = False,
                   mode: int = MODE_FULL, fmt: int = FORMAT_E4M3):
    """payloads: list of k uint8[M*B]; scales: list of k float32[M,2].
    Returns bf16 bits (uint16[n]) of the sum of the k decoded tensors, and the unrounded
    float64 sum if want_sum."""
    k = len(payloads)
    assert k == len(scales) and k >= 1
    M = n_blocks(n, block)
    ps = [np.ascontiguousarray(p, dtype=np.uint8).reshape(-1) for p in payloads]
    ss = [np.ascontiguousarray(s, dtype=np.float32).reshape(-1) for s in scales]
    for p, s in zip(ps, ss):
        if p.size != M * block or s.size != 2 * M:
            raise ValueError("payload / scales size does not match n and block")
    parr = (ctypes.c_void_p * k)(*[p.ctypes.data for p in ps])
    sarr = (ctypes.c_void_p * k)(*[s.ctypes.data for s in ss])
    out = np.empty(n, dtype=np.uint16)
    acc = np.empty(n, dtype=np.float64) if want_sum else None
    rc = lib().taco_ref_decompress_sum_ex(parr, sarr, k, n, block, mode, fmt, _ptr(out),
                                          _ptr(acc) if want_sum else None)
    if rc != 0:
        raise ValueError(f"taco_ref_decompress_sum(k={k}, n={n}, B={block}) -> {rc}")
    return (out, acc) if want_sum else out


def decompress(payload, scales, n: int, block: int = 128, want_sum: bool = False,
               mode: int = MODE_FULL, fmt: int = FORMAT_E4M3):
    return decompress_sum([payload], [scales], n, block, want_sum, mode, fmt)
