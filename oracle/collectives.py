"""Python face of the C oracle (flex_oracle.c): argument marshalling only.

Test infrastructure, not the product: imported only by tests, by the smoke
check and by the benchmark's CPU-baseline leg.  Inputs are numpy arrays;
bfloat16 data travels as its raw 16-bit patterns (dtype uint16).
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build.build())
        pp = ctypes.POINTER(ctypes.c_void_p)
        L.oracle_allreduce_f32.argtypes = [pp, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        L.oracle_allreduce_f32.restype = None
        L.oracle_allreduce_bf16.argtypes = [pp, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        L.oracle_allreduce_bf16.restype = None
        L.oracle_allreduce_f16.argtypes = [pp, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        L.oracle_allreduce_f16.restype = None
        L.oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_f16_to_f32.restype = ctypes.c_float
        L.oracle_f32_bits_to_f16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.oracle_f32_bits_to_f16.restype = None
        L.oracle_allgather.argtypes = [pp, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        L.oracle_allgather.restype = None
        L.oracle_alltoall.argtypes = [pp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        L.oracle_alltoall.restype = None
        L.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_bf16_to_f32.restype = ctypes.c_float
        L.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        L.oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.oracle_f32_bits_to_bf16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.oracle_f32_bits_to_bf16.restype = None
        L.oracle_get_threads.restype = ctypes.c_int
        L.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def _ptr_array(arrays):
    arr = (ctypes.c_void_p * len(arrays))()
    for i, a in enumerate(arrays):
        arr[i] = a.ctypes.data
    return arr


def _check_inputs(bufs):
    if len(bufs) < 1:
        raise ValueError("need at least one rank")
    first = bufs[0]
    for b in bufs:
        if not isinstance(b, np.ndarray) or b.ndim != 1 or not b.flags.c_contiguous:
            raise ValueError("rank buffers must be contiguous 1-D numpy arrays")
        if b.dtype != first.dtype or b.shape != first.shape:
            raise ValueError("rank buffers must agree in dtype and length")


def allreduce(bufs):
    """Rank-ordered sum of the rank buffers.

    bufs: list of N 1-D arrays, all float32, all float16, or all uint16 holding
    bfloat16 bit patterns.  Returns a new array of the same dtype and length.
    """
    _check_inputs(bufs)
    out = np.empty_like(bufs[0])
    ptrs = _ptr_array(bufs)
    if bufs[0].dtype == np.float32:
        lib().oracle_allreduce_f32(ptrs, len(bufs), bufs[0].size, out.ctypes.data)
    elif bufs[0].dtype == np.uint16:
        lib().oracle_allreduce_bf16(ptrs, len(bufs), bufs[0].size, out.ctypes.data)
    elif bufs[0].dtype == np.float16:
        lib().oracle_allreduce_f16(ptrs, len(bufs), bufs[0].size, out.ctypes.data)
    else:
        raise ValueError("dtype must be float32, float16 or uint16 (bfloat16 bits)")
    return out


def reducescatter(bufs, rank):
    """Rank `rank`'s slice of the rank-ordered sum: every buffer holds N slices
    of equal length; the result is the sum over ranks of slice number `rank`."""
    _check_inputs(bufs)
    n = len(bufs)
    if bufs[0].size % n:
        raise ValueError("buffer length must be a multiple of the number of ranks")
    rc = bufs[0].size // n
    return allreduce([np.ascontiguousarray(b[rank * rc:(rank + 1) * rc]) for b in bufs])


def allgather(slices):
    """Concatenation of the rank slices in rank order, byte for byte."""
    _check_inputs(slices)
    n = len(slices)
    out = np.empty(n * slices[0].size, dtype=slices[0].dtype)
    lib().oracle_allgather(_ptr_array(slices), n, slices[0].nbytes, out.ctypes.data)
    return out


def alltoall(bufs, rank):
    """Receive buffer of rank `rank`: piece r is piece number `rank` of rank r's
    buffer (every buffer holds N pieces of equal length)."""
    _check_inputs(bufs)
    n = len(bufs)
    if bufs[0].size % n:
        raise ValueError("buffer length must be a multiple of the number of ranks")
    out = np.empty_like(bufs[0])
    lib().oracle_alltoall(_ptr_array(bufs), n, rank, bufs[0].nbytes // n, out.ctypes.data)
    return out


def bf16_to_f32(h: int) -> float:
    return float(lib().oracle_bf16_to_f32(int(h)))


def f32_to_bf16(f) -> int:
    return int(lib().oracle_f32_to_bf16(ctypes.c_float(f)))


def f32_bits_to_bf16(bits):
    """Round an array of binary32 bit patterns (uint32) to bfloat16 bits."""
    bits = np.ascontiguousarray(bits, dtype=np.uint32)
    out = np.empty(bits.shape, dtype=np.uint16)
    lib().oracle_f32_bits_to_bf16(bits.ctypes.data, bits.size, out.ctypes.data)
    return out


def f16_to_f32(h: int) -> float:
    return float(lib().oracle_f16_to_f32(int(h)))


def f32_bits_to_f16(bits):
    """Round an array of binary32 bit patterns (uint32) to binary16 bits."""
    bits = np.ascontiguousarray(bits, dtype=np.uint32)
    out = np.empty(bits.shape, dtype=np.uint16)
    lib().oracle_f32_bits_to_f16(bits.ctypes.data, bits.size, out.ctypes.data)
    return out


def get_threads() -> int:
    return int(lib().oracle_get_threads())


def set_threads(n: int) -> None:
    lib().oracle_set_threads(int(n))
