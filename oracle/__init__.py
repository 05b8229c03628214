"""ctypes front-end of the CPU oracle (oracle/zpp_oracle.c).

Test infrastructure only.  Takes and returns numpy arrays on the host; 16-bit
floating inputs and outputs travel as uint16 bit patterns so that nothing here
depends on how numpy (or torch) would round them.  This module imports nothing
from the GPU package and the GPU package imports nothing from here.
"""
import ctypes
import os

import numpy as np

from . import build as _build

F16, BF16, F32 = 0, 1, 2
_lib = None


def _load(path):
    """Load an oracle shared library and declare its signatures."""
    L = ctypes.CDLL(path)
    vp, fp, sz, ci = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    L.oracle_qwz_quantize.argtypes = [vp, ci, sz, ci, ci, vp, fp]
    L.oracle_qwz_dequantize.argtypes = [vp, fp, sz, ci, ci, ci, vp]
    L.oracle_qgz_reorder.argtypes = [vp, ci, sz, ci, ci, ci, ci, ci, vp, fp]
    L.oracle_qgz_intra_reduce.argtypes = [vp, vp, ci, sz, ci, ci, vp, fp]
    L.oracle_qgz_inter_reduce.argtypes = [vp, vp, ci, sz, ci, ci, ctypes.c_float, fp]
    for f in (L.oracle_qwz_quantize, L.oracle_qwz_dequantize, L.oracle_qgz_reorder,
              L.oracle_qgz_intra_reduce, L.oracle_qgz_inter_reduce):
        f.restype = ci
    L.oracle_reorder_source_slice.argtypes = [ctypes.c_longlong, ci, ci, ci]
    L.oracle_reorder_source_slice.restype = ctypes.c_longlong
    L.oracle_reorder_mapped_slice.argtypes = [ctypes.c_longlong, ci, ci, ci]
    L.oracle_reorder_mapped_slice.restype = ctypes.c_longlong
    L.oracle_widen.argtypes = [ctypes.c_uint16, ci]
    L.oracle_widen.restype = ctypes.c_float
    L.oracle_narrow.argtypes = [ctypes.c_float, ci]
    L.oracle_narrow.restype = ctypes.c_uint16
    L.oracle_set_threads.argtypes = [ci]
    L.oracle_set_threads.restype = ci
    return L


def lib():
    """Load liboracle.so, compiling it first if it is missing or stale."""
    global _lib
    if _lib is None:
        # ZPP_ORACLE_LIB: a test may point at a deliberately broken build to show the pins catch it
        _lib = _load(os.environ.get("ZPP_ORACLE_LIB") or _build.build(force=False))
    return _lib


class OracleError(ValueError):
    pass


def _check(rc, name):
    if rc != 0:
        raise OracleError(f"{name}: invalid argument (rc={rc})")


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _as_input(x, dtype):
    """Host array in the storage type of `dtype` (uint16 bit patterns or float32)."""
    want = np.float32 if dtype == F32 else np.uint16
    x = np.ascontiguousarray(x)
    if x.dtype == np.float16 and dtype == F16:
        x = x.view(np.uint16)
    if x.dtype != want:
        raise TypeError(f"dtype code {dtype} needs a {want.__name__} array, got {x.dtype}")
    return x.reshape(-1)


def codes_nbytes(n, bits):
    return n * bits // 8


def _out(given, size, dtype, name):
    """A caller's output array (exact size and type, contiguous) or a new zeroed one."""
    if given is None:
        return np.zeros(size, dtype=dtype)
    if not (isinstance(given, np.ndarray) and given.dtype == dtype and given.size == size and given.flags.c_contiguous):
        raise TypeError(f"{name}: needs a contiguous {np.dtype(dtype).name} array of {size} elements")
    return given


def set_threads(t):
    """Set the OpenMP thread count (t < 1: leave); returns the count in effect."""
    return lib().oracle_set_threads(int(t))


def qwz_quantize(x, dtype, block, bits=8, codes=None, scales=None):
    """codes / scales / out arguments of this module: optional arrays to write the result into."""
    x = _as_input(x, dtype)
    n = x.size
    codes = _out(codes, codes_nbytes(n, bits), np.uint8, "codes")
    scales = _out(scales, max(n // max(block, 1), 0), np.float32, "scales")
    _check(lib().oracle_qwz_quantize(_ptr(x), dtype, n, block, bits, _ptr(codes), _ptr(scales)),
           "qwz_quantize")
    return codes, scales


def qwz_dequantize(codes, scales, n, block, bits=8, out_dtype=F16, out=None):
    codes = np.ascontiguousarray(codes).view(np.uint8).reshape(-1)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    y = _out(out, n, np.float32 if out_dtype == F32 else np.uint16, "out")
    _check(lib().oracle_qwz_dequantize(_ptr(codes), _ptr(scales), n, block, bits, out_dtype, _ptr(y)),
           "qwz_dequantize")
    return y


def qgz_reorder(grad, dtype, X, Y, S, block, bits=4, codes=None, scales=None):
    grad = _as_input(grad, dtype)
    n = grad.size
    codes = _out(codes, codes_nbytes(n, bits), np.uint8, "codes")
    scales = _out(scales, n // max(block, 1), np.float32, "scales")
    _check(lib().oracle_qgz_reorder(_ptr(grad), dtype, n, X, Y, S, block, bits, _ptr(codes), _ptr(scales)),
           "qgz_reorder")
    return codes, scales


def _ptr_array(arrs):
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def qgz_intra_reduce(codes_in, scales_in, m, block, bits=4, codes=None, scales=None):
    codes_in = [np.ascontiguousarray(c).view(np.uint8).reshape(-1) for c in codes_in]
    scales_in = [np.ascontiguousarray(s, dtype=np.float32) for s in scales_in]
    X = len(codes_in)
    codes = _out(codes, codes_nbytes(m, bits), np.uint8, "codes")
    scales = _out(scales, m // max(block, 1), np.float32, "scales")
    _check(lib().oracle_qgz_intra_reduce(_ptr_array(codes_in), _ptr_array(scales_in), X, m, block, bits,
                                         _ptr(codes), _ptr(scales)), "qgz_intra_reduce")
    return codes, scales


def qgz_inter_reduce(codes_in, scales_in, m, block, bits=4, divisor=1.0, out=None):
    codes_in = [np.ascontiguousarray(c).view(np.uint8).reshape(-1) for c in codes_in]
    scales_in = [np.ascontiguousarray(s, dtype=np.float32) for s in scales_in]
    Y = len(codes_in)
    out = _out(out, m, np.float32, "out")
    _check(lib().oracle_qgz_inter_reduce(_ptr_array(codes_in), _ptr_array(scales_in), Y, m, block, bits,
                                         float(divisor), _ptr(out)), "qgz_inter_reduce")
    return out


def reorder_source_slice(p, X, Y, S=1):
    return int(lib().oracle_reorder_source_slice(p, X, Y, S))


def reorder_mapped_slice(pid, X, Y, S=1):
    return int(lib().oracle_reorder_mapped_slice(pid, X, Y, S))


def widen(bits16, dtype):
    """uint16 bit patterns -> float32 values (element by element through the C routine)."""
    L = lib()
    b = np.asarray(bits16, dtype=np.uint16).reshape(-1)
    return np.array([L.oracle_widen(int(v), dtype) for v in b], dtype=np.float32)


def narrow(vals, dtype):
    """float32 values -> uint16 bit patterns (element by element through the C routine)."""
    L = lib()
    v = np.asarray(vals, dtype=np.float32).reshape(-1)
    return np.array([L.oracle_narrow(float(x), dtype) for x in v], dtype=np.uint16)


def unpack_codes(codes, n, bits):
    """Signed integer codes as int32 (storage convention: see zpp_oracle.c header)."""
    c = np.ascontiguousarray(codes).view(np.uint8).reshape(-1)
    if bits == 8:
        return c.view(np.int8)[:n].astype(np.int32)
    if bits == 32:
        return c.view(np.float32)[:n]
    lo = (c & 0xF).astype(np.int32)
    hi = (c >> 4).astype(np.int32)
    q = np.empty(2 * c.size, dtype=np.int32)
    q[0::2], q[1::2] = lo, hi
    q = np.where(q >= 8, q - 16, q)
    return q[:n]
