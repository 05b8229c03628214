"""Thin ctypes binding of libzpp_gfx950.so (include/zpp.h).

Argument marshalling only: torch supplies device memory and the stream, every
step of the computation runs in the library's kernels.  There is no fallback: if
the shared library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

F16, BF16, F32 = 0, 1, 2
MAX_PEERS = 64

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "lib", "libzpp_gfx950.so")

# what include/zpp.h declares
EXPORTS = ("zpp_codes_bytes", "zpp_scales_count", "zpp_strerror", "zpp_reorder_source_slice",
           "zpp_reorder_mapped_slice", "qwz_quantize", "qwz_dequantize", "qgz_reorder",
           "qgz_intra_reduce", "qgz_inter_reduce")

_lib = None


class ZppError(RuntimeError):
    pass


def lib():
    """The loaded C-ABI library.  Raises if it has not been built (run
    `python -m paper_2306_10209_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ZppError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_10209_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.zpp_codes_bytes.argtypes, L.zpp_codes_bytes.restype = [sz, ci], sz
        L.zpp_scales_count.argtypes, L.zpp_scales_count.restype = [sz, ci], sz
        L.zpp_strerror.argtypes, L.zpp_strerror.restype = [ci], ctypes.c_char_p
        for f in (L.zpp_reorder_source_slice, L.zpp_reorder_mapped_slice):
            f.argtypes, f.restype = [ctypes.c_longlong, ci, ci, ci], ctypes.c_longlong
        L.qwz_quantize.argtypes = [vp, ci, sz, ci, ci, vp, vp, vp]
        L.qwz_dequantize.argtypes = [vp, vp, sz, ci, ci, ci, vp, vp]
        L.qgz_reorder.argtypes = [vp, ci, sz, ci, ci, ci, ci, ci, vp, vp, vp]
        L.qgz_intra_reduce.argtypes = [vp, vp, ci, sz, ci, ci, vp, vp, vp]
        L.qgz_inter_reduce.argtypes = [vp, vp, ci, sz, ci, ci, ctypes.c_float, vp, vp]
        for name in ("qwz_quantize", "qwz_dequantize", "qgz_reorder", "qgz_intra_reduce", "qgz_inter_reduce"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _check(rc, name):
    if rc != 0:
        raise ZppError(f"{name}: {lib().zpp_strerror(rc).decode()} (rc={rc})")


def dtype_code(t):
    try:
        return {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}[t]
    except KeyError:
        raise ZppError(f"unsupported dtype {t}") from None


def torch_dtype(code):
    return {F16: torch.float16, BF16: torch.bfloat16, F32: torch.float32}[code]


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t, name, nbytes=None, dtype=None):
    """Device pointer of a contiguous device tensor.  nbytes: the bytes the library will read or
    write there (the tensor must hold at least that many); dtype: the element type it must have."""
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise ZppError(f"{name}: needs a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ZppError(f"{name}: needs dtype {dtype}, got {t.dtype}")
    if nbytes is not None and t.numel() * t.element_size() < nbytes:
        raise ZppError(f"{name}: holds {t.numel() * t.element_size()} bytes, the call needs {nbytes}")
    return t.data_ptr()


def _sizes(n, block, bits):
    """(code bytes, scale count) of an n-element tensor; bad block / bits are left to the library's checks."""
    cb = n * bits // 8 if bits in (4, 8) else 0
    sc = n // block if block > 0 else 0
    return cb, sc


def codes_bytes(n, bits):
    return int(lib().zpp_codes_bytes(n, bits))


def scales_count(n, block):
    return int(lib().zpp_scales_count(n, block))


def reorder_source_slice(p, X, Y, S=1):
    return int(lib().zpp_reorder_source_slice(p, X, Y, S))


def reorder_mapped_slice(pid, X, Y, S=1):
    return int(lib().zpp_reorder_mapped_slice(pid, X, Y, S))


def qwz_quantize(x, block, bits=8, codes=None, scales=None, stream=None):
    """Block-quantize the flat tensor x.  `codes` (uint8) / `scales` (float32) may be
    views into a larger buffer (a shard's slot of the gather buffer)."""
    n = x.numel()
    cb, sc = _sizes(n, block, bits)
    if codes is None:
        codes = torch.empty(cb, dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(sc, dtype=torch.float32, device=x.device)
    _check(lib().qwz_quantize(_dev(x, "x"), dtype_code(x.dtype), n, block, bits, _dev(codes, "codes", cb, torch.uint8),
                              _dev(scales, "scales", 4 * sc, torch.float32), _stream(stream)), "qwz_quantize")
    return codes, scales


def qwz_dequantize(codes, scales, n, block, bits=8, out_dtype=torch.float16, out=None, stream=None):
    cb, sc = _sizes(n, block, bits)
    if out is None:
        out = torch.empty(n, dtype=out_dtype, device=codes.device)
    odt = dtype_code(out.dtype)
    _check(lib().qwz_dequantize(_dev(codes, "codes", cb, torch.uint8), _dev(scales, "scales", 4 * sc, torch.float32), n,
                                block, bits, odt, _dev(out, "out", n * out.element_size()), _stream(stream)),
           "qwz_dequantize")
    return out


def qgz_reorder(grad, X, Y, S, block, bits=4, codes=None, scales=None, stream=None):
    n = grad.numel()
    cb, sc = _sizes(n, block, bits)
    if codes is None:
        codes = torch.empty(cb, dtype=torch.uint8, device=grad.device)
    if scales is None:
        scales = torch.empty(sc, dtype=torch.float32, device=grad.device)
    _check(lib().qgz_reorder(_dev(grad, "grad"), dtype_code(grad.dtype), n, X, Y, S, block, bits,
                             _dev(codes, "codes", cb, torch.uint8), _dev(scales, "scales", 4 * sc, torch.float32),
                             _stream(stream)), "qgz_reorder")
    return codes, scales


def _table(tensors, name, dtype):
    if len(tensors) == 0:
        raise ZppError(f"{name}: empty pointer table")
    return (ctypes.c_void_p * len(tensors))(*[_dev(t, name, None, dtype) for t in tensors])


class PeerTable:
    """Host arrays of device pointers for the reduce stages, built once and reusable
    across launches (the library copies them into each launch).  Keeps the tensors
    alive."""

    def __init__(self, codes_in, scales_in):
        if len(codes_in) != len(scales_in):
            raise ZppError("codes_in and scales_in differ in length")
        self.count = len(codes_in)
        self.codes = _table(codes_in, "codes_in", torch.uint8)
        self.scales = _table(scales_in, "scales_in", torch.float32)
        self.device = codes_in[0].device
        self.min_code_bytes = min(t.numel() for t in codes_in)
        self.min_scales = min(t.numel() for t in scales_in)
        self._keep = (list(codes_in), list(scales_in))

    def check(self, m, block, bits, name):
        """Every peer's buffers must hold m elements' worth of codes and scales."""
        cb, sc = _sizes(m, block, bits)
        if self.min_code_bytes < cb or self.min_scales < sc:
            raise ZppError(f"{name}: a peer buffer is shorter than {m} elements need "
                           f"({cb} code bytes, {sc} scales)")


def _peers(codes_in, scales_in):
    if isinstance(codes_in, PeerTable):
        return codes_in
    return PeerTable(codes_in, scales_in)


def qgz_intra_reduce(codes_in, scales_in, m, block, bits=4, codes_out=None, scales_out=None, stream=None):
    """codes_in / scales_in: lists of device tensors, or a PeerTable as codes_in (scales_in ignored)."""
    t = _peers(codes_in, scales_in)
    t.check(m, block, bits, "qgz_intra_reduce")
    cb, sc = _sizes(m, block, bits)
    if codes_out is None:
        codes_out = torch.empty(cb, dtype=torch.uint8, device=t.device)
    if scales_out is None:
        scales_out = torch.empty(sc, dtype=torch.float32, device=t.device)
    _check(lib().qgz_intra_reduce(t.codes, t.scales, t.count, m, block, bits,
                                  _dev(codes_out, "codes_out", cb, torch.uint8),
                                  _dev(scales_out, "scales_out", 4 * sc, torch.float32), _stream(stream)),
           "qgz_intra_reduce")
    return codes_out, scales_out


def qgz_inter_reduce(codes_in, scales_in, m, block, bits=4, divisor=1.0, out=None, stream=None):
    """codes_in / scales_in: lists of device tensors, or a PeerTable as codes_in (scales_in ignored)."""
    t = _peers(codes_in, scales_in)
    t.check(m, block, bits, "qgz_inter_reduce")
    if out is None:
        out = torch.empty(m, dtype=torch.float32, device=t.device)
    _check(lib().qgz_inter_reduce(t.codes, t.scales, t.count, m, block, bits, float(divisor),
                                  _dev(out, "out", 4 * m, torch.float32), _stream(stream)), "qgz_inter_reduce")
    return out
