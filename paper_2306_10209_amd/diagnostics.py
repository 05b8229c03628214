"""ctypes binding of include/zpp_diagnostics.h: the library's self-checks and its plain copy
kernel.  Used by tests and benchmarks; nothing of the method goes through here."""
import ctypes

import torch

from . import binding as zpp

EXPORTS = ("zpp_selfcheck_block_scale", "zpp_selfcheck_divide", "zpp_stream_copy")

_ready = False


def _lib():
    global _ready
    L = zpp.lib()
    if not _ready:
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.zpp_selfcheck_block_scale.argtypes, L.zpp_selfcheck_block_scale.restype = [ci, ci, vp, vp], ci
        L.zpp_selfcheck_divide.argtypes, L.zpp_selfcheck_divide.restype = [ctypes.c_float, vp, vp], ci
        L.zpp_stream_copy.argtypes, L.zpp_stream_copy.restype = [vp, vp, sz, vp], ci
        _ready = True
    return L


def selfcheck_block_scale(bits, exponent, stream=None):
    """(mismatches of absmax/qmax, mismatches of qmax/absmax) over all 2^23 mantissas at one
    binary exponent; both must be 0."""
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    zpp._check(_lib().zpp_selfcheck_block_scale(bits, exponent, zpp._dev(counts, "counts"), zpp._stream(stream)),
               "zpp_selfcheck_block_scale")
    return tuple(int(v) for v in counts.cpu())


def selfcheck_divide(divisor, stream=None):
    """Mismatches between the short division by `divisor` and fp32 division over every dividend
    the inter-node stage hands to it; must be 0."""
    count = torch.zeros(1, dtype=torch.int64, device="cuda")
    zpp._check(_lib().zpp_selfcheck_divide(float(divisor), zpp._dev(count, "count"), zpp._stream(stream)),
               "zpp_selfcheck_divide")
    return int(count.cpu()[0])


def stream_copy(dst, src, stream=None):
    """Plain 16-byte-per-lane device copy (the bandwidth the kernels are compared with)."""
    nbytes = src.numel() * src.element_size()
    zpp._check(_lib().zpp_stream_copy(zpp._dev(dst, "dst", nbytes), zpp._dev(src, "src"), nbytes, zpp._stream(stream)),
               "zpp_stream_copy")
    return dst
