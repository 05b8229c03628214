"""Second evaluator of the block codec, by a different route than the C oracle.

Every fp32 operation of the definition is carried out in float64 and rounded
once to float32.  For +, *, / on binary32 operands that is the correctly rounded
binary32 result (53 >= 2*24+2 bits, so the double rounding is innocuous), i.e.
what IEEE-754 fixes for each step, without using fp32 machine arithmetic at all.
`round_fraction_to_f32` goes further for scalars: exact rational arithmetic and a
hand-written round-to-nearest-even.
"""
from fractions import Fraction

import numpy as np


def qmax_of(bits):
    return (1 << (bits - 1)) - 1


def f16_bits_to_f64(bits16):
    return np.asarray(bits16, dtype=np.uint16).view(np.float16).astype(np.float64)


def bf16_bits_to_f64(bits16):
    import torch
    t = torch.from_numpy(np.asarray(bits16, dtype=np.uint16).view(np.int16).copy())
    return t.view(torch.bfloat16).to(torch.float64).numpy()


def widen64(x, dtype):
    if dtype == 0:
        return f16_bits_to_f64(x)
    if dtype == 1:
        return bf16_bits_to_f64(x)
    return np.asarray(x, dtype=np.float32).astype(np.float64)


def rn32(v64):
    """Round float64 value(s) to the nearest float32, returned as float64."""
    return np.asarray(v64, dtype=np.float64).astype(np.float32).astype(np.float64)


def quant_blocks(v64, block, bits):
    """v64: float64 array of values exactly representable in fp32, length multiple
    of block.  Returns (int codes, float32 scales)."""
    qmax = float(qmax_of(bits))
    v = np.asarray(v64, dtype=np.float64).reshape(-1, block)
    a = np.max(np.abs(v), axis=1)
    tiny = a < 2.0 ** -100
    a_safe = np.where(tiny, 1.0, a)
    scale = rn32(a_safe / qmax)
    inv = rn32(qmax / a_safe)
    t = rn32(v * inv[:, None])
    q = np.clip(np.rint(t), -qmax, qmax)  # np.rint: half to even
    q = np.where(tiny[:, None], 0.0, q)
    scale = np.where(tiny, 0.0, scale)
    return q.astype(np.int32).reshape(-1), scale.astype(np.float32)


def dequant(q, scales, block):
    """fp32 decode: float(q) * scale, rounded once to fp32; returned as float64."""
    q = np.asarray(q, dtype=np.float64).reshape(-1, block)
    s = np.asarray(scales, dtype=np.float32).astype(np.float64)
    return rn32(q * s[:, None]).reshape(-1)


def fold_sum(terms64):
    """Sequential fp32 sum in the order given (list of arrays), start at +0."""
    s = np.zeros_like(terms64[0], dtype=np.float64)
    for t in terms64:
        s = rn32(s + t)
    return s


def round_fraction_to_f32(fr):
    """Exact rational -> nearest binary32 (ties to even), normal range only.
    Returned as a Python float holding that binary32 value."""
    if fr == 0:
        return 0.0
    sign = -1 if fr < 0 else 1
    fr = abs(fr)
    e = 0
    # scale into [2^23, 2^24)
    while fr >= (1 << 24):
        fr /= 2
        e += 1
    while fr < (1 << 23):
        fr *= 2
        e -= 1
    assert -149 <= e + 23 - 23 and e > -126 - 23 + 0, "subnormal range not handled"
    m = fr.numerator // fr.denominator
    rem = fr - m
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (m & 1)):
        m += 1
    return sign * float(m) * 2.0 ** e


def unpack_nibbles(codes_u8, n):
    """Independent decode of the int4 storage convention: byte i holds element 2i
    in bits 0-3 and element 2i+1 in bits 4-7, two's complement."""
    out = []
    for i in range(n):
        b = int(codes_u8[i // 2])
        nib = (b >> 4) if (i % 2) else (b & 15)
        out.append(nib - 16 if nib & 8 else nib)
    return np.array(out, dtype=np.int32)
