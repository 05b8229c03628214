"""Blocked versus non-blocked quantization error (the comparison of Sec. 3.1 of the
paper, whose own figures are for BERT weights that are not available here): RMS
reconstruction error of the library's block quantizer for several block sizes,
next to a single scale for the whole tensor, on the synthetic outlier-laden
weights of the benchmark.

    python -m paper_2306_10209_amd.error_study [--n ELEMENTS] [--bits 8]

The non-blocked baseline (one scale for the whole tensor) is not an option of the
library, whose blocks are at most 4096 elements, but it can be had from the library's
own quantizer: every block of 4096 is given 4064 elements of the tensor and 32 copies
of the tensor's largest-magnitude element, so every block's scale is the tensor-wide
one.  All quantization arithmetic therefore stays in the library's kernels (and is
checked against the CPU oracle like the rest); torch only moves elements.
"""
import argparse
import json

import torch

from . import binding as zpp
from . import workloads


def rms(t):
    return float(torch.sqrt(torch.mean(t.double() ** 2)))


def blocked_error(x, block, bits):
    n = x.numel()
    codes, scales = zpp.qwz_quantize(x, block, bits)
    y = zpp.qwz_dequantize(codes, scales, n, block, bits, out_dtype=torch.float32)
    return rms(y - x.float())


WHOLE_BLOCK, WHOLE_PAD = 4096, 32   # block used for the one-scale baseline, and how much of it is padding


def whole_tensor_layout(x):
    """x cut into rows of 4064 elements (a remainder is dropped), each followed by 32 copies of
    the largest-magnitude element of x: (padded flat tensor, the elements of x it holds)."""
    data = WHOLE_BLOCK - WHOLE_PAD
    rows = x.numel() // data
    kept = x.reshape(-1)[:rows * data]
    peak = kept[torch.argmax(kept.float().abs())]
    padded = torch.empty(rows, WHOLE_BLOCK, dtype=x.dtype, device=x.device)
    padded[:, :data] = kept.view(rows, data)
    padded[:, data:] = peak
    return padded.reshape(-1), kept


def unblocked_error(x, bits):
    """RMS error with one scale for the whole tensor, through the library's block quantizer."""
    padded, kept = whole_tensor_layout(x)
    n = padded.numel()
    codes, scales = zpp.qwz_quantize(padded, WHOLE_BLOCK, bits)
    y = zpp.qwz_dequantize(codes, scales, n, WHOLE_BLOCK, bits, out_dtype=torch.float32)
    y = y.view(-1, WHOLE_BLOCK)[:, :WHOLE_BLOCK - WHOLE_PAD].reshape(-1)
    return rms(y - kept.float())


def study(x, blocks=(32, 64, 128, 256, 512, 1024, 2048, 4096), bits=8):
    base = unblocked_error(x, bits)
    rows = {"unblocked_rms": base, "signal_rms": rms(x.float()), "bits": bits, "blocks": {}}
    for b in blocks:
        if x.numel() % b:
            continue
        e = blocked_error(x, b, bits)
        rows["blocks"][b] = {"rms": e, "unblocked_over_blocked": base / e if e > 0 else float("inf")}
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1 << 26)
    ap.add_argument("--bits", type=int, default=8)
    args = ap.parse_args()
    x = workloads.weights(args.n, device="cuda:0")
    print(json.dumps(study(x, bits=args.bits), indent=1))


if __name__ == "__main__":
    main()
