"""Blocked versus non-blocked quantization error (the comparison of Sec. 3.1 of the
paper, whose own figures are for BERT weights that are not available here): RMS
reconstruction error of the library's block quantizer for several block sizes,
next to a single scale for the whole tensor, on the synthetic outlier-laden
weights of the benchmark.

    python -m paper_2306_10209_amd.error_study [--n ELEMENTS] [--bits 8]

The non-blocked baseline is not something the library offers (blocks are at most
4096 elements); it is emulated here with elementwise torch operations using the
same scale / round-half-even rule.
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


def unblocked_error(x, bits):
    qmax = float((1 << (bits - 1)) - 1)
    xf = x.float()
    a = xf.abs().max()
    scale, inv = a / qmax, qmax / a
    return rms(torch.round(xf * inv) * scale - xf)


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
