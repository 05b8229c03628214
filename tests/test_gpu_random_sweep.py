"""Seeded random sweep over the valid argument space of the five operations: dtypes, code
widths, block sizes (powers of two and not), X, Y, S, divisors and value ranges that no
hand-picked case combines.  Every output byte is compared with the oracle."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2306_10209_amd import binding as zpp
from paper_2306_10209_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TORCH_DT = {oracle.F16: torch.float16, oracle.BF16: torch.bfloat16, oracle.F32: torch.float32}
BLOCKS = [32, 64, 96, 128, 160, 256, 384, 512, 736, 1024, 1536, 2048, 3072, 4096]


def eq(dev_tensor, host_array):
    got = dev_tensor.detach().cpu().contiguous()
    if got.dtype in (torch.float16, torch.bfloat16):
        got = got.view(torch.int16)
    got = got.numpy().view(np.uint8).reshape(-1)
    want = np.ascontiguousarray(host_array).view(np.uint8).reshape(-1)
    return got.size == want.size and np.array_equal(got, want)


def draw_values(rng, n, block, dtype):
    """host tensor of n values in `dtype`: per-block magnitudes over many decades, some blocks all
    zero, some holding one extreme value, some below the zero-scale threshold (bf16 / fp32 only).
    Magnitudes stop short of where a sum over nine peers could overflow fp32: the interface
    leaves non-finite values unspecified."""
    nb = n // block
    top = {oracle.F16: 4.0, oracle.BF16: 35.0, oracle.F32: 35.0}[dtype]
    low = {oracle.F16: -7.0, oracle.BF16: -30.0, oracle.F32: -36.0}[dtype]
    mag = 10.0 ** rng.uniform(low, top, size=nb)
    v = rng.standard_normal((nb, block)) * mag[:, None]
    kind = rng.integers(0, 12, size=nb)
    v[kind == 0] = 0.0
    t = torch.from_numpy(v.reshape(-1)).to(torch.float32)
    finfo = torch.finfo(TORCH_DT[dtype])
    t = t.clamp(-finfo.max / 16, finfo.max / 16).to(TORCH_DT[dtype])
    extreme = finfo.max if dtype == oracle.F16 else finfo.max / 16
    for b in np.flatnonzero(kind == 1):                   # one extreme element in the block
        t[b * block + int(rng.integers(0, block))] = extreme if rng.integers(0, 2) else -extreme
    return t


# ZPP_SWEEP_SEEDS widens the sweep for an occasional long run
@pytest.mark.parametrize("seed", range(int(os.environ.get("ZPP_SWEEP_SEEDS", "160"))))
def test_random_configuration(seed):
    rng = np.random.default_rng(9000 + seed)
    dtype = [oracle.F16, oracle.BF16, oracle.F32][int(rng.integers(0, 3))]
    bits = int(rng.choice([4, 8]))
    block = int(rng.choice(BLOCKS))
    X, Y, S = int(rng.integers(1, 10)), int(rng.integers(1, 10)), int(rng.integers(1, 4))
    bps = int(rng.integers(1, 5))
    if seed % 16 == 0:                                   # every 16th draw is large: grids beyond the XCD-remap threshold
        bps *= max(1, (24 << 20) // (S * X * Y * block * bps))
    L = block * bps                                      # elements per slice
    n = S * X * Y * L
    print(f"seed={seed} dtype={dtype} bits={bits} block={block} X={X} Y={Y} S={S} bps={bps} n={n}", flush=True)

    # qwz: quantize, decode to the input's type and to fp32
    x = draw_values(rng, n, block, dtype)
    hc, hs = oracle.qwz_quantize(workloads.as_bits(x), dtype, block, bits)
    dc, ds = zpp.qwz_quantize(x.to(DEV), block, bits)
    torch.cuda.synchronize()
    assert eq(ds, hs), "qwz_quantize scales"
    assert eq(dc, hc), "qwz_quantize codes"
    for odt in {dtype, oracle.F32, oracle.BF16}:
        y = torch.empty(n, dtype=TORCH_DT[odt], device=DEV)
        zpp.qwz_dequantize(dc, ds, n, block, bits, out=y)
        torch.cuda.synchronize()
        assert eq(y, oracle.qwz_dequantize(hc, hs, n, block, bits, odt)), f"qwz_dequantize to {odt}"

    # qgz: K "GPUs" reorder their own gradient
    K = max(X, Y)
    grads = [draw_values(rng, n, block, dtype) for _ in range(K)]
    host = [oracle.qgz_reorder(workloads.as_bits(g), dtype, X, Y, S, block, bits) for g in grads]
    dev = [zpp.qgz_reorder(g.to(DEV), X, Y, S, block, bits) for g in grads]
    torch.cuda.synchronize()
    for k in range(K):
        assert eq(dev[k][1], host[k][1]), f"qgz_reorder scales of GPU {k}"
        assert eq(dev[k][0], host[k][0]), f"qgz_reorder codes of GPU {k}"

    # first hop of a random (stage, local rank): group j of stage s from X of those buffers
    s, j = int(rng.integers(0, S)), int(rng.integers(0, X))
    m_s = n // (S * X)
    lo = s * (n // S) + j * m_s
    cs = slice(lo * bits // 8, (lo + m_s) * bits // 8)
    ss = slice(lo // block, (lo + m_s) // block)
    hic, his = oracle.qgz_intra_reduce([host[k][0][cs] for k in range(X)], [host[k][1][ss] for k in range(X)],
                                       m_s, block, bits)
    dic, dis = zpp.qgz_intra_reduce([dev[k][0][cs] for k in range(X)], [dev[k][1][ss] for k in range(X)],
                                    m_s, block, bits)
    torch.cuda.synchronize()
    assert eq(dis, his), "qgz_intra_reduce scales"
    assert eq(dic, hic), "qgz_intra_reduce codes"

    # second hop: slice i of Y buffers (any valid codes serve), a random divisor
    i = int(rng.integers(0, S * X * Y))
    cs = slice(i * L * bits // 8, (i + 1) * L * bits // 8)
    ss = slice(i * bps, (i + 1) * bps)
    divisor = float(rng.choice([1.0, 2.0, 3.0, float(X * Y), 384.0, 1000.0, 0.5, 7.25]))
    hout = oracle.qgz_inter_reduce([host[k][0][cs] for k in range(Y)], [host[k][1][ss] for k in range(Y)],
                                   L, block, bits, divisor)
    dout = zpp.qgz_inter_reduce([dev[k][0][cs] for k in range(Y)], [dev[k][1][ss] for k in range(Y)],
                                L, block, bits, divisor)
    torch.cuda.synchronize()
    assert eq(dout, hout), f"qgz_inter_reduce with divisor {divisor}"
