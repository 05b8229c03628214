"""GPU parity at the full benchmark sizes against the CPU oracle on EVERY element.

With all host cores the oracle streams a few GB/s, so whole tensors of the
benchmark configurations are within reach (a couple of seconds per call).  Each
case hands the raw seeded inputs to the oracle (nothing the library wrote ever
enters it), compares all output bytes, and prints a 64-bit position-weighted
checksum of every output computed twice: on the device from the library's output
and on the host from the oracle's (run pytest with -s or -rA to see them).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_10209_amd import binding as zpp
from paper_2306_10209_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MASK = (1 << 64) - 1


def host_checksum(a):
    """sum_i word_i * (2i + 1) mod 2^64 over the little-endian 64-bit words of the bytes of a"""
    b = np.ascontiguousarray(a).view(np.uint8).reshape(-1)
    if b.size % 8:
        b = np.concatenate([b, np.zeros(-b.size % 8, dtype=np.uint8)])
    w = b.view(np.uint64)
    total, step = 0, 1 << 24
    for lo in range(0, w.size, step):
        idx = np.arange(lo, min(lo + step, w.size), dtype=np.uint64)
        with np.errstate(over="ignore"):
            total += int((w[lo:lo + step] * (idx * np.uint64(2) + np.uint64(1))).sum(dtype=np.uint64))
    return total & MASK


def device_checksum(t):
    """the same sum with wrapping int64 arithmetic on the device"""
    b = t.detach().contiguous().view(torch.uint8).reshape(-1)
    if b.numel() % 8:
        b = torch.cat([b, torch.zeros(-b.numel() % 8, dtype=torch.uint8, device=b.device)])
    w = b.view(torch.int64)
    total, step = 0, 1 << 27
    for lo in range(0, w.numel(), step):
        hi = min(lo + step, w.numel())
        idx = torch.arange(lo, hi, dtype=torch.int64, device=t.device)
        total += int((w[lo:hi] * (idx * 2 + 1)).sum().item())
    return total & MASK


def same(name, dev_tensor, host_array):
    """all bytes equal, and the two checksums (printed) equal"""
    got = dev_tensor.detach().contiguous().view(torch.uint8).reshape(-1).cpu().numpy()
    want = np.ascontiguousarray(host_array).view(np.uint8).reshape(-1)
    assert got.size == want.size, name
    equal = np.array_equal(got, want)
    cd, ch = device_checksum(dev_tensor), host_checksum(host_array)
    print(f"checksum {name}: library 0x{cd:016x} oracle 0x{ch:016x} {'identical' if equal else 'DIFFERENT'}",
          flush=True)
    assert equal, f"{name}: first difference at byte {int(np.flatnonzero(got != want)[0])}"
    assert cd == ch, name


def test_checksums_agree_and_see_a_swap():
    x = torch.arange(4096, dtype=torch.int32, device=DEV) * 2654435761
    h = x.cpu().numpy()
    assert device_checksum(x) == host_checksum(h)
    h2 = h.copy()
    h2[[10, 11, 12, 13]] = h2[[12, 13, 10, 11]]          # two 64-bit words swapped
    assert host_checksum(h2) != host_checksum(h)


def test_weights_hidden_8192_layer_every_element():
    """bf16 weights of one hidden-8192 layer, 8 flat shards per matrix, int8 blocks of 2048"""
    P, B, bits = 8, 2048, 8
    shapes = workloads.gpt_layer_shapes(8192)
    n_total = sum(r * c for _, r, c in shapes)
    codes = torch.empty(n_total, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n_total // B, dtype=torch.float32, device=DEV)
    out = torch.empty(n_total, dtype=torch.bfloat16, device=DEV)
    host_w, off = [], 0
    for tid, (_, r, c) in enumerate(shapes):
        n = r * c
        w = workloads.weights(n, device=DEV, tensor_id=10 + tid)
        host_w.append(workloads.as_bits(w))
        sh = n // P
        for rank in range(P):
            lo = off + rank * sh
            zpp.qwz_quantize(w[rank * sh:(rank + 1) * sh], B, bits, codes=codes[lo:lo + sh],
                             scales=scales[lo // B:(lo + sh) // B])
        off += n
        del w
    zpp.qwz_dequantize(codes, scales, n_total, B, bits, out=out)
    torch.cuda.synchronize()
    oc, os_ = oracle.qwz_quantize(np.concatenate(host_w), oracle.BF16, B, bits)
    same("hidden-8192 layer int8 codes", codes, oc)
    same("hidden-8192 layer scales", scales, os_)
    same("hidden-8192 layer dequantized bf16", out, oracle.qwz_dequantize(oc, os_, n_total, B, bits, oracle.BF16))


def test_batched_small_tensors_fp16_block_256_every_element():
    """1024 tensors of 4096 x 256 fp16 in one launch, int8 blocks of 256"""
    B, bits = 256, 8
    n = 1024 << 20
    x = workloads.weights(n, device=DEV, tensor_id=30, dtype=torch.float16, outlier_prob=0.0)
    codes, scales = zpp.qwz_quantize(x, B, bits)
    y = zpp.qwz_dequantize(codes, scales, n, B, bits, out_dtype=torch.float16)
    torch.cuda.synchronize()
    oc, os_ = oracle.qwz_quantize(workloads.as_bits(x), oracle.F16, B, bits)
    same("1024 small tensors int8 codes", codes, oc)
    same("1024 small tensors scales", scales, os_)
    same("1024 small tensors dequantized fp16", y, oracle.qwz_dequantize(oc, os_, n, B, bits, oracle.F16))


def test_intra_stage_8_ranks_2p28_every_element():
    """8 ranks x 2^28 fp16 heavy-tailed gradients, X = 8, Y = 64, int4 blocks of 512"""
    X, Y, B, bits = 8, 64, 512, 4
    n = 1 << 28
    m = n // X
    first_dev, first_host = [], []
    for r in range(X):
        g = workloads.gradients(n, device=DEV, tensor_id=40 + r)
        first_dev.append(zpp.qgz_reorder(g, X, Y, 1, B, bits))
        first_host.append(oracle.qgz_reorder(workloads.as_bits(g), oracle.F16, X, Y, 1, B, bits))
        del g
    torch.cuda.synchronize()
    for r in range(X):
        same(f"rank {r} reordered int4 codes", first_dev[r][0], first_host[r][0])
        same(f"rank {r} reordered scales", first_dev[r][1], first_host[r][1])
    cb, sb = m // 2, m // B
    for j in range(X):
        codes, scales = zpp.qgz_intra_reduce([first_dev[k][0][j * cb:(j + 1) * cb] for k in range(X)],
                                             [first_dev[k][1][j * sb:(j + 1) * sb] for k in range(X)], m, B, bits)
        oc, os_ = oracle.qgz_intra_reduce([first_host[k][0][j * cb:(j + 1) * cb] for k in range(X)],
                                          [first_host[k][1][j * sb:(j + 1) * sb] for k in range(X)], m, B, bits)
        torch.cuda.synchronize()
        same(f"local rank {j} first-hop codes", codes, oc)
        same(f"local rank {j} first-hop scales", scales, os_)


def test_inter_stage_48_nodes_every_element():
    """48 chunks of 46,875,136 fp16 gradients (an 18B-parameter model's share on 384 GPUs)"""
    Y, B, bits, W = 48, 512, 4, 384.0
    L = 46875136
    enc_dev, enc_host = [], []
    for i in range(Y):
        g = workloads.gradients(L, device=DEV, tensor_id=60 + i, tail_std=0.0)
        enc_dev.append(zpp.qwz_quantize(g, B, bits))
        enc_host.append(oracle.qwz_quantize(workloads.as_bits(g), oracle.F16, B, bits))
        del g
    out = zpp.qgz_inter_reduce([c for c, _ in enc_dev], [s for _, s in enc_dev], L, B, bits, W)
    torch.cuda.synchronize()
    oo = oracle.qgz_inter_reduce([c for c, _ in enc_host], [s for _, s in enc_host], L, B, bits, W)
    same("48-node second-hop fp32 partition", out, oo)


def test_benchmark_layer_hidden_12288_every_element():
    """one layer of the benchmark step: the six calls on 1,811,939,328 elements, X = 8, Y = 48"""
    X, Y, W = 8, 48, 384
    WB, GB = 2048, 512
    n_L = workloads.layer_numel(12288)
    m, L = n_L // X, n_L // W

    w = workloads.weights(n_L, device=DEV, tensor_id=1)
    wc, ws = zpp.qwz_quantize(w, WB, 8)
    y = torch.empty(n_L, dtype=torch.bfloat16, device=DEV)
    zpp.qwz_dequantize(wc, ws, n_L, WB, 8, out=y)
    torch.cuda.synchronize()
    oc, os_ = oracle.qwz_quantize(workloads.as_bits(w), oracle.BF16, WB, 8)
    del w
    same("layer weights int8 codes", wc, oc)
    same("layer weights scales", ws, os_)
    same("layer weights dequantized bf16", y, oracle.qwz_dequantize(oc, os_, n_L, WB, 8, oracle.BF16))
    del wc, ws, y, oc, os_

    grad = workloads.gradients(n_L, device=DEV, tensor_id=3, tail_std=0.0)
    gc, gs = zpp.qgz_reorder(grad, X, Y, 1, GB, 4)
    hgc, hgs = oracle.qgz_reorder(workloads.as_bits(grad), oracle.F16, X, Y, 1, GB, 4)
    del grad
    same("layer gradient reordered int4 codes", gc, hgc)
    same("layer gradient reordered scales", gs, hgs)

    peers_dev, peers_host = [], []
    for k in range(X - 1):                                   # what the 7 other local GPUs sent
        g = workloads.gradients(m, device=DEV, tensor_id=100 + k, tail_std=0.0)
        peers_dev.append(zpp.qwz_quantize(g, GB, 4))
        peers_host.append(oracle.qwz_quantize(workloads.as_bits(g), oracle.F16, GB, 4))
        del g
    ic, isc = zpp.qgz_intra_reduce([gc[:m // 2]] + [p[0] for p in peers_dev],
                                   [gs[:m // GB]] + [p[1] for p in peers_dev], m, GB, 4)
    hic, hisc = oracle.qgz_intra_reduce([hgc[:m // 2]] + [p[0] for p in peers_host],
                                        [hgs[:m // GB]] + [p[1] for p in peers_host], m, GB, 4)
    torch.cuda.synchronize()
    same("layer first-hop codes", ic, hic)
    same("layer first-hop scales", isc, hisc)

    nodes_dev, nodes_host = [], []
    for i in range(Y - 1):                                   # what the 47 other nodes sent
        g = workloads.gradients(L, device=DEV, tensor_id=200 + i, tail_std=0.0)
        nodes_dev.append(zpp.qwz_quantize(g, GB, 4))
        nodes_host.append(oracle.qwz_quantize(workloads.as_bits(g), oracle.F16, GB, 4))
        del g
    out = zpp.qgz_inter_reduce([ic[:L // 2]] + [c for c, _ in nodes_dev], [isc[:L // GB]] + [s for _, s in nodes_dev],
                               L, GB, 4, float(W))
    torch.cuda.synchronize()
    hout = oracle.qgz_inter_reduce([hic[:L // 2]] + [c for c, _ in nodes_host],
                                   [hisc[:L // GB]] + [s for _, s in nodes_host], L, GB, 4, float(W))
    same("layer gradient partition fp32", out, hout)

    own = workloads.weights(L, device=DEV, tensor_id=2)          # the updated shard, quantized for the next gather
    qc, qs = zpp.qwz_quantize(own, WB, 8)
    torch.cuda.synchronize()
    hqc, hqs = oracle.qwz_quantize(workloads.as_bits(own), oracle.BF16, WB, 8)
    same("own shard int8 codes", qc, hqc)
    same("own shard scales", qs, hqs)
