"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times.

Each case checks
  (1) sampled output blocks against the oracle called one block at a time, whose
      inputs are the raw seeded tensors (copied block by block to the host), never
      anything the library wrote;
  (2) every output element against a separate evaluation with elementwise torch ops
      (IEEE fp32 multiply / add / round-half-even, one kernel per operation, so
      nothing is contracted) -- a property check that holds at any size.
test_gpu_fullsize_oracle.py adds the whole-tensor comparison with the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_10209_amd import binding as zpp
from paper_2306_10209_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


# ----------------------------------------------------------------------------
# helpers
# ----------------------------------------------------------------------------

def bits_of(t):
    """host uint16/float32 numpy view of a (slice of a) device tensor"""
    return workloads.as_bits(t)


def dev_bytes(t):
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        t = t.view(torch.int16)
    return t.numpy().view(np.uint8).reshape(-1)


def host_scale_inv(absmax_dev, bits):
    """IEEE fp32 scale = a/qmax and inv = qmax/a on the host (numpy), from block maxima."""
    qmax = np.float32((1 << (bits - 1)) - 1)
    a = absmax_dev.detach().cpu().numpy().astype(np.float32)
    tiny = a < np.float32(2.0 ** -100)
    safe = np.where(tiny, np.float32(1), a)
    scale = np.where(tiny, np.float32(0), safe / qmax).astype(np.float32)
    inv = np.where(tiny, np.float32(0), qmax / safe).astype(np.float32)
    return torch.from_numpy(scale).to(DEV), torch.from_numpy(inv).to(DEV)


def torch_codes(x, block, bits):
    """(signed codes int8 tensor, scales) by elementwise torch ops; x: 16-bit device tensor."""
    xf = x.float().view(-1, block)
    scale, inv = host_scale_inv(xf.abs().amax(dim=1), bits)
    q = torch.round(xf * inv[:, None]).to(torch.int8).view(-1)
    return q, scale


def unpack_dev(codes, bits):
    """device uint8 codes -> signed int8 tensor, one entry per element"""
    if bits == 8:
        return codes.view(torch.int8)
    lo = (codes & 0xF).to(torch.int8)
    hi = (codes >> 4).to(torch.int8)
    q = torch.stack([lo, hi], dim=1).view(-1)
    return torch.where(q >= 8, q - 16, q)


def torch_fold(codes_list, scales_list, block, bits):
    """left-to-right fp32 sum of decoded peers, elementwise torch ops"""
    s = None
    for c, sc in zip(codes_list, scales_list):
        d = (unpack_dev(c, bits).float().view(-1, block) * sc[:, None]).view(-1)
        s = d + 0.0 if s is None else s + d
    return s


def host_divide(sum_dev, divisor):
    """IEEE fp32 division on the host (numpy)"""
    return (sum_dev.detach().cpu().numpy() / np.float32(divisor)).astype(np.float32)


def sample_blocks(nblocks, count, seed, always=()):
    rng = np.random.default_rng(seed)
    picks = set(int(b) for b in always if 0 <= b < nblocks)
    picks.update(int(b) for b in rng.integers(0, nblocks, size=count))
    return sorted(picks)


# ----------------------------------------------------------------------------
# qwZ on one transformer layer, hidden 8192, bf16, P = 8 shards, int8 block 2048
# ----------------------------------------------------------------------------

def test_qwz_layer_hidden_8192():
    P, B, bits = 8, 2048, 8
    shapes = workloads.gpt_layer_shapes(8192)
    n_total = sum(r * c for _, r, c in shapes)
    assert n_total == 12 * 8192 * 8192
    codes = torch.empty(n_total, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n_total // B, dtype=torch.float32, device=DEV)
    out = torch.empty(n_total, dtype=torch.bfloat16, device=DEV)
    mats, off = [], 0
    for tid, (_, r, c) in enumerate(shapes):
        n = r * c
        w = workloads.weights(n, device=DEV, tensor_id=10 + tid)
        mats.append((off, w))
        sh = n // P
        assert sh % B == 0
        for rank in range(P):           # each rank writes its shard at its offset: the simulated all-gather
            lo = off + rank * sh
            zpp.qwz_quantize(w[rank * sh:(rank + 1) * sh], B, bits, codes=codes[lo:lo + sh],
                             scales=scales[lo // B:(lo + sh) // B])
        off += n
    zpp.qwz_dequantize(codes, scales, n_total, B, bits, out=out)
    torch.cuda.synchronize()

    for off, w in mats:
        n = w.numel()
        # (2) every element, torch route
        q, sc = torch_codes(w, B, bits)
        assert torch.equal(scales[off // B:(off + n) // B].view(torch.int32), sc.view(torch.int32))
        assert torch.equal(codes[off:off + n].view(torch.int8), q)
        want = (q.float().view(-1, B) * sc[:, None]).view(-1).to(torch.bfloat16)
        assert torch.equal(out[off:off + n].view(torch.int16), want.view(torch.int16))
        del q, sc, want
        # (1) sampled blocks, oracle from the raw weights
        nb = n // B
        shb = nb // P
        for b in sample_blocks(nb, 24, seed=off % 9973, always=(0, nb - 1, shb - 1, shb, 3 * shb)):
            xb = bits_of(w[b * B:(b + 1) * B])
            oc, os_ = oracle.qwz_quantize(xb, oracle.BF16, B, bits)
            g = off + b * B
            assert np.array_equal(dev_bytes(codes[g:g + B]), oc)
            assert np.array_equal(dev_bytes(scales[g // B:g // B + 1]), os_.view(np.uint8))
            oy = oracle.qwz_dequantize(oc, os_, B, B, bits, oracle.BF16)
            assert np.array_equal(dev_bytes(out[g:g + B]), oy.view(np.uint8))


def test_qwz_batched_small_tensors_fp16_block_256():
    """1024 tensors of 4096 x 256 fp16 in one launch (the small round-trip
    configuration, batched so that the launch is long enough to time)."""
    B, bits = 256, 8
    n = 1024 << 20
    x = workloads.weights(n, device=DEV, tensor_id=30, dtype=torch.float16, outlier_prob=0.0)
    codes, scales = zpp.qwz_quantize(x, B, bits)
    y = zpp.qwz_dequantize(codes, scales, n, B, bits, out_dtype=torch.float16)
    torch.cuda.synchronize()
    q, sc = torch_codes(x, B, bits)
    assert torch.equal(scales.view(torch.int32), sc.view(torch.int32))
    assert torch.equal(codes.view(torch.int8), q)
    want = (q.float().view(-1, B) * sc[:, None]).view(-1).to(torch.float16)
    assert torch.equal(y.view(torch.int16), want.view(torch.int16))
    for b in sample_blocks(n // B, 32, seed=1, always=(0, n // B - 1)):
        oc, os_ = oracle.qwz_quantize(bits_of(x[b * B:(b + 1) * B]), oracle.F16, B, bits)
        assert np.array_equal(dev_bytes(codes[b * B:(b + 1) * B]), oc)
        assert np.array_equal(dev_bytes(scales[b:b + 1]), os_.view(np.uint8))
        assert np.array_equal(dev_bytes(y[b * B:(b + 1) * B]),
                              oracle.qwz_dequantize(oc, os_, B, B, bits, oracle.F16).view(np.uint8))


# ----------------------------------------------------------------------------
# qgZ intra-node stage: 8 ranks x 2^28 fp16 heavy-tailed gradients, X = 8, Y = 64
# ----------------------------------------------------------------------------

def test_qgz_intra_stage_8_ranks_2p28():
    X, Y, B, bits = 8, 64, 512, 4
    n = 1 << 28
    T = X * Y
    L = n // T
    m = n // X
    bps = L // B
    grads = [workloads.gradients(n, device=DEV, tensor_id=40 + r) for r in range(X)]
    first = [zpp.qgz_reorder(g, X, Y, 1, B, bits) for g in grads]
    torch.cuda.synchronize()

    # reorder: every element by the torch route (quantize in place, then move whole slices)
    order = torch.tensor([oracle.reorder_source_slice(p, X, Y, 1) for p in range(T)], device=DEV)
    for r in (0, 5):
        q, sc = torch_codes(grads[r], B, bits)
        q = q.view(T, L)[order].reshape(-1)
        sc = sc.view(T, bps)[order].reshape(-1)
        assert torch.equal(first[r][1].view(torch.int32), sc.view(torch.int32))
        assert torch.equal(unpack_dev(first[r][0], bits), q)
        del q, sc
    # reorder: sampled output blocks against the oracle
    nb = n // B
    for r in range(X):
        for ob in sample_blocks(nb, 12, seed=r, always=(0, nb - 1, bps - 1, bps)):
            p, rb = divmod(ob, bps)
            src = oracle.reorder_source_slice(p, X, Y, 1)
            lo = src * L + rb * B
            oc, os_ = oracle.qwz_quantize(bits_of(grads[r][lo:lo + B]), oracle.F16, B, bits)
            assert np.array_equal(dev_bytes(first[r][0][ob * B // 2:(ob + 1) * B // 2]), oc)
            assert np.array_equal(dev_bytes(first[r][1][ob:ob + 1]), os_.view(np.uint8))

    cb, sb = m // 2, m // B
    for j in range(X):                  # simulated local rank j: group j of every peer, by pointer offset
        cin = [first[k][0][j * cb:(j + 1) * cb] for k in range(X)]
        sin = [first[k][1][j * sb:(j + 1) * sb] for k in range(X)]
        codes, scales = zpp.qgz_intra_reduce(cin, sin, m, B, bits)
        torch.cuda.synchronize()
        if j in (0, 7):                 # every element, torch route
            r = torch_fold(cin, sin, B, bits).view(-1, B)
            sc, inv = host_scale_inv(r.abs().amax(dim=1), bits)
            q = torch.round(r * inv[:, None]).to(torch.int8).view(-1)
            assert torch.equal(scales.view(torch.int32), sc.view(torch.int32))
            assert torch.equal(unpack_dev(codes, bits), q)
            del r, q
        # sampled output blocks: oracle on the raw gradients of all 8 peers
        for ob in sample_blocks(sb, 6, seed=100 + j, always=(0, sb - 1)):
            gb = j * sb + ob                        # block index inside the peers' reordered buffers
            p, rb = divmod(gb, bps)
            src = oracle.reorder_source_slice(p, X, Y, 1)
            lo = src * L + rb * B
            peers = [oracle.qwz_quantize(bits_of(grads[k][lo:lo + B]), oracle.F16, B, bits) for k in range(X)]
            oc, os_ = oracle.qgz_intra_reduce([c for c, _ in peers], [s for _, s in peers], B, B, bits)
            assert np.array_equal(dev_bytes(codes[ob * B // 2:(ob + 1) * B // 2]), oc)
            assert np.array_equal(dev_bytes(scales[ob:ob + 1]), os_.view(np.uint8))


# ----------------------------------------------------------------------------
# qgZ inter-node stage: 48 chunks of 46,875,136 elements (one GPU's share of an
# 18B-parameter model on 384 GPUs; 46,875,000 padded up to a multiple of 512)
# ----------------------------------------------------------------------------

def test_qgz_inter_stage_48_nodes_18b_share():
    Y, B, bits, W = 48, 512, 4, 384.0
    L = 46875136
    assert L % B == 0 and Y * L > 2 ** 31           # 64-bit element offsets are needed
    raw = [workloads.gradients(L, device=DEV, tensor_id=60 + i, tail_std=0.0) for i in range(Y)]
    enc = [zpp.qwz_quantize(g, B, bits) for g in raw]     # untimed setup in the benchmark
    out = zpp.qgz_inter_reduce([c for c, _ in enc], [s for _, s in enc], L, B, bits, W)
    torch.cuda.synchronize()
    # every element: torch route on the encoded inputs
    want = host_divide(torch_fold([c for c, _ in enc], [s for _, s in enc], B, bits), W)
    assert np.array_equal(dev_bytes(out), want.view(np.uint8))
    del want
    # sampled blocks: oracle from the raw chunks
    nb = L // B
    for ob in sample_blocks(nb, 10, seed=7, always=(0, nb - 1)):
        peers = [oracle.qwz_quantize(bits_of(g[ob * B:(ob + 1) * B]), oracle.F16, B, bits) for g in raw]
        oo = oracle.qgz_inter_reduce([c for c, _ in peers], [s for _, s in peers], B, B, bits, W)
        assert np.array_equal(dev_bytes(out[ob * B:(ob + 1) * B]), oo.view(np.uint8))


# ----------------------------------------------------------------------------
# one layer of the benchmark step: hidden 12288, X = 8, Y = 48
# ----------------------------------------------------------------------------

def test_one_layer_of_the_benchmark_step_hidden_12288():
    X, Y, W = 8, 48, 384
    WB, GB = 2048, 512
    n_L = workloads.layer_numel(12288)
    assert n_L == 1811939328
    m, L = n_L // X, n_L // W
    bps = L // GB

    # weights: quantize (setup) and dequantize
    w = workloads.weights(n_L, device=DEV, tensor_id=1)
    wc, ws = zpp.qwz_quantize(w, WB, 8)
    y = torch.empty(n_L, dtype=torch.bfloat16, device=DEV)
    zpp.qwz_dequantize(wc, ws, n_L, WB, 8, out=y)
    torch.cuda.synchronize()
    q, sc = torch_codes(w, WB, 8)
    assert torch.equal(ws.view(torch.int32), sc.view(torch.int32)) and torch.equal(wc.view(torch.int8), q)
    want = (q.float().view(-1, WB) * sc[:, None]).view(-1).to(torch.bfloat16)
    assert torch.equal(y.view(torch.int16), want.view(torch.int16))
    del q, sc, want
    for b in sample_blocks(n_L // WB, 16, seed=3, always=(0, n_L // WB - 1)):
        oc, os_ = oracle.qwz_quantize(bits_of(w[b * WB:(b + 1) * WB]), oracle.BF16, WB, 8)
        assert np.array_equal(dev_bytes(wc[b * WB:(b + 1) * WB]), oc)
        assert np.array_equal(dev_bytes(y[b * WB:(b + 1) * WB]),
                              oracle.qwz_dequantize(oc, os_, WB, WB, 8, oracle.BF16).view(np.uint8))
    del w, wc, ws, y

    # gradient path of this GPU (node 0, local rank 0)
    grad = workloads.gradients(n_L, device=DEV, tensor_id=3, tail_std=0.0)
    gc, gs = zpp.qgz_reorder(grad, X, Y, 1, GB, 4)
    peers_raw = [workloads.gradients(m, device=DEV, tensor_id=100 + k, tail_std=0.0) for k in range(X - 1)]
    peers = [zpp.qwz_quantize(g, GB, 4) for g in peers_raw]            # what the 7 other local GPUs sent
    ic, isc = zpp.qgz_intra_reduce([gc[:m // 2]] + [p[0] for p in peers], [gs[:m // GB]] + [p[1] for p in peers],
                                   m, GB, 4)
    nodes_raw = workloads.gradients((Y - 1) * L, device=DEV, tensor_id=200, tail_std=0.0)
    nc, ns = zpp.qwz_quantize(nodes_raw, GB, 4)                           # what the 47 other nodes sent
    cin = [ic[:L // 2]] + [nc[i * L // 2:(i + 1) * L // 2] for i in range(Y - 1)]
    sin = [isc[:L // GB]] + [ns[i * L // GB:(i + 1) * L // GB] for i in range(Y - 1)]
    out = zpp.qgz_inter_reduce(cin, sin, L, GB, 4, float(W))
    torch.cuda.synchronize()

    # torch route, every element of the three gradient kernels
    T = X * Y
    order = torch.tensor([oracle.reorder_source_slice(p, X, Y, 1) for p in range(T)], device=DEV)
    q, sc = torch_codes(grad, GB, 4)
    q = q.view(T, L)[order].reshape(-1)
    sc = sc.view(T, bps)[order].reshape(-1)
    assert torch.equal(gs.view(torch.int32), sc.view(torch.int32)) and torch.equal(unpack_dev(gc, 4), q)
    del q, sc
    r = torch_fold([gc[:m // 2]] + [p[0] for p in peers], [gs[:m // GB]] + [p[1] for p in peers], GB, 4).view(-1, GB)
    sc, inv = host_scale_inv(r.abs().amax(dim=1), 4)
    q = torch.round(r * inv[:, None]).to(torch.int8).view(-1)
    assert torch.equal(isc.view(torch.int32), sc.view(torch.int32)) and torch.equal(unpack_dev(ic, 4), q)
    del r, q, sc, inv
    want = host_divide(torch_fold(cin, sin, GB, 4), float(W))
    assert np.array_equal(dev_bytes(out), want.view(np.uint8))

    # oracle on sampled blocks of the final partition, from raw inputs only
    def raw_first_hop_block(gb):
        """the 8 local GPUs' quantized contributions to block gb of group 0"""
        p, rb = divmod(gb, bps)
        src = oracle.reorder_source_slice(p, X, Y, 1)
        lo = src * L + rb * GB
        mine = oracle.qwz_quantize(bits_of(grad[lo:lo + GB]), oracle.F16, GB, 4)
        others = [oracle.qwz_quantize(bits_of(g[gb * GB:(gb + 1) * GB]), oracle.F16, GB, 4) for g in peers_raw]
        return [mine] + others

    for ob in sample_blocks(bps, 6, seed=9, always=(0, bps - 1)):
        hop1 = raw_first_hop_block(ob)                      # slice 0 of group 0 is this GPU's own partition
        c1, s1 = oracle.qgz_intra_reduce([c for c, _ in hop1], [s for _, s in hop1], GB, GB, 4)
        assert np.array_equal(dev_bytes(ic[ob * GB // 2:(ob + 1) * GB // 2]), c1)
        others = [oracle.qwz_quantize(bits_of(nodes_raw[i * L + ob * GB:i * L + (ob + 1) * GB]), oracle.F16, GB, 4)
                  for i in range(Y - 1)]
        oo = oracle.qgz_inter_reduce([c1] + [c for c, _ in others], [s1] + [s for _, s in others], GB, GB, 4, float(W))
        assert np.array_equal(dev_bytes(out[ob * GB:(ob + 1) * GB]), oo.view(np.uint8))


# ----------------------------------------------------------------------------
# a single tensor of more than 2^32 elements: 64-bit element offsets everywhere
# ----------------------------------------------------------------------------

def test_single_tensor_beyond_32_bit_offsets():
    B = 2048
    n = (1 << 32) + 3 * B * 1001            # 4.3e9 elements, ragged against every tile size
    x = workloads.weights(n, device=DEV, tensor_id=77)
    codes, scales = zpp.qwz_quantize(x, B, 8)
    y = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    zpp.qwz_dequantize(codes, scales, n, B, 8, out=y)
    torch.cuda.synchronize()
    # every element, torch route, in pieces to bound the temporaries
    piece = B << 18
    for lo in range(0, n, piece):
        hi = min(lo + piece, n)
        q, sc = torch_codes(x[lo:hi], B, 8)
        assert torch.equal(scales[lo // B:hi // B].view(torch.int32), sc.view(torch.int32)), lo
        assert torch.equal(codes[lo:hi].view(torch.int8), q), lo
        want = (q.float().view(-1, B) * sc[:, None]).view(-1).to(torch.bfloat16)
        assert torch.equal(y[lo:hi].view(torch.int16), want.view(torch.int16)), lo
        del q, sc, want
    nb = n // B
    for b in sample_blocks(nb, 12, seed=11, always=(0, nb - 1, (1 << 32) // B - 1, (1 << 32) // B, (1 << 31) // B)):
        oc, os_ = oracle.qwz_quantize(bits_of(x[b * B:(b + 1) * B]), oracle.BF16, B, 8)
        assert np.array_equal(dev_bytes(codes[b * B:(b + 1) * B]), oc)
        assert np.array_equal(dev_bytes(scales[b:b + 1]), os_.view(np.uint8))
        assert np.array_equal(dev_bytes(y[b * B:(b + 1) * B]),
                              oracle.qwz_dequantize(oc, os_, B, B, 8, oracle.BF16).view(np.uint8))
    # the gradient path on the same scale: reorder of 4.3e9 fp16 elements, X = 8, Y = 48
    del codes, scales, y
    g = x.view(torch.float16)               # reinterpret the bits: any finite pattern is a valid input
    g = torch.nan_to_num(g, nan=0.0, posinf=1.0, neginf=-1.0)
    X, Y, GB = 8, 48, 512
    n2 = (n // (X * Y * GB)) * (X * Y * GB)
    g = g[:n2]
    L = n2 // (X * Y)
    gc, gs = zpp.qgz_reorder(g, X, Y, 1, GB, 4)
    torch.cuda.synchronize()
    bps = L // GB
    for ob in sample_blocks(n2 // GB, 16, seed=12, always=(0, n2 // GB - 1, (1 << 32) // GB, (1 << 32) // GB - 1)):
        p, rb = divmod(ob, bps)
        src = oracle.reorder_source_slice(p, X, Y, 1)
        lo = src * L + rb * GB
        oc, os_ = oracle.qwz_quantize(bits_of(g[lo:lo + GB]), oracle.F16, GB, 4)
        assert np.array_equal(dev_bytes(gc[ob * GB // 2:(ob + 1) * GB // 2]), oc)
        assert np.array_equal(dev_bytes(gs[ob:ob + 1]), os_.view(np.uint8))
