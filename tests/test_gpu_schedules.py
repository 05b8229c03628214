"""The launch schedules of Sec. 4.1 (pipelined two-hop gradient reduction with S
stages on two streams; weight quantization of the next layer overlapped with the
current layer's gather) give, bit for bit, what the oracle computes for the same
chain, with and without overlap."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_10209_amd import binding as zpp
from paper_2306_10209_amd import workloads
from paper_2306_10209_amd.schedule import QgzPipeline, QwzPrefetch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def up(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def dev_bytes(t):
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        t = t.view(torch.int16)
    return t.numpy().view(np.uint8).reshape(-1)


@pytest.mark.parametrize("X,Y,S,block,local,node", [(4, 3, 1, 64, 0, 0), (4, 3, 2, 64, 2, 1), (2, 5, 3, 32, 1, 4),
                                                    (8, 6, 4, 512, 7, 5)])
@pytest.mark.parametrize("two_streams", [False, True])
def test_pipelined_two_hop_reduction_matches_oracle(X, Y, S, block, local, node, two_streams):
    bits, W = 4, X * Y
    n = S * W * block * 3
    m_s, L_s = n // (S * X), n // (S * W)
    grad = workloads.gradients(n, seed=91, tensor_id=0)
    peers_raw = [workloads.gradients(n // X, seed=91, tensor_id=10 + k) for k in range(X - 1)]
    nodes_raw = [workloads.gradients(n // W, seed=91, tensor_id=50 + i) for i in range(Y - 1)]
    # oracle chain
    oc, os_ = oracle.qgz_reorder(workloads.as_bits(grad), oracle.F16, X, Y, S, block, bits)
    opeers = [oracle.qwz_quantize(workloads.as_bits(p), oracle.F16, block, bits) for p in peers_raw]
    onodes = [oracle.qwz_quantize(workloads.as_bits(p), oracle.F16, block, bits) for p in nodes_raw]

    def piece(c, s, start, count):
        return c[start * bits // 8:(start + count) * bits // 8], s[start // block:(start + count) // block]

    want = []
    for st in range(S):
        own = piece(oc, os_, st * (n // S) + local * m_s, m_s)
        others = [piece(c, s, st * m_s, m_s) for c, s in opeers]
        order = others[:local] + [own] + others[local:]
        mc, ms = oracle.qgz_intra_reduce([c for c, _ in order], [s for _, s in order], m_s, block, bits)
        own2 = piece(mc, ms, node * L_s, L_s)
        others2 = [piece(c, s, st * L_s, L_s) for c, s in onodes]
        order2 = others2[:node] + [own2] + others2[node:]
        want.append(oracle.qgz_inter_reduce([c for c, _ in order2], [s for _, s in order2], L_s, block, bits, float(W)))
    want = np.concatenate(want)
    # GPU schedule; the peers' and nodes' buffers are uploaded oracle encodings of the raw tensors
    pipe = QgzPipeline(n, X, Y, S, block, bits, device=DEV, two_streams=two_streams)
    pipe.bind(local, node, [(up(c), up(s)) for c, s in opeers], [(up(c), up(s)) for c, s in onodes])
    out = torch.full((S * L_s,), float("nan"), dtype=torch.float32, device=DEV)
    g = grad.to(DEV)
    for _ in range(2):          # twice: the second run must not depend on leftovers of the first
        pipe.run(g, out, float(W))
        torch.cuda.synchronize()
        assert np.array_equal(dev_bytes(out), want.view(np.uint8))
        out.fill_(float("nan"))
        torch.cuda.synchronize()


@pytest.mark.parametrize("overlap", [False, True])
def test_weight_prefetch_schedule_matches_oracle(overlap):
    P, block, bits, layers = 8, 2048, 8, 5
    n = P * block * 6
    shard, rank = n // P, 3
    full = [workloads.weights(n, seed=92, tensor_id=k) for k in range(layers)]
    enc = [oracle.qwz_quantize(workloads.as_bits(w), oracle.BF16, block, bits) for w in full]
    want = [oracle.qwz_dequantize(c, s, n, block, bits, oracle.BF16) for c, s in enc]
    sched = QwzPrefetch(n, shard, rank * shard, block, bits, device=DEV, overlap=overlap)
    shards = [w[rank * shard:(rank + 1) * shard].to(DEV) for w in full]
    outs = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for _ in range(layers)]

    # The other ranks' slots: the schedule alternates two gather buffers, so refill the slot of
    # layer k+2 only after layer k has been gathered.  For the test, run layer pairs separately.
    for k0 in range(0, layers, 2):
        ks = list(range(k0, min(k0 + 2, layers)))
        for k in ks:
            c, s = enc[k]
            slot = (k - k0) % 2
            sched.gather_codes[slot].copy_(up(c))
            sched.gather_scales[slot].copy_(up(s))
            lo = rank * shard                      # this rank's slot is poisoned: the schedule must fill it
            sched.gather_codes[slot][lo:lo + shard].fill_(0x55)
            sched.gather_scales[slot][lo // block:(lo + shard) // block].fill_(-1.0)
        torch.cuda.synchronize()
        sched.run([shards[k] for k in ks], [outs[k] for k in ks])
        torch.cuda.synchronize()
    for k in range(layers):
        assert np.array_equal(dev_bytes(outs[k]), want[k].view(np.uint8)), k


def test_calls_return_before_the_gpu_finishes():
    """The entry points only enqueue (Sec. 4.1: quantization must be launchable
    asynchronously): after a long-running kernel is queued, issuing the whole qgZ
    chain returns while the GPU is still busy."""
    import time
    n = 1 << 28
    g = workloads.gradients(n, device=DEV, tail_std=0.0)
    codes = torch.empty(n // 2, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n // 512, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    done = torch.cuda.Event()
    t0 = time.perf_counter()
    for _ in range(50):
        zpp.qgz_reorder(g, 8, 64, 1, 512, 4, codes=codes, scales=scales)
    done.record()
    issued = time.perf_counter() - t0
    busy = not done.query()
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    assert busy, f"host issue took {issued * 1e3:.2f} ms of {total * 1e3:.2f} ms: calls appear to block"
