"""The five launches of a layer recorded into a HIP graph (torch's capture on the stream the
library is given) and replayed: every replay, with eager work and synchronisations between
replays, must give the bytes of the eager run, which are checked against the oracle.  The
library enqueues kernels only (no memset or copy nodes, no allocation, no host sync), which
is what makes it capturable."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_10209_amd import binding as zpp
from paper_2306_10209_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def host(t):
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        t = t.view(torch.int16)
    return t.numpy().view(np.uint8).reshape(-1)


def test_layer_sequence_replays_bit_identically():
    X, Y, WB, GB = 4, 6, 2048, 512
    W = X * Y
    n = W * GB * 2048 // 8 * 3            # 9.4M elements: thousands of wave tiles per launch
    m, L = n // X, n // W
    assert n % WB == 0 and L % WB == 0
    w = workloads.weights(n, device=DEV, tensor_id=1)
    wc, ws = zpp.qwz_quantize(w, WB, 8)
    y = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    grad = workloads.gradients(n, device=DEV, tensor_id=3)
    gc = torch.empty(n // 2, dtype=torch.uint8, device=DEV)
    gs = torch.empty(n // GB, dtype=torch.float32, device=DEV)
    peers_raw = [workloads.gradients(m, device=DEV, tensor_id=100 + k) for k in range(X - 1)]
    peers = [zpp.qwz_quantize(g, GB, 4) for g in peers_raw]
    nodes_raw = [workloads.gradients(L, device=DEV, tensor_id=200 + i) for i in range(Y - 1)]
    nodes = [zpp.qwz_quantize(g, GB, 4) for g in nodes_raw]
    ic = torch.empty(m // 2, dtype=torch.uint8, device=DEV)
    isc = torch.empty(m // GB, dtype=torch.float32, device=DEV)
    out = torch.empty(L, dtype=torch.float32, device=DEV)
    own = workloads.weights(L, device=DEV, tensor_id=2)
    oc = torch.empty(L, dtype=torch.uint8, device=DEV)
    osc = torch.empty(L // WB, dtype=torch.float32, device=DEV)
    hop1 = zpp.PeerTable([gc[:m // 2]] + [p[0] for p in peers], [gs[:m // GB]] + [p[1] for p in peers])
    hop2 = zpp.PeerTable([ic[:L // 2]] + [c for c, _ in nodes], [isc[:L // GB]] + [s for _, s in nodes])
    outputs = (y, gc, gs, ic, isc, out, oc, osc)

    def layer():
        zpp.qwz_dequantize(wc, ws, n, WB, 8, out=y)
        zpp.qgz_reorder(grad, X, Y, 1, GB, 4, codes=gc, scales=gs)
        zpp.qgz_intra_reduce(hop1, None, m, GB, 4, codes_out=ic, scales_out=isc)
        zpp.qgz_inter_reduce(hop2, None, L, GB, 4, float(W), out=out)
        zpp.qwz_quantize(own, WB, 8, codes=oc, scales=osc)

    layer()
    torch.cuda.synchronize()
    eager = [t.clone() for t in outputs]

    # the eager result is the oracle's
    hwc, hws = oracle.qwz_quantize(workloads.as_bits(w), oracle.BF16, WB, 8)
    assert np.array_equal(host(y), oracle.qwz_dequantize(hwc, hws, n, WB, 8, oracle.BF16).view(np.uint8))
    hgc, hgs = oracle.qgz_reorder(workloads.as_bits(grad), oracle.F16, X, Y, 1, GB, 4)
    hp = [oracle.qwz_quantize(workloads.as_bits(g), oracle.F16, GB, 4) for g in peers_raw]
    hic, hisc = oracle.qgz_intra_reduce([hgc[:m // 2]] + [c for c, _ in hp], [hgs[:m // GB]] + [s for _, s in hp],
                                        m, GB, 4)
    hn = [oracle.qwz_quantize(workloads.as_bits(g), oracle.F16, GB, 4) for g in nodes_raw]
    hout = oracle.qgz_inter_reduce([hic[:L // 2]] + [c for c, _ in hn], [hisc[:L // GB]] + [s for _, s in hn],
                                   L, GB, 4, float(W))
    assert np.array_equal(host(out), hout.view(np.uint8))
    assert np.array_equal(host(ic), hic) and np.array_equal(host(gc), hgc)

    side = torch.cuda.Stream(device=DEV)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        layer()                              # warm the stream before recording
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            layer()
    torch.cuda.synchronize()
    for replay in range(4):
        for t in outputs:                    # eager work between replays: wipe every output
            t.view(torch.uint8).fill_(0x5A)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, e in zip(outputs, eager):
            assert torch.equal(t.view(torch.uint8), e.view(torch.uint8)), f"replay {replay} differs from the eager run"
        layer()                              # and an eager pass of the same work
        torch.cuda.synchronize()
