"""Launch schedules of Sec. 4.1 of the paper on top of the five kernels.

Only stream and event plumbing lives here (torch streams at the default
priority); every byte is still produced by the library's kernels.  On one GPU
the collectives are stand-ins: an "all-to-all" is a pointer table into buffers
the peers already filled, the "all-gather" of the weight schedule is a plain
device copy of the gathered codes.

* QgzPipeline: the gradient is cut into S pipeline stages; stage s's
  dequantize -> reduce -> quantize (intra-node hop) runs on one stream while
  stage s-1's dequantize -> reduce (inter-node hop) runs on another (Sec. 4.1, the
  pipelining figure; the slice order for S stages is the generalized reordering of
  Alg. 2).
* QwzPrefetch: layer k+1's own-shard quantization is enqueued on a side stream
  while layer k's (stand-in) all-gather and dequantization run on the main
  stream; the main stream waits on an event only where it needs layer k+1's
  codes.  No call blocks the host.
"""
import torch

from . import binding as zpp


class QgzPipeline:
    """One GPU's share of the two-hop quantized gradient reduction with S stages.

    Layout (all stage-major, as qgz_reorder writes it): the reordered gradient is S
    stage regions of n/S elements; inside a region, group j (n/(S*X) elements) goes
    to local GPU j.  A peer's contribution for this GPU is therefore S pieces of
    m_s = n/(S*X) elements; they are passed as one buffer of n/X elements with stage
    s at offset s*m_s.  Likewise a node's contribution to the second hop is S pieces
    of L_s = n/(S*X*Y) elements in one buffer of n/(X*Y) elements.  The result is this
    rank's gradient partition: S pieces of L_s fp32 values, stage-major.
    """

    def __init__(self, n, X, Y, S, block, bits=4, device="cuda:0", two_streams=True):
        if n % (S * X * Y * block) != 0:
            raise zpp.ZppError("n must be a multiple of S*X*Y*block")
        self.n, self.X, self.Y, self.S, self.block, self.bits = n, X, Y, S, block, bits
        self.m_s = n // (S * X)
        self.L_s = n // (S * X * Y)
        self.device = torch.device(device)
        self.codes = torch.empty(n * bits // 8, dtype=torch.uint8, device=device)
        self.scales = torch.empty(n // block, dtype=torch.float32, device=device)
        self.mid_codes = torch.empty(self.m_s * S * bits // 8, dtype=torch.uint8, device=device)
        self.mid_scales = torch.empty(self.m_s * S // block, dtype=torch.float32, device=device)
        self.intra_stream = torch.cuda.Stream(device=device) if two_streams else None
        self.inter_stream = torch.cuda.Stream(device=device) if two_streams else None
        self._tables = None

    def _slice(self, codes, scales, start, count):
        b, B = self.bits, self.block
        return codes[start * b // 8:(start + count) * b // 8], scales[start // B:(start + count) // B]

    def bind(self, local_rank, node_rank, peers, nodes):
        """Build the pointer tables once.  peers: X-1 (codes, scales) buffers of n/X elements from
        the other local GPUs (ascending local rank, this GPU's own place skipped); nodes: Y-1
        buffers of n/(X*Y) elements from the other nodes (ascending node rank, own skipped)."""
        X, Y, S, m_s, L_s = self.X, self.Y, self.S, self.m_s, self.L_s
        if len(peers) != X - 1 or len(nodes) != Y - 1:
            raise zpp.ZppError("need X-1 peer buffers and Y-1 node buffers")
        self.local_rank, self.node_rank = local_rank, node_rank
        intra, inter = [], []
        for s in range(S):
            own = self._slice(self.codes, self.scales, s * (self.n // S) + local_rank * m_s, m_s)
            others = [self._slice(c, sc, s * m_s, m_s) for c, sc in peers]
            ordered = others[:local_rank] + [own] + others[local_rank:]
            intra.append(zpp.PeerTable([c for c, _ in ordered], [sc for _, sc in ordered]))
            # second hop: this GPU keeps the slice of its own node out of the Y it just reduced
            own2 = self._slice(self.mid_codes, self.mid_scales, s * m_s + node_rank * L_s, L_s)
            others2 = [self._slice(c, sc, s * L_s, L_s) for c, sc in nodes]
            ordered2 = others2[:node_rank] + [own2] + others2[node_rank:]
            inter.append(zpp.PeerTable([c for c, _ in ordered2], [sc for _, sc in ordered2]))
        self._tables = (intra, inter)
        return self

    def run(self, grad, out, divisor):
        """Enqueue reorder + S x (intra, inter).  Returns `out` (S*L_s floats); the caller's
        current stream waits for the result before this returns control of it."""
        if self._tables is None:
            raise zpp.ZppError("bind() first")
        intra, inter = self._tables
        S, m_s, L_s, B, b = self.S, self.m_s, self.L_s, self.block, self.bits
        main = torch.cuda.current_stream(self.device)
        zpp.qgz_reorder(grad, self.X, self.Y, S, B, b, codes=self.codes, scales=self.scales)
        if self.intra_stream is None:
            for s in range(S):
                mc, ms = self._slice(self.mid_codes, self.mid_scales, s * m_s, m_s)
                zpp.qgz_intra_reduce(intra[s], None, m_s, B, b, codes_out=mc, scales_out=ms)
                zpp.qgz_inter_reduce(inter[s], None, L_s, B, b, divisor, out=out[s * L_s:(s + 1) * L_s])
            return out
        a_stream, b_stream = self.intra_stream, self.inter_stream
        a_stream.wait_stream(main)
        b_stream.wait_stream(main)
        for s in range(S):
            mc, ms = self._slice(self.mid_codes, self.mid_scales, s * m_s, m_s)
            zpp.qgz_intra_reduce(intra[s], None, m_s, B, b, codes_out=mc, scales_out=ms, stream=a_stream)
            done = torch.cuda.Event()
            done.record(a_stream)
            b_stream.wait_event(done)
            zpp.qgz_inter_reduce(inter[s], None, L_s, B, b, divisor, out=out[s * L_s:(s + 1) * L_s], stream=b_stream)
        main.wait_stream(b_stream)
        main.wait_stream(a_stream)
        return out


class QwzPrefetch:
    """Forward-pass weight schedule over `layers` layers of n elements each.

    Per layer k on the main stream: stand-in all-gather (device copy of the gathered
    codes and scales into the receive buffer) -> qwz_dequantize.  On the side stream:
    qwz_quantize of this rank's shard of layer k+1 into its slot of layer k+1's gather
    buffer.  The main stream waits on the side stream's event just before layer k+1's
    gather.  With overlap=False everything is enqueued on the main stream in order.
    """

    def __init__(self, n, shard, shard_offset, block, bits=8, device="cuda:0", overlap=True):
        if shard % block or shard_offset % block or n % block:
            raise zpp.ZppError("sizes must be multiples of the block")
        self.n, self.shard, self.off, self.block, self.bits = n, shard, shard_offset, block, bits
        self.device = torch.device(device)
        self.side = torch.cuda.Stream(device=device) if overlap else None
        cb = n * bits // 8
        # two gather buffers (layer k in flight, layer k+1 being filled) and one receive buffer
        self.gather_codes = [torch.empty(cb, dtype=torch.uint8, device=device) for _ in range(2)]
        self.gather_scales = [torch.empty(n // block, dtype=torch.float32, device=device) for _ in range(2)]
        self.recv_codes = torch.empty(cb, dtype=torch.uint8, device=device)
        self.recv_scales = torch.empty(n // block, dtype=torch.float32, device=device)

    def _quantize_shard(self, w_shard, slot, stream):
        b, B = self.bits, self.block
        c = self.gather_codes[slot][self.off * b // 8:(self.off + self.shard) * b // 8]
        s = self.gather_scales[slot][self.off // B:(self.off + self.shard) // B]
        zpp.qwz_quantize(w_shard, B, b, codes=c, scales=s, stream=stream)

    def run(self, shards, outs):
        """shards[k]: this rank's 16-bit shard of layer k; outs[k]: n-element output of layer k
        (may all be the same buffer).  The other ranks' slots of the gather buffers are whatever
        the caller put there (gather_codes / gather_scales)."""
        main = torch.cuda.current_stream(self.device)
        side = self.side if self.side is not None else main
        layers = len(shards)
        ready = [None] * layers
        if side is not main:
            side.wait_stream(main)
        self._quantize_shard(shards[0], 0, side)
        ready[0] = torch.cuda.Event()
        ready[0].record(side)
        gathered = None
        for k in range(layers):
            if k + 1 < layers:
                if gathered is not None and side is not main:
                    side.wait_event(gathered)      # slot (k+1)%2 was last read by layer k-1's gather
                self._quantize_shard(shards[k + 1], (k + 1) % 2, side)
                ready[k + 1] = torch.cuda.Event()
                ready[k + 1].record(side)
            if side is not main:
                main.wait_event(ready[k])
            slot = k % 2
            self.recv_codes.copy_(self.gather_codes[slot], non_blocking=True)   # stand-in all-gather
            self.recv_scales.copy_(self.gather_scales[slot], non_blocking=True)
            gathered = torch.cuda.Event()
            gathered.record(main)
            zpp.qwz_dequantize(self.recv_codes, self.recv_scales, self.n, self.block, self.bits, out=outs[k])
        if side is not main:
            main.wait_stream(side)
        return outs
