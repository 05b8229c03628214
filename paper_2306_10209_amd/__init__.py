"""MI355X-native kernels for the compute ZeRO++ (arxiv 2306.10209) puts around
its collectives: qwZ block quantize/dequantize (Sec. 3.1) and the qgZ fused
reorder+quantize, dequant-reduce-requant and dequant-reduce stages (Sec. 3.3,
4.2).  `binding` is the thin ctypes layer over the C-ABI library; `workloads`
draws the seeded synthetic tensors."""
