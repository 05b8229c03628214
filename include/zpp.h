/*
 * zpp.h - C ABI of libzpp_gfx950: the compute ZeRO++ (arxiv 2306.10209) places
 * around its collectives, as HIP kernels for AMD MI355X (gfx950).
 *
 *   qwZ  (Sec. 3.1)   block-quantize a rank's weight shard before the all-gather,
 *                     dequantize the gathered tensor on the receiver.
 *   qgZ  (Sec. 3.3)   all-to-all based quantized gradient reduction in two hops:
 *                     slice reordering fused with quantization (Sec. 3.3.3 Eq. 1-2,
 *                     Sec. 4.1 Alg. 2, Sec. 4.2), then dequantize->reduce->quantize
 *                     after the intra-node hop and dequantize->reduce after the
 *                     inter-node hop (Sec. 3.3.2, Sec. 4.2).
 *
 * The collectives themselves are not part of this library: the caller moves the
 * bytes (or, on one GPU, passes pointers into the peers' buffers).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; the library
 *     never allocates, frees or keeps them.  Code pointers must be 16-byte
 *     aligned, scale pointers 4-byte aligned.  Inputs and outputs must not
 *     overlap.  Outputs are fully overwritten; nothing outside them is touched.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work: no synchronisation, no allocation, no state kept
 *     between calls (Sec. 4.1: quantization must be launchable asynchronously).
 *   - Pointer tables (codes_in, scales_in) are HOST arrays of device pointers;
 *     they are copied into the launch and may be reused at once.
 *   - Return value: ZPP_OK, or a negative ZPP_E* code; on error nothing is
 *     launched (ZPP_ELAUNCH: the runtime refused the launch).
 *   - dtype: ZPP_F16 / ZPP_BF16 are 16-bit storage; ZPP_F32 is 32-bit.
 *   - bits: 8 or 4.  qmax = 2^(bits-1) - 1 (127 or 7).
 *   - block: elements per quantization block; multiple of 32, 32 <= block <= 4096,
 *     so a packed block is a multiple of 16 bytes (Sec. 4.2: quantization
 *     granularities are 16 B aligned).  Tensor lengths must be multiples of the
 *     block; padding is the caller's job.
 *   - Inputs must be finite.  NaN/Inf give unspecified codes (never a fault).
 *   - Sizes: every call accepts up to 2^31 - 1 blocks; beyond that a call may
 *     return ZPP_EINVAL (nothing is launched).
 *
 * Arithmetic (fp32, each operation rounded to nearest-even on its own, no fused
 * multiply-add; results are bit-identical to a plain CPU evaluation of these
 * formulas).  For a block v[0..block):
 *     a = max|v_i|;  if a < 2^-100: scale = 0, codes = 0
 *     scale = a / qmax;  inv = qmax / a;  code_i = roundeven(v_i * inv)
 *     decode(code, scale) = float(code) * scale
 *
 * Storage: int8 codes are two's-complement bytes.  int4 codes are two's-complement
 * nibbles, element 2i in bits 0-3 and element 2i+1 in bits 4-7 of byte i.  Scales
 * are a dense float array, one per block, in the order of the blocks.
 */
#ifndef ZPP_H
#define ZPP_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZPP_OK 0
#define ZPP_EINVAL (-1)       /* bad argument: null, misaligned, size not a multiple, out of range */
#define ZPP_ELAUNCH (-2)      /* the HIP runtime reported an error for the launch */

#define ZPP_F16 0
#define ZPP_BF16 1
#define ZPP_F32 2

#define ZPP_MAX_PEERS 64 /* upper limit of `ranks` / `nodes` in the reduce stages */

/* Bytes of `n` packed codes: n*bits/8.  0 if bits is not 4 or 8. */
size_t zpp_codes_bytes(size_t n, int bits);
/* Number of scales of an n-element tensor: n/block.  0 if block <= 0. */
size_t zpp_scales_count(size_t n, int block);
/* Static text for a return code. */
const char* zpp_strerror(int code);

/* Sec. 3.3.3 Eq. (2) / Sec. 4.1 Alg. 2, host helpers (no GPU work).
 * With X GPUs per node, Y nodes and S pipeline stages a gradient is S*X*Y slices.
 * zpp_reorder_source_slice: which original slice sits at new position p;
 * zpp_reorder_mapped_slice: new position of original slice pid.  -1 on bad input.
 * Within each stage's X*Y slices, new position j*Y + i holds slice i*X + j. */
long long zpp_reorder_source_slice(long long p, int ranks_per_node, int nodes, int stages);
long long zpp_reorder_mapped_slice(long long pid, int ranks_per_node, int nodes, int stages);

/*
 * qwz_quantize - Sec. 3.1 (sender side of the quantized weight all-gather).
 *   x       [in]  n elements of `dtype` (F16/BF16/F32), the rank's flat shard
 *   codes   [out] zpp_codes_bytes(n, bits) bytes
 *   scales  [out] n/block floats
 * Block b covers flat elements [b*block, (b+1)*block).  Writing a shard's codes
 * and scales at its offset inside a larger buffer gives the same bytes as
 * quantizing the whole tensor at once, so no concatenation step is needed.
 * n = 0 is a no-op.
 */
int qwz_quantize(const void* x, int dtype, size_t n, int block, int bits,
                 void* codes, float* scales, void* stream);

/*
 * qwz_dequantize - Sec. 3.1 (receiver side): y_i = narrow(float(code_i) * scale[i/block]),
 * narrowed to out_dtype with round-to-nearest-even (F32: stored as is).
 *   codes [in] zpp_codes_bytes(n, bits) bytes;  scales [in] n/block floats;
 *   y     [out] n elements of out_dtype.
 */
int qwz_dequantize(const void* codes, const float* scales, size_t n, int block, int bits,
                   int out_dtype, void* y, void* stream);

/*
 * qgz_reorder - Sec. 3.3.3 + Sec. 4.2: tensor-slice reordering fused with block
 * quantization, one pass over the gradient.
 *   grad [in] n elements of `dtype`, viewed as stages*X*Y slices of L = n/(stages*X*Y)
 *   codes/scales [out] as qwz_quantize, in the reordered slice order: output slice p
 *   holds the quantized original slice zpp_reorder_source_slice(p, X, Y, stages).
 * With stages = 1 the output bytes [j*n/X, (j+1)*n/X) (in elements) are what local
 * GPU j of the node receives in the intra-node all-to-all.
 * Requires n % (stages*X*Y*block) == 0 (the block grid restarts at each slice).
 */
int qgz_reorder(const void* grad, int dtype, size_t n,
                int ranks_per_node, int nodes, int stages,
                int block, int bits, void* codes, float* scales, void* stream);

/*
 * qgz_intra_reduce - Sec. 3.3.2 first hop + Sec. 4.2 fused dequantize->reduce->quantize.
 *   codes_in[k], scales_in[k]  k < ranks: peer k's contribution, m elements each
 *   codes_out [out] zpp_codes_bytes(m, bits) bytes;  scales_out [out] m/block floats
 * r_e = sum over k ascending of decode(code_k[e], scale_k[e/block]) in fp32, starting
 * from +0; then every block of r is quantized as in qwz_quantize.  A plain sum: the
 * division for the average is taken once, in qgz_inter_reduce.
 */
int qgz_intra_reduce(const void* const* codes_in, const float* const* scales_in, int ranks,
                     size_t m, int block, int bits,
                     void* codes_out, float* scales_out, void* stream);

/*
 * qgz_inter_reduce - Sec. 3.3.1/3.3.2 second hop: dequantize, reduce in full precision.
 *   codes_in[i], scales_in[i]  i < nodes: node i's contribution, m elements each
 *   out [out] m floats:  out_e = (sum over i ascending of decode(...)) / divisor
 * divisor = world size for the gradient average, 1 for the sum; must be > 0.
 */
int qgz_inter_reduce(const void* const* codes_in, const float* const* scales_in, int nodes,
                     size_t m, int block, int bits, float divisor,
                     float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZPP_H */
