/*
 * zpp_diagnostics.h - self-checks and a measurement helper of libzpp_gfx950.
 *
 * Not part of the method of ZeRO++ (arxiv 2306.10209) and not needed to use the five
 * operations of zpp.h: these calls exist so that tests can check, on the device they run
 * on, the short arithmetic sequences the kernels use in place of division instructions,
 * and so that benchmarks have a plain copy to compare bandwidth with.  Conventions
 * (device pointers, `stream`, return codes) are those of zpp.h.
 */
#ifndef ZPP_DIAGNOSTICS_H
#define ZPP_DIAGNOSTICS_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * zpp_selfcheck_block_scale - diagnostic.  The encoders take a block's two quotients
 * (absmax/qmax and qmax/absmax, Sec. 3.1's per-block scaling coefficient and its
 * inverse) by short fused multiply-add sequences instead of division instructions.
 * This call checks, on the device it runs on, that the sequences give the correctly
 * rounded quotients: for every one of the 2^23 fp32 mantissas at binary exponent
 * `exponent` (-100 .. 99) it compares them with plain division and ADDS the number
 * of differing a/qmax results to counts[0] and of qmax/a results to counts[1]
 * (device memory, 8-byte aligned, zeroed by the caller).  Both stay 0.
 */
int zpp_selfcheck_block_scale(int bits, int exponent, unsigned long long* counts, void* stream);

/*
 * zpp_stream_copy - measurement helper, not part of the paper's method: copies
 * `bytes` (a multiple of 16) from src to dst, 16 bytes per lane, as the bandwidth
 * ceiling the kernels are compared with (Sec. 4.2 claims full memory bandwidth).
 */
int zpp_stream_copy(void* dst, const void* src, size_t bytes, void* stream);

/*
 * zpp_selfcheck_divide - diagnostic.  qgz_inter_reduce (Sec. 3.3.2: the final reduction in
 * full precision) divides every sum by one divisor per launch.  For a divisor in
 * [2^-10, 2^16] that is not a power of two, and sums known to be 0 or in [2^-53, 2^69), it
 * does so with a correctly rounded reciprocal prepared on the host and two exact-remainder
 * corrections (5 fused operations) instead of the division sequence.  This call compares the
 * two for EVERY such dividend (both signs, and 0) and ADDS the number of differing results to
 * *count (device memory, 8-byte aligned, zeroed by the caller).  It stays 0.
 * ZPP_EINVAL if the divisor is one the kernels never treat this way.
 */
int zpp_selfcheck_divide(float divisor, unsigned long long* count, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZPP_DIAGNOSTICS_H */
