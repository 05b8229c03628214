/*
 * CPU oracle for the ZeRO++ quantized-communication compute (arxiv 2306.10209).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
 * correct statement of what the five hot-path operations compute, written from
 * the paper (Sec. 3.1 block quantization of weights; Sec. 3.3.1-3.3.3 all-to-all
 * quantized gradient reduction with tensor-slice reordering, Eq. 1-2; Sec. 4.1
 * Alg. 2 generalized reordering with pipeline stages; Sec. 4.2 the fused
 * operators).  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  It shares no code with the GPU library.
 *
 * The paper gives no formula for its "symmetric quantization with an
 * independent scaling coefficient per block"; the arithmetic below is the
 * reading this build fixes (all fp32, every operation rounded separately to
 * nearest-even, no fused multiply-add):
 *
 *   QUANT(v[0..B), bits):   qmax = 2^(bits-1) - 1
 *       a     = max_i |v_i|
 *       if a < 2^-100:  scale = +0, all codes = 0
 *       scale = a / qmax                       (stored)
 *       inv   = qmax / a                       (not stored; one division per block)
 *       q_i   = clamp(roundeven(v_i * inv), -qmax, +qmax)
 *   DEQUANT(q, scale) = float(q) * scale
 *
 * Storage: int8 codes are two's-complement bytes; int4 codes are two's-complement
 * nibbles, element 2i in the low nibble and element 2i+1 in the high nibble of
 * byte i; scales are a dense float array, one per block, in block order.
 *
 * bits == 32 is the oracle-only "exact mode": codes are the fp32 values
 * themselves and every scale is 1, so the routing (reorder, two-hop sums) can
 * be checked against the textbook definition of reduce-scatter.
 *
 * Parallelism: OpenMP over blocks / output elements only, never inside a
 * reduction, so results do not depend on the thread count.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)

enum { DT_F16 = 0, DT_BF16 = 1, DT_F32 = 2 };

/* ------------------------------------------------------------------ */
/* 16-bit storage formats <-> fp32                                      */
/* ------------------------------------------------------------------ */

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* IEEE binary16 -> binary32, exact (subnormals become normal fp32 numbers). */
static float widen_f16(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu;
    uint32_t m = h & 0x3ffu;
    if (e == 0x1fu) return bits_to_float(sign | 0x7f800000u | (m << 13));
    if (e == 0) {
        /* value = m * 2^-24, exactly representable */
        float v = (float)m * 0x1p-24f;
        return sign ? -v : v;
    }
    return bits_to_float(sign | ((e + 112u) << 23) | (m << 13));
}

/* bfloat16 is the upper half of a binary32. */
static float widen_bf16(uint16_t h) { return bits_to_float((uint32_t)h << 16); }

/* binary32 -> binary16, round to nearest even, overflow to infinity. */
static uint16_t narrow_f16(float f)
{
    uint32_t u = float_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t au = u & 0x7fffffffu;
    if (au >= 0x7f800000u) /* inf / nan */
        return (uint16_t)(sign | 0x7c00u | ((au > 0x7f800000u) ? 0x200u : 0u));
    float a = bits_to_float(au);
    if (a >= 65520.0f) return (uint16_t)(sign | 0x7c00u); /* rounds to inf */
    if (a < 0x1p-14f) {
        /* result is subnormal (or zero): integer multiple of 2^-24; the product
           below is exact, nearbyintf rounds half to even */
        float r = nearbyintf(a * 0x1p24f);
        return (uint16_t)(sign | (uint16_t)r); /* r == 1024 gives the smallest normal */
    }
    /* normal: drop 13 mantissa bits with round-half-even */
    uint32_t e = (au >> 23) - 112u;
    uint32_t m = au & 0x7fffffu;
    uint32_t keep = m >> 13, rest = m & 0x1fffu;
    uint32_t h = (e << 10) | keep;
    if (rest > 0x1000u || (rest == 0x1000u && (keep & 1u))) h += 1; /* may carry into exponent */
    return (uint16_t)(sign | h);
}

/* binary32 -> bfloat16, round to nearest even. */
static uint16_t narrow_bf16(float f)
{
    uint32_t u = float_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u); /* nan */
    uint32_t keep = u >> 16, rest = u & 0xffffu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
    return (uint16_t)keep;
}

static float load_elem(const void* x, int dtype, size_t i)
{
    switch (dtype) {
    case DT_F16: return widen_f16(((const uint16_t*)x)[i]);
    case DT_BF16: return widen_bf16(((const uint16_t*)x)[i]);
    default: return ((const float*)x)[i];
    }
}

static void store_elem(void* y, int dtype, size_t i, float v)
{
    switch (dtype) {
    case DT_F16: ((uint16_t*)y)[i] = narrow_f16(v); break;
    case DT_BF16: ((uint16_t*)y)[i] = narrow_bf16(v); break;
    default: ((float*)y)[i] = v; break;
    }
}

/* exported so the conversions themselves can be pinned against numpy */
float oracle_widen(uint16_t h, int dtype) { return dtype == DT_F16 ? widen_f16(h) : widen_bf16(h); }
uint16_t oracle_narrow(float f, int dtype) { return dtype == DT_F16 ? narrow_f16(f) : narrow_bf16(f); }

/* ------------------------------------------------------------------ */
/* code storage                                                         */
/* ------------------------------------------------------------------ */

static int valid_bits(int bits) { return bits == 8 || bits == 4 || bits == 32; }

static void put_code(void* codes, int bits, size_t i, int q)
{
    if (bits == 8) {
        ((int8_t*)codes)[i] = (int8_t)q;
    } else {
        uint8_t* p = (uint8_t*)codes + (i >> 1);
        uint8_t nib = (uint8_t)(q & 0xf);
        if (i & 1) *p = (uint8_t)((*p & 0x0fu) | (nib << 4));
        else *p = (uint8_t)((*p & 0xf0u) | nib);
    }
}

static int get_code(const void* codes, int bits, size_t i)
{
    if (bits == 8) return ((const int8_t*)codes)[i];
    uint8_t b = ((const uint8_t*)codes)[i >> 1];
    int nib = (i & 1) ? (b >> 4) : (b & 0xf);
    return nib >= 8 ? nib - 16 : nib;
}

/* ------------------------------------------------------------------ */
/* QUANT / DEQUANT of one block                                         */
/* ------------------------------------------------------------------ */

/* v: B fp32 values; writes codes for elements [base, base+B) and returns the scale. */
static float quant_block(const float* v, int B, int bits, void* codes, size_t base)
{
    if (bits == 32) { /* exact mode */
        memcpy((float*)codes + base, v, (size_t)B * sizeof(float));
        return 1.0f;
    }
    const float qmax = (float)((1 << (bits - 1)) - 1);
    float a = 0.0f;
    for (int i = 0; i < B; ++i) {
        float m = fabsf(v[i]);
        if (m > a) a = m;
    }
    if (a < 0x1p-100f) {
        for (int i = 0; i < B; ++i) put_code(codes, bits, base + (size_t)i, 0);
        return 0.0f;
    }
    const float scale = a / qmax;
    const float inv = qmax / a;
    for (int i = 0; i < B; ++i) {
        float t = v[i] * inv;
        float r = nearbyintf(t); /* default rounding mode: half to even */
        if (r > qmax) r = qmax;
        if (r < -qmax) r = -qmax;
        put_code(codes, bits, base + (size_t)i, (int)r);
    }
    return scale;
}

static float dequant_elem(const void* codes, const float* scales, int bits, int B, size_t e)
{
    if (bits == 32) return ((const float*)codes)[e];
    float q = (float)get_code(codes, bits, e);
    return q * scales[e / (size_t)B];
}

/* ------------------------------------------------------------------ */
/* argument checks shared by the entry points                           */
/* ------------------------------------------------------------------ */

static int valid_block(size_t n, int block) { return block >= 1 && n % (size_t)block == 0; }
static int valid_dtype(int dtype) { return dtype == DT_F16 || dtype == DT_BF16 || dtype == DT_F32; }

#define MAX_ORACLE_BLOCK 16384

/* ------------------------------------------------------------------ */
/* Slice reordering, Sec. 3.3.3 Eq. (1)-(2) and Sec. 4.1 Alg. 2        */
/* ------------------------------------------------------------------ */

/* Gather form: which ORIGINAL slice sits at NEW position p.
 * Within one pipeline stage of T = X*Y slices, Eq. (2) lists the new order as
 * 0, X, 2X, ..., (Y-1)X, 1, X+1, ...: new position j*Y + i holds slice i*X + j
 * (i = node, j = GPU inside the node).  With S stages the tensor is S such
 * groups back to back and the permutation acts inside each group. */
long long oracle_reorder_source_slice(long long p, int X, int Y, int S)
{
    long long T = (long long)X * Y;
    if (X < 1 || Y < 1 || S < 1 || p < 0 || p >= T * S) return -1;
    long long st = p / T, w = p % T;
    long long j = w / Y, i = w % Y;
    return st * T + i * X + j;
}

/* Scatter form: the NEW position of ORIGINAL slice pid (what Alg. 2 returns). */
long long oracle_reorder_mapped_slice(long long pid, int X, int Y, int S)
{
    long long T = (long long)X * Y;
    if (X < 1 || Y < 1 || S < 1 || pid < 0 || pid >= T * S) return -1;
    long long st = pid / T, w = pid % T;
    long long i = w / X, j = w % X;
    return st * T + j * Y + i;
}

/* ------------------------------------------------------------------ */
/* the five operations                                                  */
/* ------------------------------------------------------------------ */

/* Sec. 3.1: cut the flat tensor into blocks of `block` elements, quantize each
 * block with its own scale. */
int oracle_qwz_quantize(const void* x, int dtype, size_t n, int block, int bits,
                        void* codes, float* scales)
{
    if (!x || !codes || !scales || !valid_dtype(dtype) || !valid_bits(bits)) return ORACLE_EINVAL;
    if (!valid_block(n, block) || block > MAX_ORACLE_BLOCK) return ORACLE_EINVAL;
    if (bits == 4 && (block & 1)) return ORACLE_EINVAL;
    const long long nb = (long long)(n / (size_t)block);
#pragma omp parallel for schedule(static)
    for (long long b = 0; b < nb; ++b) {
        float v[MAX_ORACLE_BLOCK];
        size_t base = (size_t)b * (size_t)block;
        for (int i = 0; i < block; ++i) v[i] = load_elem(x, dtype, base + (size_t)i);
        scales[b] = quant_block(v, block, bits, codes, base);
    }
    return ORACLE_OK;
}

/* Sec. 3.1: receiver side, integer code times the block's scale, narrowed to
 * the 16-bit training dtype. */
int oracle_qwz_dequantize(const void* codes, const float* scales, size_t n, int block, int bits,
                          int out_dtype, void* y)
{
    if (!y || !codes || !scales || !valid_dtype(out_dtype) || !valid_bits(bits)) return ORACLE_EINVAL;
    if (!valid_block(n, block)) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (long long e = 0; e < (long long)n; ++e)
        store_elem(y, out_dtype, (size_t)e, dequant_elem(codes, scales, bits, block, (size_t)e));
    return ORACLE_OK;
}

/* Sec. 3.3.3 + Sec. 4.2 "fused quantization and remapping": slices are moved
 * to their new positions and block-quantized there.  The block grid restarts
 * at every slice (slice length is a multiple of the block). */
int oracle_qgz_reorder(const void* grad, int dtype, size_t n, int X, int Y, int S,
                       int block, int bits, void* codes, float* scales)
{
    if (!grad || !codes || !scales || !valid_dtype(dtype) || !valid_bits(bits)) return ORACLE_EINVAL;
    if (X < 1 || Y < 1 || S < 1 || block < 1 || block > MAX_ORACLE_BLOCK) return ORACLE_EINVAL;
    if (bits == 4 && (block & 1)) return ORACLE_EINVAL;
    const size_t slices = (size_t)X * (size_t)Y * (size_t)S;
    if (n % (slices * (size_t)block) != 0) return ORACLE_EINVAL;
    const size_t L = n / slices;
    const size_t bps = L / (size_t)block; /* blocks per slice */
    const long long nb = (long long)(n / (size_t)block);
#pragma omp parallel for schedule(static)
    for (long long ob = 0; ob < nb; ++ob) {
        float v[MAX_ORACLE_BLOCK];
        size_t p = (size_t)ob / bps, r = (size_t)ob % bps;
        size_t src = (size_t)oracle_reorder_source_slice((long long)p, X, Y, S);
        size_t in_base = src * L + r * (size_t)block;
        size_t out_base = (size_t)ob * (size_t)block;
        for (int i = 0; i < block; ++i) v[i] = load_elem(grad, dtype, in_base + (size_t)i);
        scales[ob] = quant_block(v, block, bits, codes, out_base);
    }
    return ORACLE_OK;
}

/* Sec. 3.3.2 first hop, after the intra-node all-to-all: decode the X peers'
 * contributions, add them in fp32 in ascending peer order, quantize the sums
 * again for the inter-node hop (Sec. 4.2: one fused operator). */
int oracle_qgz_intra_reduce(const void* const* codes_in, const float* const* scales_in, int X,
                            size_t m, int block, int bits, void* codes_out, float* scales_out)
{
    if (!codes_in || !scales_in || !codes_out || !scales_out || !valid_bits(bits)) return ORACLE_EINVAL;
    if (X < 1 || !valid_block(m, block) || block > MAX_ORACLE_BLOCK) return ORACLE_EINVAL;
    if (bits == 4 && (block & 1)) return ORACLE_EINVAL;
    for (int k = 0; k < X; ++k)
        if (!codes_in[k] || !scales_in[k]) return ORACLE_EINVAL;
    const long long nb = (long long)(m / (size_t)block);
#pragma omp parallel for schedule(static)
    for (long long b = 0; b < nb; ++b) {
        float r[MAX_ORACLE_BLOCK];
        size_t base = (size_t)b * (size_t)block;
        for (int i = 0; i < block; ++i) {
            float s = 0.0f;
            for (int k = 0; k < X; ++k)
                s = s + dequant_elem(codes_in[k], scales_in[k], bits, block, base + (size_t)i);
            r[i] = s;
        }
        scales_out[b] = quant_block(r, block, bits, codes_out, base);
    }
    return ORACLE_OK;
}

/* Sec. 3.3.1 / 3.3.2 second hop, after the inter-node all-to-all: decode the Y
 * nodes' contributions, add in fp32 in ascending node order, divide once by
 * `divisor` (world size for the average, 1 for the sum). */
int oracle_qgz_inter_reduce(const void* const* codes_in, const float* const* scales_in, int Y,
                            size_t m, int block, int bits, float divisor, float* out)
{
    if (!codes_in || !scales_in || !out || !valid_bits(bits)) return ORACLE_EINVAL;
    if (Y < 1 || !valid_block(m, block) || !(divisor > 0.0f)) return ORACLE_EINVAL;
    for (int i = 0; i < Y; ++i)
        if (!codes_in[i] || !scales_in[i]) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (long long e = 0; e < (long long)m; ++e) {
        float s = 0.0f;
        for (int i = 0; i < Y; ++i)
            s = s + dequant_elem(codes_in[i], scales_in[i], bits, block, (size_t)e);
        out[e] = s / divisor;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* thread control for the timed baseline                                */
/* ------------------------------------------------------------------ */

int oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t >= 1) omp_set_num_threads(t);
    return omp_get_max_threads();
#else
    (void)t;
    return 1;
#endif
}
