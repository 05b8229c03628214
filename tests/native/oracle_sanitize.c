/* Drives every entry point of the CPU oracle (oracle/zpp_oracle.c) over a sweep of shapes with
 * heap buffers of exactly the documented sizes, so that a build with -fsanitize=address,undefined
 * reports any access outside them and any undefined arithmetic.  Prints one hash line per case;
 * tests/test_sanitizers.py builds it twice (plain and sanitized), runs both and compares the
 * lines.  Test infrastructure: compiled together with the oracle's source, no GPU involved.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_qwz_quantize(const void* x, int dtype, size_t n, int block, int bits, void* codes, float* scales);
int oracle_qwz_dequantize(const void* codes, const float* scales, size_t n, int block, int bits, int out_dtype,
                          void* y);
int oracle_qgz_reorder(const void* grad, int dtype, size_t n, int X, int Y, int S, int block, int bits, void* codes,
                       float* scales);
int oracle_qgz_intra_reduce(const void* const* codes_in, const float* const* scales_in, int X, size_t m, int block,
                            int bits, void* codes_out, float* scales_out);
int oracle_qgz_inter_reduce(const void* const* codes_in, const float* const* scales_in, int Y, size_t m, int block,
                            int bits, float divisor, float* out);
long long oracle_reorder_source_slice(long long p, int X, int Y, int S);
long long oracle_reorder_mapped_slice(long long pid, int X, int Y, int S);
float oracle_widen(uint16_t h, int dtype);
uint16_t oracle_narrow(float f, int dtype);
int oracle_set_threads(int t);

static uint64_t rng = 0x9E3779B97F4A7C15ULL;
static uint32_t next_u32(void)
{
    rng = rng * 6364136223846793005ULL + 1442695040888963407ULL;
    return (uint32_t)(rng >> 32);
}

static uint64_t fnv(uint64_t h, const void* p, size_t bytes)
{
    const unsigned char* b = (const unsigned char*)p;
    for (size_t i = 0; i < bytes; ++i) h = (h ^ b[i]) * 1099511628211ULL;
    return h;
}

static void* must(size_t bytes)
{
    void* p = malloc(bytes ? bytes : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    return p;
}

/* n finite values of `dtype` (0 fp16, 1 bf16, 2 fp32) over many magnitudes, with zeros, subnormals and
 * the largest finite values mixed in */
static void* make_input(int dtype, size_t n)
{
    if (dtype == 2) {
        float* f = (float*)must(n * 4);
        for (size_t i = 0; i < n; ++i) {
            uint32_t r = next_u32(), e = 1u + r % 253u;           /* biased exponents 1..253 */
            uint32_t u = (r & 0x80000000u) | (e << 23) | ((r >> 7) & 0x7FFFFFu);
            if (r % 37u == 0u) u &= 0x80000000u;                  /* +-0 */
            if (r % 41u == 0u) u &= 0x807FFFFFu;                  /* subnormal */
            memcpy(&f[i], &u, 4);
        }
        return f;
    }
    uint16_t* h = (uint16_t*)must(n * 2);
    for (size_t i = 0; i < n; ++i) {
        uint32_t r = next_u32();
        uint16_t v;
        if (dtype == 0) {
            uint32_t e = r % 31u;                                 /* 0 (zero / subnormal) .. 30 */
            v = (uint16_t)(((r >> 16) & 0x8000u) | (e << 10) | ((r >> 5) & 0x3FFu));
        } else {
            uint32_t e = r % 255u;                                /* 0 .. 254 */
            v = (uint16_t)(((r >> 16) & 0x8000u) | (e << 7) | ((r >> 5) & 0x7Fu));
        }
        if (r % 29u == 0u) v &= 0x8000u;
        h[i] = v;
    }
    return h;
}

static size_t codes_bytes(size_t n, int bits) { return bits == 32 ? n * 4 : n * (size_t)bits / 8; }
static size_t elem_bytes(int dtype) { return dtype == 2 ? 4 : 2; }

int main(void)
{
    static const int blocks_sizes[] = {32, 96, 256, 512, 2048, 4096};
    static const int widths[] = {8, 4, 32};
    uint64_t all = 14695981039346656037ULL;
    int cases = 0;
    oracle_set_threads(2);

    /* conversions: every 16-bit pattern through widen, and back through narrow */
    for (int dt = 0; dt < 2; ++dt) {
        uint64_t h = 14695981039346656037ULL;
        for (uint32_t u = 0; u < 65536u; ++u) {
            float f = oracle_widen((uint16_t)u, dt);
            if (f == f && f - f == 0.0f) {                        /* finite */
                uint16_t back = oracle_narrow(f, dt);
                h = fnv(h, &back, 2);
            }
            h = fnv(h, &f, 4);
        }
        printf("convert dtype=%d %016llx\n", dt, (unsigned long long)h);
        all = fnv(all, &h, 8);
    }

    /* the slice maps: every index of several shapes, and the rejected ones */
    {
        uint64_t h = 14695981039346656037ULL;
        static const int shp[][3] = {{1, 1, 1}, {2, 2, 1}, {8, 6, 2}, {3, 5, 4}, {16, 7, 1}, {1, 9, 3}};
        for (size_t s = 0; s < sizeof shp / sizeof shp[0]; ++s) {
            long long total = (long long)shp[s][0] * shp[s][1] * shp[s][2];
            for (long long p = -1; p <= total; ++p) {
                long long a = oracle_reorder_source_slice(p, shp[s][0], shp[s][1], shp[s][2]);
                long long b = oracle_reorder_mapped_slice(p, shp[s][0], shp[s][1], shp[s][2]);
                h = fnv(h, &a, 8);
                h = fnv(h, &b, 8);
            }
        }
        long long bad = oracle_reorder_source_slice(0, 0, 1, 1);
        h = fnv(h, &bad, 8);
        printf("slice maps %016llx\n", (unsigned long long)h);
        all = fnv(all, &h, 8);
    }

    for (size_t bi = 0; bi < sizeof blocks_sizes / sizeof blocks_sizes[0]; ++bi)
        for (size_t wi = 0; wi < sizeof widths / sizeof widths[0]; ++wi)
            for (int dtype = 0; dtype < 3; ++dtype) {
                const int B = blocks_sizes[bi], bits = widths[wi];
                if (bits == 32 && dtype != 2 && B != 32) continue;   /* exact mode: a few cases are enough */
                const int X = 2 + (int)(bi % 3), Y = 1 + (int)((bi + wi) % 3), S = 1 + (int)(wi % 2);
                const size_t L = (size_t)B * (1 + (bi + (size_t)dtype) % 2);
                const size_t n = L * (size_t)X * Y * S, nb = n / B;
                uint64_t h = 14695981039346656037ULL;

                /* quantize, dequantize */
                void* x = make_input(dtype, n);
                void* codes = must(codes_bytes(n, bits));
                float* scales = (float*)must(nb * 4);
                if (oracle_qwz_quantize(x, dtype, n, B, bits, codes, scales)) return 3;
                h = fnv(h, codes, codes_bytes(n, bits));
                h = fnv(h, scales, nb * 4);
                for (int odt = 0; odt < 3; ++odt) {
                    void* y = must(n * elem_bytes(odt));
                    if (oracle_qwz_dequantize(codes, scales, n, B, bits, odt, y)) return 3;
                    h = fnv(h, y, n * elem_bytes(odt));
                    free(y);
                }
                /* reorder of X peers' gradients, first hop on local rank 0, second hop on node 0 */
                void** pc = (void**)must(sizeof(void*) * (size_t)X);
                float** ps = (float**)must(sizeof(float*) * (size_t)X);
                for (int k = 0; k < X; ++k) {
                    void* g = make_input(dtype, n);
                    pc[k] = must(codes_bytes(n, bits));
                    ps[k] = (float*)must(nb * 4);
                    if (oracle_qgz_reorder(g, dtype, n, X, Y, S, B, bits, pc[k], ps[k])) return 3;
                    h = fnv(h, pc[k], codes_bytes(n, bits));
                    h = fnv(h, ps[k], nb * 4);
                    free(g);
                }
                if (S == 1) {
                    const size_t m = n / (size_t)X, mb = m / B;
                    void* ic = must(codes_bytes(m, bits));
                    float* is = (float*)must(mb * 4);
                    if (oracle_qgz_intra_reduce((const void* const*)pc, (const float* const*)ps, X, m, B, bits, ic, is))
                        return 3;
                    h = fnv(h, ic, codes_bytes(m, bits));
                    h = fnv(h, is, mb * 4);
                    /* the Y slices of the first hop's result stand in for Y nodes' contributions */
                    const size_t Ls = m / (size_t)Y, lb = Ls / B;
                    const void** nc = (const void**)must(sizeof(void*) * (size_t)Y);
                    const float** ns = (const float**)must(sizeof(float*) * (size_t)Y);
                    for (int i = 0; i < Y; ++i) {
                        nc[i] = (const char*)ic + codes_bytes(Ls, bits) * (size_t)i;
                        ns[i] = is + lb * (size_t)i;
                    }
                    float* out = (float*)must(Ls * 4);
                    if (oracle_qgz_inter_reduce(nc, ns, Y, Ls, B, bits, (float)(X * Y), out)) return 3;
                    h = fnv(h, out, Ls * 4);
                    free(out); free(nc); free(ns); free(ic); free(is);
                }
                for (int k = 0; k < X; ++k) { free(pc[k]); free(ps[k]); }
                free(pc); free(ps); free(x); free(codes); free(scales);
                printf("block=%d bits=%d dtype=%d X=%d Y=%d S=%d n=%zu %016llx\n", B, bits, dtype, X, Y, S, n,
                       (unsigned long long)h);
                all = fnv(all, &h, 8);
                ++cases;
            }

    /* arguments the oracle must refuse without touching memory */
    {
        char dummy[64] = {0};
        float f[4] = {0};
        int rc = 0;
        rc += oracle_qwz_quantize(dummy, 0, 100, 32, 8, dummy, f) != 0;      /* n % block */
        rc += oracle_qwz_quantize(dummy, 7, 32, 32, 8, dummy, f) != 0;       /* dtype */
        rc += oracle_qwz_quantize(dummy, 0, 32, 32, 3, dummy, f) != 0;       /* bits */
        rc += oracle_qwz_dequantize(dummy, f, 32, 0, 8, 0, dummy) != 0;      /* block */
        rc += oracle_qgz_reorder(dummy, 0, 64, 2, 2, 1, 32, 4, dummy, f) != 0; /* n % (slices * block) */
        printf("refusals %d of 5\n", rc);
        if (rc != 5) return 4;
    }
    printf("cases %d all %016llx\n", cases, (unsigned long long)all);
    return 0;
}
