/* A consumer of the C ABI written in plain C: no Python, no torch, no C++.
 *
 * It allocates device memory with the HIP runtime's C interface, calls the five
 * operations of include/zpp.h on a small two-node / three-GPU gradient and on a
 * weight tensor, on a stream it created itself, and compares every output byte with
 * the CPU oracle it is linked against.  Test infrastructure: the GPU test
 * tests/test_gpu_native_client.py builds and runs it.  Exit status 0 = all equal.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "zpp.h"

/* the oracle's entry points (oracle/zpp_oracle.c) */
int oracle_qwz_quantize(const void* x, int dtype, size_t n, int block, int bits, void* codes, float* scales);
int oracle_qwz_dequantize(const void* codes, const float* scales, size_t n, int block, int bits, int out_dtype,
                          void* y);
int oracle_qgz_reorder(const void* grad, int dtype, size_t n, int X, int Y, int S, int block, int bits, void* codes,
                       float* scales);
int oracle_qgz_intra_reduce(const void* const* codes_in, const float* const* scales_in, int X, size_t m, int block,
                            int bits, void* codes_out, float* scales_out);
int oracle_qgz_inter_reduce(const void* const* codes_in, const float* const* scales_in, int Y, size_t m, int block,
                            int bits, float divisor, float* out);

#define HIP_OK(call)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            fprintf(stderr, "%s:%d: %s -> %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_)); \
            exit(2);                                                                          \
        }                                                                                     \
    } while (0)

#define ZPP_OKAY(call)                                                                  \
    do {                                                                                \
        int r_ = (call);                                                                \
        if (r_ != ZPP_OK) {                                                             \
            fprintf(stderr, "%s:%d: %s -> %s\n", __FILE__, __LINE__, #call, zpp_strerror(r_)); \
            exit(3);                                                                    \
        }                                                                               \
    } while (0)

static uint64_t rng_state = 0x2306102092023ULL;
static uint32_t next_u32(void)
{
    rng_state = rng_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (uint32_t)(rng_state >> 33);
}

/* finite fp16 bit patterns spread over a few binades around 2^-10 (gradient-like), both signs, some zeros */
static void fill_f16(uint16_t* p, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        uint32_t r = next_u32();
        if ((r & 63u) == 0u) { p[i] = (uint16_t)((r >> 8) & 0x8000u); continue; }
        uint32_t exp = 2u + (r >> 6) % 8u; /* biased exponents 2..9 */
        p[i] = (uint16_t)(((r >> 16) & 0x8000u) | (exp << 10) | ((r >> 20) & 0x3FFu));
    }
}

static void* dev_from(const void* host, size_t bytes)
{
    void* d = NULL;
    HIP_OK(hipMalloc(&d, bytes ? bytes : 16));
    if (bytes) HIP_OK(hipMemcpy(d, host, bytes, hipMemcpyHostToDevice));
    return d;
}

static void* dev_filled(size_t bytes)
{
    void* d = NULL;
    HIP_OK(hipMalloc(&d, bytes ? bytes : 16));
    HIP_OK(hipMemset(d, 0xA5, bytes)); /* outputs must not depend on what was there */
    return d;
}

static int failures = 0;
static void expect_same(const char* what, const void* dev, const void* host, size_t bytes)
{
    unsigned char* got = (unsigned char*)malloc(bytes ? bytes : 1);
    HIP_OK(hipMemcpy(got, dev, bytes, hipMemcpyDeviceToHost));
    if (memcmp(got, host, bytes) != 0) {
        size_t i = 0;
        while (got[i] == ((const unsigned char*)host)[i]) ++i;
        printf("FAIL %s: first difference at byte %zu of %zu\n", what, i, bytes);
        ++failures;
    } else {
        printf("ok   %s (%zu bytes)\n", what, bytes);
    }
    fflush(stdout);
    free(got);
}

int main(void)
{
    hipStream_t stream;
    HIP_OK(hipSetDevice(0));
    HIP_OK(hipStreamCreate(&stream));

    /* ---- weights: fp16 -> int8 blocks of 256 -> fp16, a ragged number of wave tiles ---- */
    {
        const int B = 256, bits = 8;
        const size_t n = (size_t)B * 1237;
        uint16_t* x = (uint16_t*)malloc(n * 2);
        fill_f16(x, n);
        unsigned char* oc = (unsigned char*)malloc(zpp_codes_bytes(n, bits));
        float* os = (float*)malloc(zpp_scales_count(n, B) * sizeof(float));
        uint16_t* oy = (uint16_t*)malloc(n * 2);
        if (oracle_qwz_quantize(x, ZPP_F16, n, B, bits, oc, os) || oracle_qwz_dequantize(oc, os, n, B, bits, ZPP_F16, oy))
            return 4;
        void* dx = dev_from(x, n * 2);
        void* dc = dev_filled(zpp_codes_bytes(n, bits));
        float* ds = (float*)dev_filled(zpp_scales_count(n, B) * sizeof(float));
        void* dy = dev_filled(n * 2);
        ZPP_OKAY(qwz_quantize(dx, ZPP_F16, n, B, bits, dc, ds, stream));
        ZPP_OKAY(qwz_dequantize(dc, ds, n, B, bits, ZPP_F16, dy, stream));
        HIP_OK(hipStreamSynchronize(stream));
        expect_same("qwz_quantize codes", dc, oc, zpp_codes_bytes(n, bits));
        expect_same("qwz_quantize scales", ds, os, zpp_scales_count(n, B) * sizeof(float));
        expect_same("qwz_dequantize fp16", dy, oy, n * 2);
        HIP_OK(hipFree(dx)); HIP_OK(hipFree(dc)); HIP_OK(hipFree(ds)); HIP_OK(hipFree(dy));
        free(x); free(oc); free(os); free(oy);
    }

    /* ---- gradients: X = 3 GPUs per node, Y = 2 nodes, int4 blocks of 512, all six GPUs simulated ---- */
    {
        enum { X = 3, Y = 2, W = X * Y };
        const int B = 512, bits = 4;
        const size_t L = (size_t)B * 5;    /* elements per slice */
        const size_t n = L * W, m = n / X; /* gradient length; elements a GPU receives per peer in hop 1 */
        const size_t cb = zpp_codes_bytes(n, bits), sc = zpp_scales_count(n, B);
        uint16_t* g[W];
        unsigned char* hc[W]; float* hs[W];   /* oracle: reordered codes / scales of each GPU */
        void* dc[W]; float* ds[W];            /* library: the same on the device */
        for (int r = 0; r < W; ++r) {
            g[r] = (uint16_t*)malloc(n * 2);
            fill_f16(g[r], n);
            hc[r] = (unsigned char*)malloc(cb);
            hs[r] = (float*)malloc(sc * sizeof(float));
            if (oracle_qgz_reorder(g[r], ZPP_F16, n, X, Y, 1, B, bits, hc[r], hs[r])) return 4;
            void* dg = dev_from(g[r], n * 2);
            dc[r] = dev_filled(cb);
            ds[r] = (float*)dev_filled(sc * sizeof(float));
            ZPP_OKAY(qgz_reorder(dg, ZPP_F16, n, X, Y, 1, B, bits, dc[r], ds[r], stream));
            HIP_OK(hipStreamSynchronize(stream));
            HIP_OK(hipFree(dg));
        }
        expect_same("qgz_reorder codes (GPU 0)", dc[0], hc[0], cb);
        expect_same("qgz_reorder scales (GPU 5)", ds[5], hs[5], sc * sizeof(float));

        /* hop 1: GPU (node y, local j) sums group j of the X GPUs of node y */
        const size_t mcb = zpp_codes_bytes(m, bits), msc = zpp_scales_count(m, B);
        unsigned char* h1c[W]; float* h1s[W];
        void* d1c[W]; float* d1s[W];
        for (int y = 0; y < Y; ++y)
            for (int j = 0; j < X; ++j) {
                const int me = y * X + j;
                const void* hin_c[X]; const float* hin_s[X];
                const void* din_c[X]; const float* din_s[X];
                for (int k = 0; k < X; ++k) {
                    const int peer = y * X + k;
                    hin_c[k] = hc[peer] + (size_t)j * mcb;
                    hin_s[k] = hs[peer] + (size_t)j * msc;
                    din_c[k] = (const unsigned char*)dc[peer] + (size_t)j * mcb;
                    din_s[k] = ds[peer] + (size_t)j * msc;
                }
                h1c[me] = (unsigned char*)malloc(mcb);
                h1s[me] = (float*)malloc(msc * sizeof(float));
                if (oracle_qgz_intra_reduce(hin_c, hin_s, X, m, B, bits, h1c[me], h1s[me])) return 4;
                d1c[me] = dev_filled(mcb);
                d1s[me] = (float*)dev_filled(msc * sizeof(float));
                ZPP_OKAY(qgz_intra_reduce(din_c, din_s, X, m, B, bits, d1c[me], d1s[me], stream));
            }
        HIP_OK(hipStreamSynchronize(stream));
        expect_same("qgz_intra_reduce codes (node 1, local 2)", d1c[5], h1c[5], mcb);
        expect_same("qgz_intra_reduce scales (node 0, local 1)", d1s[1], h1s[1], msc * sizeof(float));

        /* hop 2: GPU (node y, local j) sums slice y of the Y GPUs with local index j, divides by W */
        const size_t lcb = zpp_codes_bytes(L, bits), lsc = zpp_scales_count(L, B);
        for (int y = 0; y < Y; ++y)
            for (int j = 0; j < X; ++j) {
                const void* hin_c[Y]; const float* hin_s[Y];
                const void* din_c[Y]; const float* din_s[Y];
                for (int i = 0; i < Y; ++i) {
                    const int peer = i * X + j;
                    hin_c[i] = h1c[peer] + (size_t)y * lcb;
                    hin_s[i] = h1s[peer] + (size_t)y * lsc;
                    din_c[i] = (const unsigned char*)d1c[peer] + (size_t)y * lcb;
                    din_s[i] = d1s[peer] + (size_t)y * lsc;
                }
                float* ho = (float*)malloc(L * sizeof(float));
                if (oracle_qgz_inter_reduce(hin_c, hin_s, Y, L, B, bits, (float)W, ho)) return 4;
                float* dout = (float*)dev_filled(L * sizeof(float));
                ZPP_OKAY(qgz_inter_reduce(din_c, din_s, Y, L, B, bits, (float)W, dout, stream));
                HIP_OK(hipStreamSynchronize(stream));
                char what[96];
                snprintf(what, sizeof what, "qgz_inter_reduce partition of GPU (node %d, local %d)", y, j);
                expect_same(what, dout, ho, L * sizeof(float));
                /* the partition this GPU ends with is slice y*X + j of the original gradient order */
                if (zpp_reorder_source_slice((long long)j * Y + y, X, Y, 1) != (long long)y * X + j) {
                    printf("FAIL slice bookkeeping for (node %d, local %d)\n", y, j);
                    ++failures;
                }
                HIP_OK(hipFree(dout));
                free(ho);
            }
        for (int r = 0; r < W; ++r) {
            HIP_OK(hipFree(dc[r])); HIP_OK(hipFree(ds[r])); HIP_OK(hipFree(d1c[r])); HIP_OK(hipFree(d1s[r]));
            free(g[r]); free(hc[r]); free(hs[r]); free(h1c[r]); free(h1s[r]);
        }
    }

    /* ---- error behaviour: bad arguments come back as codes, nothing is launched ---- */
    if (qwz_quantize(NULL, ZPP_F16, 256, 256, 8, NULL, NULL, stream) != ZPP_EINVAL) {
        printf("FAIL null pointers not rejected\n");
        ++failures;
    }
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipStreamDestroy(stream));
    printf(failures ? "FAILED (%d)\n" : "ALL EQUAL\n", failures);
    return failures ? 1 : 0;
}
