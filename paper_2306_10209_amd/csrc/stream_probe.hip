// stream_probe: what plain streaming kernels reach on this GPU, so that the library's
// kernels can be read against what the memory system gives rather than only against the
// published peak.  A measurement tool, not part of the library: nothing in the library
// calls it.  All kernels move 16 bytes per lane and access; U = accesses per thread.
//
//   read / write / copy        : one direction or both, non-temporal or plain accesses
//   copy, XCD runs             : workgroup b works on tile ((r / 64) * 8 + b % 8) * 64 + r % 64
//                                with r = b / 8, i.e. each XCD streams runs of 64 tiles
//   copy, grid-stride          : a fixed grid loops over the buffer
//   read 1 : write 2           : the dequantizer's traffic mix (8 B in, 16 B out per lane)
//                                in a few lane layouts
//
// Buffers are fixed powers of two and every grid covers its buffer exactly, so no access
// needs a bounds check.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <vector>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define HIP_OK(call)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            fprintf(stderr, "%s:%d: %s -> %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_)); \
            exit(2);                                                                          \
        }                                                                                     \
    } while (0)

constexpr int kThreads = 256;
constexpr uint64_t kBytes = 1ull << 31;       // per buffer
constexpr uint64_t kVecs = kBytes / 16;       // 16-byte vectors per buffer (2^27)

template <bool NT, class T>
__device__ __forceinline__ T ld(const T* p) { return NT ? __builtin_nontemporal_load(p) : *p; }
template <bool NT, class T>
__device__ __forceinline__ void st(T v, T* p)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// grid = kVecs / (256 * U)
template <int U, bool NT>
__global__ __launch_bounds__(kThreads) void k_read(const u32x4* __restrict__ s, uint32_t* __restrict__ sink)
{
    const uint64_t i0 = (uint64_t)blockIdx.x * kThreads * U + threadIdx.x;
    uint32_t acc = 0;
#pragma unroll
    for (int k = 0; k < U; ++k) {
        const u32x4 v = ld<NT>(s + i0 + (uint64_t)k * kThreads);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345678u) sink[threadIdx.x] = acc;  // never true for the fill pattern; keeps the loads
}

template <int U, bool NT>
__global__ __launch_bounds__(kThreads) void k_write(u32x4* __restrict__ d)
{
    const uint64_t i0 = (uint64_t)blockIdx.x * kThreads * U + threadIdx.x;
    const u32x4 v = {1u, 2u, 3u, (uint32_t)threadIdx.x};
#pragma unroll
    for (int k = 0; k < U; ++k) st<NT>(v, d + i0 + (uint64_t)k * kThreads);
}

// XCD_RUNS: see the header; needs gridDim.x to be a multiple of 512
template <int U, bool NT, bool XCD_RUNS>
__global__ __launch_bounds__(kThreads) void k_copy(const u32x4* __restrict__ s, u32x4* __restrict__ d)
{
    uint32_t tile = blockIdx.x;
    if (XCD_RUNS) {
        const uint32_t x = tile & 7u, r = tile >> 3;
        tile = ((r >> 6) * 8u + x) * 64u + (r & 63u);
    }
    const uint64_t i0 = (uint64_t)tile * kThreads * U + threadIdx.x;
    u32x4 v[U];
#pragma unroll
    for (int k = 0; k < U; ++k) v[k] = ld<NT>(s + i0 + (uint64_t)k * kThreads);
#pragma unroll
    for (int k = 0; k < U; ++k) st<NT>(v[k], d + i0 + (uint64_t)k * kThreads);
}

// any grid whose thread count * U divides kVecs
template <int U>
__global__ __launch_bounds__(kThreads) void k_copy_stride(const u32x4* __restrict__ s, u32x4* __restrict__ d)
{
    const uint64_t stride = (uint64_t)gridDim.x * kThreads * U;
    for (uint64_t i0 = (uint64_t)blockIdx.x * kThreads * U + threadIdx.x; i0 < kVecs; i0 += stride) {
        u32x4 v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) v[k] = ld<true>(s + i0 + (uint64_t)k * kThreads);
#pragma unroll
        for (int k = 0; k < U; ++k) st<true>(v[k], d + i0 + (uint64_t)k * kThreads);
    }
}

// read 1 : write 2.  The source is the first half of a buffer (1 GiB), the destination a
// whole one (2 GiB).
// wave-contiguous: a lane reads 8 B and writes 16 B, V steps per wave (the dequantizer's layout)
template <int V>
__global__ __launch_bounds__(kThreads) void k_mix_wave(const u32x2* __restrict__ s, u32x4* __restrict__ d)
{
    const uint64_t w = (uint64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const uint64_t i = (w * V + k) * 64 + lane;
        const u32x2 a = ld<true>(s + i);
        const u32x4 o = {a.x, a.y, a.x ^ 1u, a.y ^ 1u};
        st<true>(o, d + i);
    }
}
// lane-contiguous: a lane reads 16 B and writes the 32 B that follow each other
__global__ __launch_bounds__(kThreads) void k_mix_lane(const u32x4* __restrict__ s, u32x4* __restrict__ d)
{
    const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    const u32x4 a = ld<true>(s + i);
    const u32x4 o1 = {a.x, a.y, a.x ^ 1u, a.y ^ 1u}, o2 = {a.z, a.w, a.z ^ 1u, a.w ^ 1u};
    st<true>(o1, d + 2 * i);
    st<true>(o2, d + 2 * i + 1);
}
// narrow: a lane reads 4 B and writes 8 B
__global__ __launch_bounds__(kThreads) void k_mix_narrow(const uint32_t* __restrict__ s, u32x2* __restrict__ d)
{
    const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    const uint32_t a = ld<true>(s + i);
    const u32x2 o = {a, a ^ 1u};
    st<true>(o, d + i);
}

template <class F>
static float median_ms(F launch, int reps = 9)
{
    hipEvent_t a, b;
    HIP_OK(hipEventCreate(&a));
    HIP_OK(hipEventCreate(&b));
    launch();
    launch();
    std::vector<float> t;
    for (int i = 0; i < reps; ++i) {
        HIP_OK(hipEventRecord(a, 0));
        launch();
        HIP_OK(hipEventRecord(b, 0));
        HIP_OK(hipEventSynchronize(b));
        float ms = 0.0f;
        HIP_OK(hipEventElapsedTime(&ms, a, b));
        t.push_back(ms);
    }
    HIP_OK(hipGetLastError());
    HIP_OK(hipEventDestroy(a));
    HIP_OK(hipEventDestroy(b));
    std::sort(t.begin(), t.end());
    return t[t.size() / 2];
}

static void report(const char* name, float ms, double bytes)
{
    const double gbs = bytes / ms / 1e6;
    printf("%-52s %8.1f us %8.0f GB/s %6.1f %%\n", name, ms * 1e3, gbs, gbs / 80.0);
    fflush(stdout);
}

int main()
{
    u32x4 *s = nullptr, *d = nullptr;
    HIP_OK(hipSetDevice(0));
    HIP_OK(hipMalloc(&s, kBytes));
    HIP_OK(hipMalloc(&d, kBytes));
    HIP_OK(hipMemset(s, 1, kBytes));
    HIP_OK(hipMemset(d, 2, kBytes));
    HIP_OK(hipDeviceSynchronize());
    printf("stream_probe: 2 GiB buffers, 16 B per lane and access, 256-thread workgroups, median of 9 launches\n");
    printf("%-52s %11s %13s %8s\n", "kernel", "time", "bandwidth", "of 8TB/s");
    const double one = (double)kBytes, both = 2.0 * kBytes;
#define GRID(U) dim3((unsigned)(kVecs / ((uint64_t)kThreads * (U))))
    report("read, U=2, non-temporal", median_ms([&] { k_read<2, true><<<GRID(2), kThreads>>>(s, (uint32_t*)d); }), one);
    report("read, U=4, non-temporal", median_ms([&] { k_read<4, true><<<GRID(4), kThreads>>>(s, (uint32_t*)d); }), one);
    report("read, U=4, plain", median_ms([&] { k_read<4, false><<<GRID(4), kThreads>>>(s, (uint32_t*)d); }), one);
    report("write, U=1, non-temporal", median_ms([&] { k_write<1, true><<<GRID(1), kThreads>>>(d); }), one);
    report("write, U=4, non-temporal", median_ms([&] { k_write<4, true><<<GRID(4), kThreads>>>(d); }), one);
    report("write, U=4, plain", median_ms([&] { k_write<4, false><<<GRID(4), kThreads>>>(d); }), one);
    report("copy, U=1, non-temporal", median_ms([&] { k_copy<1, true, false><<<GRID(1), kThreads>>>(s, d); }), both);
    report("copy, U=2, non-temporal", median_ms([&] { k_copy<2, true, false><<<GRID(2), kThreads>>>(s, d); }), both);
    report("copy, U=4, non-temporal", median_ms([&] { k_copy<4, true, false><<<GRID(4), kThreads>>>(s, d); }), both);
    report("copy, U=8, non-temporal", median_ms([&] { k_copy<8, true, false><<<GRID(8), kThreads>>>(s, d); }), both);
    report("copy, U=1, plain", median_ms([&] { k_copy<1, false, false><<<GRID(1), kThreads>>>(s, d); }), both);
    report("copy, U=4, plain", median_ms([&] { k_copy<4, false, false><<<GRID(4), kThreads>>>(s, d); }), both);
    report("copy, U=1, non-temporal, XCD runs of 64 tiles", median_ms([&] { k_copy<1, true, true><<<GRID(1), kThreads>>>(s, d); }), both);
    report("copy, U=2, non-temporal, XCD runs of 64 tiles", median_ms([&] { k_copy<2, true, true><<<GRID(2), kThreads>>>(s, d); }), both);
    report("copy, U=4, grid-stride loop, 2048 workgroups", median_ms([&] { k_copy_stride<4><<<2048, kThreads>>>(s, d); }), both);
    report("copy, U=4, grid-stride loop, 8192 workgroups", median_ms([&] { k_copy_stride<4><<<8192, kThreads>>>(s, d); }), both);
    report("hipMemcpyAsync device to device", median_ms([&] { HIP_OK(hipMemcpyAsync(d, s, kBytes, hipMemcpyDeviceToDevice, 0)); }), both);
    // read 1 GiB : write 2 GiB
    const double mix = 1.5 * kBytes;
    const uint64_t n8 = kBytes / 2 / 8, n16 = kBytes / 2 / 16, n4 = kBytes / 2 / 4;
    report("read 1 : write 2, lane 8 B -> 16 B, 1 step per wave", median_ms([&] { k_mix_wave<1><<<(unsigned)(n8 / 256), kThreads>>>((const u32x2*)s, d); }), mix);
    report("read 1 : write 2, lane 8 B -> 16 B, 2 steps per wave", median_ms([&] { k_mix_wave<2><<<(unsigned)(n8 / 512), kThreads>>>((const u32x2*)s, d); }), mix);
    report("read 1 : write 2, lane 8 B -> 16 B, 4 steps per wave", median_ms([&] { k_mix_wave<4><<<(unsigned)(n8 / 1024), kThreads>>>((const u32x2*)s, d); }), mix);
    report("read 1 : write 2, lane 16 B -> 32 B contiguous", median_ms([&] { k_mix_lane<<<(unsigned)(n16 / 256), kThreads>>>(s, d); }), mix);
    report("read 1 : write 2, lane 4 B -> 8 B", median_ms([&] { k_mix_narrow<<<(unsigned)(n4 / 256), kThreads>>>((const uint32_t*)s, (u32x2*)d); }), mix);
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipFree(s));
    HIP_OK(hipFree(d));
    return 0;
}
