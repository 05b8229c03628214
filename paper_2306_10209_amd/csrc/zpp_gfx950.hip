// libzpp_gfx950: HIP kernels for AMD MI355X (gfx950, wave64) of the compute that
// ZeRO++ (arxiv 2306.10209) wraps around its collectives, and their C ABI
// (include/zpp.h).  Everything here is streaming work bound by HBM bandwidth or
// by plain vector ALU issue, so there is no matrix-core code: lanes move 16-byte
// vectors, block maxima are folded with DPP / swizzle lane exchanges, and codes
// are packed in registers before a single coalesced store.
//
// Arithmetic contract (see zpp.h): fp32, one rounding per operation, built with
// -ffp-contract=off.  Where a fused multiply-add appears below it is written
// explicitly and computes a single correctly rounded product (the addend only
// removes a bias exactly), so results stay bit-identical to the plain formulas.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "zpp.h"
#include "zpp_diagnostics.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Tile shapes (all measured on MI355X).
//
// Loads per lane and tile, i.e. a wave's tile is 512 * V elements.  Best: two for int8
// output and for dequantize, four for int4 output, whose stores are narrower.
constexpr int kQuantV8 = 2;
constexpr int kQuantV4 = 4;
constexpr int kDeqV = 2;

constexpr int kWave = 64;
constexpr int kWavesPerWG = 4;
constexpr int kThreads = kWave * kWavesPerWG;
constexpr float kTiny = 0x1p-100f;  // blocks with a smaller maximum are coded as all zero

// Streaming accesses: every byte is touched once, so loads and stores carry the
// non-temporal hint (measured: +5 % on loads, +2 % on stores against plain accesses;
// wider-scope write-through store policies gave nothing further in these kernels).
template <class T>
__device__ __forceinline__ T ld_stream(const T* p)
{
    return __builtin_nontemporal_load(p);
}
template <class T>
__device__ __forceinline__ void st_stream(T v, T* p)
{
    __builtin_nontemporal_store(v, p);
}

// Workgroups are handed to the 8 XCDs round-robin by their index.  For large grids
// the quantize and dequantize kernels remap the index so that each XCD works through
// runs of 2^kXcdShift consecutive tiles (measured 2-4 % faster than interleaving
// single tiles over the XCDs).  The grid is then padded to a multiple of 8 runs and
// surplus groups exit at once; small grids keep the plain order (shift < 0).
constexpr int kXcdShift = 6;
constexpr uint64_t kXcdMinGrid = 16ull * 8ull << kXcdShift;

__device__ __forceinline__ uint64_t logical_block(int xcd_shift)
{
    const uint32_t b = blockIdx.x;
    if (xcd_shift < 0) return b;
    const uint32_t x = b & 7u, r = b >> 3;
    return ((((uint64_t)(r >> xcd_shift) << 3) + x) << xcd_shift) + (r & ((1u << xcd_shift) - 1u));
}

// grid size and remap shift for `groups` workgroups of real work
inline uint64_t plan_grid(uint64_t groups, int& xcd_shift)
{
    xcd_shift = -1;
    if (groups < kXcdMinGrid) return groups;
    xcd_shift = kXcdShift;
    const uint64_t q = 8ull << kXcdShift;
    return (groups + q - 1) / q * q;
}

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// ---------------------------------------------------------------------------
// lane exchanges for the per-block maximum
// ---------------------------------------------------------------------------

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    int i = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(i, i, CTRL, 0xf, 0xf, false));
}

// Maximum over aligned groups of G consecutive lanes (G a power of two), left in
// every lane of the group.  Values are non-negative finite floats.
template <int G>
__device__ __forceinline__ float group_max(float v)
{
    if (G >= 2) v = fmaxf(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
    if (G >= 4) v = fmaxf(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
    if (G >= 8) v = fmaxf(v, dpp_mov<0x141>(v));   // row_half_mirror
    if (G >= 16) v = fmaxf(v, dpp_mov<0x140>(v));  // row_mirror
    if (G >= 32) {                                 // ds_swizzle: lane ^ 16 inside each half wave
        int i = __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F);
        v = fmaxf(v, __builtin_bit_cast(float, i));
    }
    if (G >= 64) v = fmaxf(v, __shfl_xor(v, 32, 64));
    return v;
}

// ---------------------------------------------------------------------------
// storage types
// ---------------------------------------------------------------------------

// Two packed 16-bit values of a dword -> fp32 (exact).
template <int DT>
__device__ __forceinline__ void widen2(uint32_t w, float& lo, float& hi)
{
    if (DT == ZPP_F16) {
        lo = (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
        hi = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
    } else {
        lo = as_f32(w << 16);
        hi = as_f32(w & 0xffff0000u);
    }
}

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = as_u32(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <int DT>
__device__ __forceinline__ uint32_t narrow2(float lo, float hi)
{
    if (DT == ZPP_F16) {
        uint32_t a = __builtin_bit_cast(uint16_t, (_Float16)lo);
        uint32_t b = __builtin_bit_cast(uint16_t, (_Float16)hi);
        return a | (b << 16);
    } else {
        return bf16_rne(lo) | (bf16_rne(hi) << 16);
    }
}

// Eight consecutive elements of a DT tensor starting at element index `e` (a
// multiple of 8), widened to fp32.
template <int DT>
__device__ __forceinline__ void load8(const void* __restrict__ base, uint64_t e, float (&f)[8])
{
    if (DT == ZPP_F32) {
        const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + e);
        f32x4 a = ld_stream(p), b = ld_stream(p + 1);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
        f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    } else {
        const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + e);
        u32x4 w = ld_stream(p);
        widen2<DT>(w.x, f[0], f[1]);
        widen2<DT>(w.y, f[2], f[3]);
        widen2<DT>(w.z, f[4], f[5]);
        widen2<DT>(w.w, f[6], f[7]);
    }
}

// fp32 tensors: a lane's 8 consecutive elements are 32 bytes, so a wave-wide 16-byte access by
// "lane l takes elements 8l.." touches every other 16 bytes of 2 KB.  Instead every load or
// store instruction moves one contiguous KB (lane l: 16-byte chunk l, then chunk 64 + l, of
// the wave's run of 512 elements) and the chunks change lanes through 2 KB of LDS.
//
// Slot of chunk c in that buffer: rows of 8 chunks, the column XORed with the row, so that
// "lane l touches chunk l" and "lane l touches chunk 2l (or 2l + 1)" both spread over all banks.
__device__ __forceinline__ uint32_t turn_slot(uint32_t c) { return (c & ~7u) | ((c ^ (c >> 3)) & 7u); }

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The two chunks lane `lane` fetches of the run of `valid` (<= 512, a multiple of 8) fp32
// elements at `run`; chunks past the end read as zero.
__device__ __forceinline__ void load_run_f32(const float* __restrict__ run, uint32_t valid, int lane, f32x4& a, f32x4& b)
{
    const f32x4* p = reinterpret_cast<const f32x4*>(run);
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    a = (uint32_t)lane * 4u < valid ? ld_stream(p + lane) : zero;
    b = (uint32_t)(kWave + lane) * 4u < valid ? ld_stream(p + kWave + lane) : zero;
}

// f = elements 8*lane .. 8*lane+7 of the run whose chunks lane and 64+lane are a and b in every lane
__device__ __forceinline__ void turn_to_lanes(const f32x4& a, const f32x4& b, int lane, f32x4* __restrict__ turn, float (&f)[8])
{
    turn[turn_slot((uint32_t)lane)] = a;
    turn[turn_slot((uint32_t)(kWave + lane))] = b;
    wave_lds_fence();
    const f32x4 u = turn[turn_slot(2u * lane)], v = turn[turn_slot(2u * lane + 1u)];
    wave_lds_fence();
    f[0] = u.x; f[1] = u.y; f[2] = u.z; f[3] = u.w;
    f[4] = v.x; f[5] = v.y; f[6] = v.z; f[7] = v.w;
}

// The reverse: d = elements 8*lane .. 8*lane+7 of a run of `valid` fp32 elements at `run`, stored
// as two contiguous KB per wave.
__device__ __forceinline__ void store_run_f32(const float (&d)[8], float* __restrict__ run, uint32_t valid, int lane,
                                              f32x4* __restrict__ turn)
{
    const f32x4 u = {d[0], d[1], d[2], d[3]}, v = {d[4], d[5], d[6], d[7]};
    turn[turn_slot(2u * lane)] = u;
    turn[turn_slot(2u * lane + 1u)] = v;
    wave_lds_fence();
    const f32x4 a = turn[turn_slot((uint32_t)lane)], b = turn[turn_slot((uint32_t)(kWave + lane))];
    wave_lds_fence();
    f32x4* o = reinterpret_cast<f32x4*>(run);
    if ((uint32_t)lane * 4u < valid) st_stream(a, o + lane);
    if ((uint32_t)(kWave + lane) * 4u < valid) st_stream(b, o + kWave + lane);
}

// ---------------------------------------------------------------------------
// block codec pieces
// ---------------------------------------------------------------------------

template <int BITS>
struct Q {
    static constexpr float qmax = (float)((1 << (BITS - 1)) - 1);
};

// The two IEEE divisions of a block, a/qmax and qmax/a, by short fused sequences
// that give the correctly rounded quotients for 2^-100 <= a < 2^100:
//   a/qmax : y = RN(1/qmax) (a constant); q = a*y; r = fma(-qmax, q, a); q' = fma(r, y, q)
//   qmax/a : y = rcp(a) refined once (e = fma(-a, y, 1); y = fma(e, y, y));
//            q = qmax*y; r = fma(-a, q, qmax); q' = fma(r, y, q)
// Both are invariant under scaling a by powers of two inside that range, and they
// were compared with the division instruction sequence for all 2^23 mantissas
// (zpp_selfcheck_block_scale does that on the device it runs on).  Outside the
// range the plain divisions are used.  About 9 operations instead of 25 per block.
template <int BITS>
__device__ __forceinline__ void exact_quotients(float a, float& a_over_qmax, float& qmax_over_a)
{
    constexpr float qm = Q<BITS>::qmax;
    constexpr float y = 1.0f / qm;
    const float q0 = a * y;
    const float r0 = __builtin_fmaf(-qm, q0, a);
    a_over_qmax = __builtin_fmaf(r0, y, q0);
    const float z0 = __builtin_amdgcn_rcpf(a);
    const float e = __builtin_fmaf(-a, z0, 1.0f);
    const float z1 = __builtin_fmaf(e, z0, z0);
    const float p0 = qm * z1;
    const float r1 = __builtin_fmaf(-a, p0, qm);
    qmax_over_a = __builtin_fmaf(r1, z1, p0);
}

// scale and encode multiplier of a block whose maximum magnitude is `a`
template <int BITS>
__device__ __forceinline__ void block_scale(float a, float& scale, float& inv)
{
    if (a < kTiny) {
        scale = 0.0f;
        inv = 0.0f;  // every product is +-0 -> code 0
    } else if (a < 0x1p100f) {
        exact_quotients<BITS>(a, scale, inv);
    } else {
        scale = a / Q<BITS>::qmax;
        inv = Q<BITS>::qmax / a;
    }
}

// Self-check of exact_quotients against the plain divisions: all 2^23 mantissas at one
// exponent; counts[0] / counts[1] += mismatches of a/qmax / qmax/a.
template <int BITS>
__global__ __launch_bounds__(kThreads) void k_selfcheck_block_scale(uint32_t exponent_bits,
                                                                    unsigned long long* __restrict__ counts)
{
    const uint32_t m = blockIdx.x * kThreads + threadIdx.x;
    const float a = as_f32((exponent_bits << 23) | m);
    float s1, i1;
    exact_quotients<BITS>(a, s1, i1);
    const float s2 = a / Q<BITS>::qmax, i2 = Q<BITS>::qmax / a;
    if (as_u32(s1) != as_u32(s2)) atomicAdd(counts, 1ull);
    if (as_u32(i1) != as_u32(i2)) atomicAdd(counts + 1, 1ull);
}

// Code of one value: roundeven(v * inv).  Adding 1.5*2^23 + bias rounds the product
// to an integer with the adder's own round-to-nearest-even and leaves code + bias
// in the low mantissa bits (bits = 0x4B400000 + bias + code).  |v*inv| <= qmax + 2^-17
// for finite input, so no clamp is needed.  With bias = qmax + 1 the low field is the
// non-negative u = code + bias, which lets several codes be packed with shift-adds:
// the upper bits of every term add up to a constant (mod 2^32) that is taken off at
// the end, and flipping each field's top bit turns u into the two's-complement code.
template <int BITS>
__device__ __forceinline__ uint32_t biased_code_bits(float v, float inv)
{
    const float t = v * inv;
    return as_u32(t + (12582912.0f + (float)(1 << (BITS - 1))));
}

// FIELDS codes of BITS bits each -> one dword (FIELDS * BITS == 32)
template <int BITS>
__device__ __forceinline__ uint32_t pack_dword(const float* __restrict__ f, float inv)
{
    constexpr int FIELDS = 32 / BITS;
    uint32_t acc = biased_code_bits<BITS>(f[FIELDS - 1], inv);
#pragma unroll
    for (int i = FIELDS - 2; i >= 0; --i) acc = (acc << BITS) + biased_code_bits<BITS>(f[i], inv);
    constexpr uint32_t ones = BITS == 4 ? 0x11111111u : 0x01010101u;  // sum of 2^(BITS*i)
    constexpr uint32_t upper = 0x4B400000u * ones;                    // what the exponent bits added up to
    constexpr uint32_t flip = ones << (BITS - 1);
    return (acc - upper) ^ flip;
}

// eight codes -> packed storage
template <int BITS>
__device__ __forceinline__ void store_codes8(uint8_t* __restrict__ codes, uint64_t e, const float (&f)[8], float inv)
{
    if (BITS == 8) {
        u32x2 o;
        o.x = pack_dword<8>(f, inv);
        o.y = pack_dword<8>(f + 4, inv);
        st_stream(o, reinterpret_cast<u32x2*>(codes + e));
    } else {
        st_stream(pack_dword<4>(f, inv), reinterpret_cast<uint32_t*>(codes + (e >> 1)));
    }
}

__device__ __forceinline__ float absmax8(const float (&f)[8])
{
    float m = fabsf(f[0]);
#pragma unroll
    for (int i = 1; i < 8; ++i) m = fmaxf(m, fabsf(f[i]));
    return m;
}

// Sec. 3.3.3 Eq. (2) / Sec. 4.1 Alg. 2, gather form: original slice at new position p.
__device__ __host__ __forceinline__ uint64_t source_slice(uint64_t p, uint32_t X, uint32_t Y)
{
    const uint64_t T = (uint64_t)X * Y;
    const uint64_t st = p / T, w = p % T;
    const uint64_t j = w / Y, i = w % Y;
    return st * T + i * X + j;
}

// Unsigned 32-bit division by a divisor that is fixed for a whole launch: one
// multiply-high, two shifts and two adds instead of the long division sequence
// (round-up multiplier method: with l = ceil(log2 d), m = floor(2^32 (2^l - d) / d) + 1,
// x / d = (t + ((x - t) >> min(l, 1))) >> max(l - 1, 0) where t = mulhi(m, x)).
// Every wave maps its index to (slice, tile) and the slice to its source with these.
struct FastDiv {
    uint32_t d, mul, sh1, sh2;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    FastDiv f;
    f.d = d;
    f.mul = (uint32_t)((((1ull << l) - d) << 32) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l > 1 ? l - 1 : 0;
    return f;
}

__device__ __host__ __forceinline__ uint32_t fast_div(uint32_t x, const FastDiv& f)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t t = __umulhi(x, f.mul);
#else
    const uint32_t t = (uint32_t)(((uint64_t)x * f.mul) >> 32);
#endif
    return (t + ((x - t) >> f.sh1)) >> f.sh2;
}

// source_slice for indices below 2^32, with the divisions by T = X*Y and by Y prepared
__device__ __host__ __forceinline__ uint64_t source_slice32(uint32_t p, uint32_t X, const FastDiv& byT,
                                                            const FastDiv& byY)
{
    const uint32_t st = fast_div(p, byT), w = p - st * byT.d;
    const uint32_t j = fast_div(w, byY), i = w - j * byY.d;
    return (uint64_t)st * byT.d + (uint64_t)i * X + j;
}

// ---------------------------------------------------------------------------
// quantize (qwz_quantize, qgz_reorder): power-of-two block sizes
// ---------------------------------------------------------------------------
//
// A wave owns a tile of 512*V consecutive elements of one output slice; load k of
// lane l covers elements (k*64 + l)*8 .. +8, so every wave-wide load or store is
// one contiguous run.  Blocks of >= 512 elements span B/512 loads (maximum folded
// across registers, then across the wave); smaller blocks sit inside one load, B/8
// lanes each.  The un-quantized values of a block stay in registers between the
// maximum and the encode (Sec. 4.2), so the tensor is read exactly once.

// One tile.  FULL: the whole tile lies inside the slice, so no lane is masked;
// otherwise lanes past the end of the slice are masked.  DEEP = false: a wave waits
// for each load before it issues the next; in a launch of very many residency rounds the
// other waves of the SIMD keep the memory system busy, and more bytes in flight only
// queue up (-3 to -7 % with all of a tile's loads outstanding).  DEEP = true: all of the
// tile's loads are issued at once; in a shorter launch the chip is not yet (or no longer)
// full for a good part of it, and a wave's own chain of load latencies is what counts.
template <int DT, int BITS, int LOG2B, int V, bool FULL, bool DEEP>
__device__ __forceinline__ void quantize_tile(const void* __restrict__ x, uint8_t* __restrict__ codes,
                                              float* __restrict__ scales, uint64_t in_base, uint64_t out_base,
                                              uint64_t rem, int lane, f32x4* __restrict__ turn /* fp32 input: 2 KB of LDS */)
{
    constexpr int B = 1 << LOG2B;
    float f[V][8];
    bool ok[V];
    if constexpr (DT == ZPP_F32) {
        f32x4 qa[V], qb[V];
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const uint32_t first = (uint32_t)k * 512u;  // of this step's run
            const uint32_t valid = FULL ? 512u : (rem > first ? (rem - first < 512 ? (uint32_t)(rem - first) : 512u) : 0u);
            ok[k] = FULL || (uint32_t)(k * kWave + lane) * 8u < rem;
            load_run_f32(static_cast<const float*>(x) + in_base + first, valid, lane, qa[k], qb[k]);
            if (!DEEP) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        }
#pragma unroll
        for (int k = 0; k < V; ++k) turn_to_lanes(qa[k], qb[k], lane, turn, f[k]);
    } else {
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const uint32_t off = (uint32_t)(k * kWave + lane) * 8u;
            ok[k] = FULL || off < rem;
            if (ok[k]) {
                load8<DT>(x, in_base + off, f[k]);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) f[k][i] = 0.0f;
            }
            if (!DEEP) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        }
    }

    if constexpr (B >= 512) {
        constexpr int LPB = B / 512 > 0 ? B / 512 : 1;  // loads per block
        static_assert(B < 512 || V % LPB == 0, "tile must hold whole blocks");
#pragma unroll
        for (int b0 = 0; b0 < V; b0 += LPB) {
            float a = absmax8(f[b0]);
#pragma unroll
            for (int k = 1; k < LPB; ++k) a = fmaxf(a, absmax8(f[b0 + k]));
            a = group_max<kWave>(a);
            float scale, inv;
            block_scale<BITS>(a, scale, inv);
            if (lane == 0 && ok[b0]) scales[(out_base + (uint64_t)b0 * 512) >> LOG2B] = scale;
#pragma unroll
            for (int k = 0; k < LPB; ++k) {
                const uint32_t off = (uint32_t)((b0 + k) * kWave + lane) * 8u;
                if (ok[b0 + k]) store_codes8<BITS>(codes, out_base + off, f[b0 + k], inv);
            }
        }
    } else {
        constexpr int G = B / 8 > 0 ? B / 8 : 1;  // lanes per block
#pragma unroll
        for (int k = 0; k < V; ++k) {
            float a = group_max<(G < kWave ? G : kWave)>(absmax8(f[k]));
            float scale, inv;
            block_scale<BITS>(a, scale, inv);
            const uint32_t off = (uint32_t)(k * kWave + lane) * 8u;
            if (ok[k]) {
                if ((lane & (G - 1)) == 0) scales[(out_base + off) >> LOG2B] = scale;
                store_codes8<BITS>(codes, out_base + off, f[k], inv);
            }
        }
    }
}

template <int DT, int BITS, int LOG2B, int V, bool DEEP>
__global__ __launch_bounds__(kThreads) void k_quantize(const void* __restrict__ x, uint8_t* __restrict__ codes,
                                                       float* __restrict__ scales, uint64_t L,
                                                       FastDiv by_tiles_per_slice, uint32_t total_tiles,
                                                       uint32_t X, FastDiv byT, FastDiv byY, int xcd_shift)
{
    constexpr int TILE = 512 * V;
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t wid = logical_block(xcd_shift) * kWavesPerWG + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wid >= total_tiles) return;
    const uint32_t p = fast_div((uint32_t)wid, by_tiles_per_slice);
    const uint32_t t = (uint32_t)wid - p * by_tiles_per_slice.d;
    const uint64_t src = (X == 1 || byY.d == 1) ? p : source_slice32(p, X, byT, byY);
    const uint64_t in_base = src * L + (uint64_t)t * TILE;
    const uint64_t out_base = (uint64_t)p * L + (uint64_t)t * TILE;
    const uint64_t rem = L - (uint64_t)t * TILE;  // elements of this slice from the tile start on (>= 1)
    f32x4* turn = nullptr;
    if constexpr (DT == ZPP_F32) {
        __shared__ f32x4 turn_lds[kWavesPerWG][2 * kWave];
        turn = turn_lds[__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)];
    }
    if (rem >= TILE)
        quantize_tile<DT, BITS, LOG2B, V, true, DEEP>(x, codes, scales, in_base, out_base, rem, lane, turn);
    else
        quantize_tile<DT, BITS, LOG2B, V, false, DEEP>(x, codes, scales, in_base, out_base, rem, lane, turn);
}

// Any other block size that is a multiple of 32 (not a power of two): one wave per block.
// The largest block, 4096 elements, is 8 rounds of 64 lanes x 8 elements, so the whole
// block waits in registers between the maximum and the encode, as in the tiled kernel: the
// tensor is read once.  R = 2, 4 or 8 rounds are compiled (fewer registers for smaller
// blocks, so more waves in flight); rounds past the end of the block are skipped (same in
// every lane), in the last round the lanes past its end are masked.
// There are fewer than 2^32 blocks in all (the host refuses more), so the wave maps its block to
// (slice, block in slice) and the slice to its source with the prepared 32-bit divisions.
constexpr int kBlockRounds = 8;

template <int DT, int BITS, int R>
__global__ __launch_bounds__(kThreads) void k_quantize_anyblock(const void* __restrict__ x,
                                                                uint8_t* __restrict__ codes,
                                                                float* __restrict__ scales, uint64_t L,
                                                                uint32_t B, uint64_t total_blocks, uint32_t X,
                                                                uint32_t Y, FastDiv by_blocks_per_slice, FastDiv byT,
                                                                FastDiv byY)
{
    static_assert(R <= kBlockRounds, "a block is at most 8 rounds");
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t ob = (uint64_t)blockIdx.x * kWavesPerWG + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (ob >= total_blocks) return;
    const uint32_t p = fast_div((uint32_t)ob, by_blocks_per_slice);
    const uint32_t r = (uint32_t)ob - p * by_blocks_per_slice.d;
    const uint64_t src = (X == 1 || Y == 1) ? (uint64_t)p : source_slice32(p, X, byT, byY);
    const uint64_t in_base = src * L + (uint64_t)r * B, out_base = ob * B;
    const uint32_t chunks = B / 8;  // 8-element pieces of the block
    float f[R][8];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const uint32_t c = (uint32_t)k * kWave + lane;
        if ((uint32_t)k * kWave < chunks && c < chunks) {
            load8<DT>(x, in_base + c * 8u, f[k]);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) f[k][i] = 0.0f;
        }
    }
    float a = 0.0f;
#pragma unroll
    for (int k = 0; k < R; ++k)
        if ((uint32_t)k * kWave < chunks) a = fmaxf(a, absmax8(f[k]));
    a = group_max<kWave>(a);
    float scale, inv;
    block_scale<BITS>(a, scale, inv);
    if (lane == 0) scales[ob] = scale;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const uint32_t c = (uint32_t)k * kWave + lane;
        if ((uint32_t)k * kWave < chunks && c < chunks) store_codes8<BITS>(codes, out_base + c * 8u, f[k], inv);
    }
}

// ---------------------------------------------------------------------------
// decode helpers
// ---------------------------------------------------------------------------

// signed code i (0..7) of a dword of eight two's-complement nibbles
__device__ __forceinline__ float nibble_f32(uint32_t w, int i)
{
    return (float)((int32_t)(w << (28 - 4 * i)) >> 28);
}
// signed code i (0..3) of a dword of four two's-complement bytes
__device__ __forceinline__ float byte_f32(uint32_t w, int i)
{
    return (float)((int32_t)(w << (24 - 8 * i)) >> 24);
}

// ---------------------------------------------------------------------------
// qwz_dequantize
// ---------------------------------------------------------------------------
//
// Lane l of a wave decodes 8 consecutive elements per step (8 B of int8 codes or
// 4 B of int4 codes in, 16 B of 16-bit values out), V steps per wave with all
// loads issued first.  The writes are two thirds of the traffic, so they get the
// full-width contiguous stores.

// One tile of qwz_dequantize.  Lanes past the end of the tensor are masked; the masked
// form is kept for full tiles too: it issues each 16-byte store as soon as its eight
// values are ready, which measured 2 % faster than an unmasked variant that stored last.
// ONE_BLOCK: the block is a multiple of the tile, so the whole wave shares one scale, which is
// then fetched once through the scalar unit instead of once per lane and step.
template <int ODT, int BITS, int V, bool POW2, bool ONE_BLOCK>
__device__ __forceinline__ void dequantize_tile(const uint8_t* __restrict__ codes, const float* __restrict__ scales,
                                                void* __restrict__ y, uint64_t base, uint64_t rem, uint32_t B,
                                                int log2b, int lane, f32x4* __restrict__ turn /* fp32 output: 2 KB of LDS */)
{
    uint32_t w[V][2];
    float s[V];
    bool ok[V];
    float s_tile = 0.0f;
    if constexpr (ONE_BLOCK) s_tile = scales[base >> log2b];  // base is the same in every lane
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const uint32_t off = (uint32_t)(k * kWave + lane) * 8u;
        ok[k] = off < rem;
        w[k][0] = w[k][1] = 0;
        s[k] = 0.0f;
        if (ok[k]) {
            const uint64_t e = base + off;
            if (BITS == 8) {
                u32x2 v = ld_stream(reinterpret_cast<const u32x2*>(codes + e));
                w[k][0] = v.x;
                w[k][1] = v.y;
            } else {
                w[k][0] = ld_stream(reinterpret_cast<const uint32_t*>(codes + (e >> 1)));
            }
            if constexpr (ONE_BLOCK) {
                s[k] = s_tile;
            } else {
                const uint64_t blk = POW2 ? (e >> log2b) : (e / B);
                s[k] = scales[blk];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < V; ++k) {
        if (ODT == ZPP_F32) {  // the whole wave takes part in the store: leave only when the step's run is empty
            if ((uint64_t)k * 512u >= rem) break;
        } else if (!ok[k]) {
            continue;
        }
        float d[8];  // lanes past the end have zero codes and a zero scale
        if (BITS == 8) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                d[i] = byte_f32(w[k][0], i) * s[k];
                d[4 + i] = byte_f32(w[k][1], i) * s[k];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) d[i] = nibble_f32(w[k][0], i) * s[k];
        }
        const uint64_t e = base + (uint32_t)(k * kWave + lane) * 8u;
        if (ODT == ZPP_F32) {
            const uint64_t first = (uint64_t)k * 512u, left = rem - first;
            store_run_f32(d, static_cast<float*>(y) + base + first, left < 512 ? (uint32_t)left : 512u, lane, turn);
        } else {
            u32x4 o;
            o.x = narrow2<ODT>(d[0], d[1]);
            o.y = narrow2<ODT>(d[2], d[3]);
            o.z = narrow2<ODT>(d[4], d[5]);
            o.w = narrow2<ODT>(d[6], d[7]);
            st_stream(o, reinterpret_cast<u32x4*>(static_cast<uint16_t*>(y) + e));
        }
    }
}

template <int ODT, int BITS, int V, bool POW2, bool ONE_BLOCK>
__global__ __launch_bounds__(kThreads) void k_dequantize(const uint8_t* __restrict__ codes,
                                                         const float* __restrict__ scales,
                                                         void* __restrict__ y, uint64_t n, uint32_t B,
                                                         int log2b /* used when POW2 */, int xcd_shift)
{
    constexpr int TILE = 512 * V;
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t wid = logical_block(xcd_shift) * kWavesPerWG + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t base = wid * TILE;
    if (base >= n) return;
    f32x4* turn = nullptr;
    if constexpr (ODT == ZPP_F32) {
        __shared__ f32x4 turn_lds[kWavesPerWG][2 * kWave];
        turn = turn_lds[__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)];
    }
    dequantize_tile<ODT, BITS, V, POW2, ONE_BLOCK>(codes, scales, y, base, n - base, B, log2b, lane, turn);
}

// ---------------------------------------------------------------------------
// the two reduce stages
// ---------------------------------------------------------------------------

struct PeerTable {
    const uint8_t* codes[ZPP_MAX_PEERS];
    const float* scales[ZPP_MAX_PEERS];
};

// elements a lane holds per vector of NW code dwords (NW = 1, 2 or 4)
template <int BITS, int NW>
struct EPL {
    static constexpr int value = NW * 32 / BITS;
};

template <int NW>
__device__ __forceinline__ void load_words(const uint8_t* __restrict__ p, uint32_t (&w)[NW])
{
    if constexpr (NW == 4) {
        const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(p));
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else if constexpr (NW == 2) {
        const u32x2 v = ld_stream(reinterpret_cast<const u32x2*>(p));
        w[0] = v.x; w[1] = v.y;
    } else {
        w[0] = ld_stream(reinterpret_cast<const uint32_t*>(p));
    }
}

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// The three operands of the exact int4 decode for a scale s with |s| < 2^100:
// s * 2^24, s * 2^20 and -8 * s (power-of-two factors, so all three are exact).
struct Dec4 {
    float lo, hi, bias;
};
__device__ __forceinline__ Dec4 dec4_operands(float s)
{
    Dec4 d;
    d.lo = s * 0x1p24f;
    d.hi = s * 0x1p20f;
    d.bias = s * -8.0f;
    return d;
}
__device__ __forceinline__ bool fused_decode_ok(float s) { return fabsf(s) < 0x1p100f; }

// acc[0..8) (+)= decode(nibble_i of w, s), i = 0..7 (nibble i = bits 4i..4i+3).
//
// decode is float(q)*s with one rounding.  It is computed as a single fused
// multiply-add whose multiplicand is read straight from the code word: after
// flipping each nibble's top bit the nibble holds u = q + 8, and a 16-bit lane
// whose only set bits are such a nibble is, read as binary16, the subnormal
// u*2^-24 (bits 0-3) or u*2^-20 (bits 4-7).  fma(u*2^-24, s*2^24, -8*s) is the
// exact value (u-8)*s = q*s rounded once, because s*2^24, s*2^20 and 8*s are exact.
// The conversion of the binary16 operand happens inside the mixed-precision fma
// instruction.
//
// FIRST: the accumulator is set instead of added to.  The sum starts from +0 and a value
// decoded this way is never -0 (code 0 gives 8s - 8s = +0 for either sign of s, a zero scale
// of either sign gives a sum of two opposite zeros = +0), so 0 + d and d are the same bits
// and the first peer needs neither the zeroing nor the add.
template <bool FIRST>
__device__ __forceinline__ void add_nibbles8(float* __restrict__ acc, uint32_t w, const Dec4& d)
{
    // (x ^ 0x88888888) & mask in one three-input bit operation each
    const uint32_t v = w >> 8;
    const f16x2 a = __builtin_bit_cast(f16x2, __builtin_amdgcn_bitop3_b32(w, 0x88888888u, 0x000F000Fu, 0x28));  // elements 0, 4
    const f16x2 b = __builtin_bit_cast(f16x2, __builtin_amdgcn_bitop3_b32(w, 0x88888888u, 0x00F000F0u, 0x28));  // elements 1, 5
    const f16x2 c = __builtin_bit_cast(f16x2, __builtin_amdgcn_bitop3_b32(v, 0x88888888u, 0x000F000Fu, 0x28));  // elements 2, 6
    const f16x2 e = __builtin_bit_cast(f16x2, __builtin_amdgcn_bitop3_b32(v, 0x88888888u, 0x00F000F0u, 0x28));  // elements 3, 7
    acc[0] = FIRST ? __builtin_fmaf((float)a.x, d.lo, d.bias) : acc[0] + __builtin_fmaf((float)a.x, d.lo, d.bias);
    acc[1] = FIRST ? __builtin_fmaf((float)b.x, d.hi, d.bias) : acc[1] + __builtin_fmaf((float)b.x, d.hi, d.bias);
    acc[2] = FIRST ? __builtin_fmaf((float)c.x, d.lo, d.bias) : acc[2] + __builtin_fmaf((float)c.x, d.lo, d.bias);
    acc[3] = FIRST ? __builtin_fmaf((float)e.x, d.hi, d.bias) : acc[3] + __builtin_fmaf((float)e.x, d.hi, d.bias);
    acc[4] = FIRST ? __builtin_fmaf((float)a.y, d.lo, d.bias) : acc[4] + __builtin_fmaf((float)a.y, d.lo, d.bias);
    acc[5] = FIRST ? __builtin_fmaf((float)b.y, d.hi, d.bias) : acc[5] + __builtin_fmaf((float)b.y, d.hi, d.bias);
    acc[6] = FIRST ? __builtin_fmaf((float)c.y, d.lo, d.bias) : acc[6] + __builtin_fmaf((float)c.y, d.lo, d.bias);
    acc[7] = FIRST ? __builtin_fmaf((float)e.y, d.hi, d.bias) : acc[7] + __builtin_fmaf((float)e.y, d.hi, d.bias);
}

// The same decode for int8 codes: after flipping each byte's top bit the byte holds u = q + 128,
// and a 16-bit lane whose only set bits are its low byte is the binary16 subnormal u*2^-24;
// fma(u*2^-24, s*2^24, -128*s) = q*s rounded once.  Operands for |s| < 2^100:
struct Dec8 {
    float lo, bias;
};
__device__ __forceinline__ Dec8 dec8_operands(float s)
{
    Dec8 d;
    d.lo = s * 0x1p24f;
    d.bias = s * -128.0f;
    return d;
}

// acc[0..4) (+)= decode(byte_i of w, s), i = 0..3.  FIRST as in add_nibbles8 (never -0 either).
template <bool FIRST>
__device__ __forceinline__ void add_bytes4(float* __restrict__ acc, uint32_t w, const Dec8& d)
{
    const f16x2 a = __builtin_bit_cast(f16x2, __builtin_amdgcn_bitop3_b32(w, 0x80808080u, 0x00FF00FFu, 0x28));       // elements 0, 2
    const f16x2 b = __builtin_bit_cast(f16x2, __builtin_amdgcn_bitop3_b32(w >> 8, 0x80808080u, 0x00FF00FFu, 0x28));  // elements 1, 3
    acc[0] = FIRST ? __builtin_fmaf((float)a.x, d.lo, d.bias) : acc[0] + __builtin_fmaf((float)a.x, d.lo, d.bias);
    acc[1] = FIRST ? __builtin_fmaf((float)b.x, d.lo, d.bias) : acc[1] + __builtin_fmaf((float)b.x, d.lo, d.bias);
    acc[2] = FIRST ? __builtin_fmaf((float)a.y, d.lo, d.bias) : acc[2] + __builtin_fmaf((float)a.y, d.lo, d.bias);
    acc[3] = FIRST ? __builtin_fmaf((float)b.y, d.lo, d.bias) : acc[3] + __builtin_fmaf((float)b.y, d.lo, d.bias);
}

// acc[i] (+)= decode(code_i, s) for the codes of NW dwords by the fused decodes above (|s| < 2^100)
template <int BITS, int NW, bool FIRST>
__device__ __forceinline__ void accumulate_fused(float* __restrict__ acc, const uint32_t (&d)[NW], float s)
{
    if constexpr (BITS == 4) {
        const Dec4 op = dec4_operands(s);
#pragma unroll
        for (int j = 0; j < NW; ++j) add_nibbles8<FIRST>(acc + j * 8, d[j], op);
    } else {
        const Dec8 op = dec8_operands(s);
#pragma unroll
        for (int j = 0; j < NW; ++j) add_bytes4<FIRST>(acc + j * 4, d[j], op);
    }
}

// acc[i] (+)= float(code_i) * s for the codes of NW dwords by convert and multiply (any
// scale).  The product can be -0 (code 0 and a negative scale, a negative code and a zero
// scale), so the first peer is added to the +0 the sum starts from.
template <int BITS, int NW, bool FIRST>
__device__ __forceinline__ void accumulate_plain(float (&acc)[(EPL<BITS, NW>::value)], const uint32_t (&d)[NW], float s)
{
    constexpr int F = 32 / BITS;
#pragma unroll
    for (int j = 0; j < NW; ++j)
#pragma unroll
        for (int i = 0; i < F; ++i) {
            const float v = (BITS == 4 ? nibble_f32(d[j], i) : byte_f32(d[j], i)) * s;
            acc[j * F + i] = FIRST ? 0.0f + v : acc[j * F + i] + v;
        }
}

// ---------------------------------------------------------------------------
// reduce stages, any block size: every lane fetches its own scales
// ---------------------------------------------------------------------------

// acc[i] (+)= decode(code_i, s) for the codes of NW dwords
template <int BITS, int NW, bool FIRST>
__device__ __forceinline__ void accumulate(float (&acc)[(EPL<BITS, NW>::value)], const uint32_t (&d)[NW], float s)
{
    if (fused_decode_ok(s)) {
        accumulate_fused<BITS, NW, FIRST>(acc, d, s);
    } else {  // scales so large that they never come from 16-bit gradients
        accumulate_plain<BITS, NW, FIRST>(acc, d, s);
    }
}

template <int NW, int U>
__device__ __forceinline__ void load_group(const PeerTable& P, int k0, uint64_t byte_off, uint64_t blk,
                                           uint32_t (&w)[U][NW], float (&s)[U])
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        load_words<NW>(P.codes[k0 + u] + byte_off, w[u]);
        s[u] = P.scales[k0 + u][blk];
    }
}

// FIRST: w[0] is the very first peer of the sum
template <int BITS, int NW, int U, bool FIRST>
__device__ __forceinline__ void add_group(float (&acc)[(EPL<BITS, NW>::value)], const uint32_t (&w)[U][NW],
                                          const float (&s)[U])
{
    accumulate<BITS, NW, FIRST>(acc, w[0], s[0]);
#pragma unroll
    for (int u = 1; u < U; ++u) accumulate<BITS, NW, false>(acc, w[u], s[u]);
}

// Sum of the K >= 1 peers' decoded values for the EPL elements starting at element e,
// whose scales are entry blk of the peers' scale arrays.  Peers are added in ascending
// order.  They are fetched in groups of U, the next group's loads issued before the
// current group is decoded.
template <int BITS, int NW, int U>
__device__ __forceinline__ void reduce_peers(const PeerTable& P, int K, uint64_t e, uint64_t blk,
                                             float (&acc)[(EPL<BITS, NW>::value)])
{
    const uint64_t byte_off = e * BITS / 8;
    const int full = K / U;
    int k = 0;  // peers done
    if (full > 0) {
        uint32_t wa[U][NW], wb[U][NW];
        float sa[U], sb[U];
        load_group<NW, U>(P, 0, byte_off, blk, wa, sa);
        if (full > 1) load_group<NW, U>(P, U, byte_off, blk, wb, sb);
        add_group<BITS, NW, U, true>(acc, wa, sa);
        // groups 1 .. full-1, alternating between the two register sets
        for (int g = 1; g < full; g += 2) {
            if (g + 1 < full) load_group<NW, U>(P, (g + 1) * U, byte_off, blk, wa, sa);
            add_group<BITS, NW, U, false>(acc, wb, sb);
            if (g + 1 < full) {
                if (g + 2 < full) load_group<NW, U>(P, (g + 2) * U, byte_off, blk, wb, sb);
                add_group<BITS, NW, U, false>(acc, wa, sa);
            }
        }
        k = full * U;
    } else {
        uint32_t w1[1][NW];
        float s1[1];
        load_group<NW, 1>(P, 0, byte_off, blk, w1, s1);
        add_group<BITS, NW, 1, true>(acc, w1, s1);
        k = 1;
    }
    for (; k < K; ++k) {
        uint32_t w1[1][NW];
        float s1[1];
        load_group<NW, 1>(P, k, byte_off, blk, w1, s1);
        add_group<BITS, NW, 1, false>(acc, w1, s1);
    }
}

// The same sum with one peer at a time and convert-and-multiply decodes: the path of the
// row-form kernels for scales their fused decode cannot take.
template <int BITS, int NW>
__device__ __forceinline__ void reduce_peers_plain(const PeerTable& P, int K, uint64_t e, uint64_t blk,
                                                   float (&acc)[(EPL<BITS, NW>::value)])
{
    const uint64_t byte_off = e * BITS / 8;
    uint32_t w[NW];
    load_words<NW>(P.codes[0] + byte_off, w);
    accumulate_plain<BITS, NW, true>(acc, w, P.scales[0][blk]);
    for (int k = 1; k < K; ++k) {
        load_words<NW>(P.codes[k] + byte_off, w);
        accumulate_plain<BITS, NW, false>(acc, w, P.scales[k][blk]);
    }
}

// ---------------------------------------------------------------------------
// qgz_inter_reduce, row form: blocks that are a whole number of rows of 16 lanes x E elements
// ---------------------------------------------------------------------------
//
// A lane takes, per peer, C vectors of NW code dwords (E = NW * 32 / BITS elements each);
// vector c of lane l starts at element (c * 64 + l) * E of the wave's tile, so every
// wave-wide load is one contiguous run.  When 16 * E divides the block, the 16 lanes of a
// row (lanes 16r .. 16r+15) decode with one scale per peer, and the scales travel through
// LDS instead of through per-lane loads: before the first peer, lane j of each row fetches
// the scales of peers j, j+16, j+32, j+48 for the row's block (a few wave-wide loads cover
// all peers), derives the operands of the fused decode for them and parks them in a table
// of the wave; each peer's operands are then read back with one broadcast LDS read per
// row.  That takes the scale load, its address arithmetic and the three multiplies per
// peer and lane off the vector ALU, which is what bounds this kernel.  (The intra-node stage
// keeps per-lane scales: with its 16-byte code vectors they are 5 of the 87 vector instructions
// a peer costs, less than a table's set-up.)
//
// Codes are fetched in groups of U peers into two register sets, the next group's loads
// issued before the current group is decoded; every branch of the steady state leaves
// the loop, so the wait before a decode never includes the loads issued after it.

// One wave's table: [row r][peer k][vector c][operand], PL operands per peer and vector (int4:
// s * 2^24, s * 2^20, -8 s; int8: s * 2^24, -128 s), so that what one peer needs, and what a group of peers
// needs, is one short run behind one address.  The row pitch is odd, so the 4 rows, which are
// read together, fall into different banks.
template <int BITS, int C>
struct RowTable {
    static constexpr int PL = BITS == 4 ? 3 : 2;
    static constexpr int row_pitch = (ZPP_MAX_PEERS * C * PL) | 1;
    static constexpr int floats = 4 * row_pitch;
};

// The wave's table is filled in three steps, so that the two dependent fetches it needs can be
// issued early and waited for late.  The host repeats the last peer in the unused entries of
// the pointer table, so all ZPP_MAX_PEERS entries can be read.
constexpr int kRowChunks = ZPP_MAX_PEERS / 16;

// 1: lane j of every row takes the scale pointers of peers j, j + 16, j + 32, j + 48
__device__ __forceinline__ void row_scale_pointers(const PeerTable& P, int lane, const float* (&sp)[kRowChunks])
{
#pragma unroll
    for (int i = 0; i < kRowChunks; ++i) sp[i] = P.scales[i * 16 + (lane & 15)];
}

// 2: their scales for the block of the lane's row in each vector (blk[c]: equal in the 16 lanes of a row)
template <int C>
__device__ __forceinline__ void row_scale_loads(const float* const (&sp)[kRowChunks], const uint64_t (&blk)[C],
                                                float (&s)[kRowChunks][C])
{
#pragma unroll
    for (int i = 0; i < kRowChunks; ++i)
#pragma unroll
        for (int c = 0; c < C; ++c) s[i][c] = sp[i][blk[c]];
}

// What a wave learns about its scales while it writes its table.
struct RowScaleFacts {
    bool exact;  // every scale can take the fused decode (else the table must not be used)
    bool mid;    // every scale is 0 or 2^-30 <= |s| < 2^60: nonzero sums then lie in [2^-53, 2^69)
};

// 3: the decode operands go to the table
template <int BITS, int C>
__device__ __forceinline__ RowScaleFacts write_row_table(const float (&s)[kRowChunks][C], int lane,
                                                         float* __restrict__ tab)
{
    using T = RowTable<BITS, C>;
    const int j = lane & 15, row = lane >> 4;
    bool fine = true, mid = true;
#pragma unroll
    for (int i = 0; i < kRowChunks; ++i)
#pragma unroll
        for (int c = 0; c < C; ++c) {
            float* t = tab + row * T::row_pitch + ((i * 16 + j) * C + c) * T::PL;
            const float mag = fabsf(s[i][c]);
            mid = mid && (mag == 0.0f || (mag >= 0x1p-30f && mag < 0x1p60f));
            fine = fine && fused_decode_ok(s[i][c]);
            if (BITS == 4) {
                const Dec4 op = dec4_operands(s[i][c]);
                t[0] = op.lo;
                t[1] = op.hi;
                t[2] = op.bias;
            } else {
                const Dec8 op = dec8_operands(s[i][c]);
                t[0] = op.lo;
                t[1] = op.bias;
            }
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    RowScaleFacts f;
    f.exact = __builtin_amdgcn_ballot_w64(!fine) == 0;
    f.mid = __builtin_amdgcn_ballot_w64(!mid) == 0;
    return f;
}

// Group of U peers from k0 on (entries past the last peer repeat it: loads that are not used).
template <int NW, int C, int U>
__device__ __forceinline__ void load_group_rows(const PeerTable& P, int k0, uint64_t tile_byte,
                                                uint32_t (&lane_byte)[C], uint32_t (&w)[U][C][NW])
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint8_t* p = P.codes[k0 + u] + tile_byte;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            // an empty statement the optimizer cannot see through keeps the 32-bit lane offset
            // next to its use (not widened once and for all outside the loop), so that the load
            // takes the scalar base + 32-bit vector offset address form instead of a 64-bit
            // vector add per load
            asm volatile("" : "+v"(lane_byte[c]));
            load_words<NW>(p + lane_byte[c], w[u][c]);
        }
    }
}

// Adds peers k0 .. k0 + count - 1 (count <= U; PARTIAL = false: count == U) from w to sums
// that the first group has started.
// row_tab: the wave's table advanced to this lane's row.
template <int BITS, int NW, int C, int U, bool PARTIAL>
__device__ __forceinline__ void add_group_rows(float (&acc)[C][(EPL<BITS, NW>::value)], const uint32_t (&w)[U][C][NW],
                                               const float* __restrict__ row_tab, int k0, int count)
{
    using T = RowTable<BITS, C>;
    const float* t = row_tab + k0 * (C * T::PL);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (PARTIAL && u >= count) break;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const float* tc = t + (u * C + c) * T::PL;
            if (BITS == 4) {
                Dec4 op;
                op.lo = tc[0];
                op.hi = tc[1];
                op.bias = tc[2];
#pragma unroll
                for (int j = 0; j < NW; ++j) add_nibbles8<false>(acc[c] + j * 8, w[u][c][j], op);
            } else {
                Dec8 op;
                op.lo = tc[0];
                op.bias = tc[1];
#pragma unroll
                for (int j = 0; j < NW; ++j) add_bytes4<false>(acc[c] + j * 4, w[u][c][j], op);
            }
        }
    }
}

// acc[c][*] = sum over the K >= 1 peers, ascending, of the decoded values of the lane's
// vectors.  Returns true if the wave knows that every nonzero sum lies in [2^-53, 2^69).  tile_byte: byte offset of the wave's tile in every peer's codes; lane_byte[c]:
// byte offset of the lane's vector c inside the tile; elem[c] / blk[c]: its first element
// and its block.  tab: LDS for this wave's table.
template <int BITS, int NW, int C, int U>
__device__ __forceinline__ bool reduce_rows(const PeerTable& P, int K, uint64_t tile_byte,
                                            uint32_t (&lane_byte)[C], const uint64_t (&elem)[C],
                                            const uint64_t (&blk)[C], int lane, float* __restrict__ tab,
                                            float (&acc)[C][(EPL<BITS, NW>::value)])
{
    uint32_t wa[U][C][NW], wb[U][C][NW];
    const int n = (K + U - 1) / U;  // groups
    // Issue order: the table's scale pointers, the first group's codes and the lanes' own scales
    // for it, the table's scales, the second group's codes.  The first group is decoded with the
    // lanes' own scales while the table's fetches are still on their way.
    const float* sp[kRowChunks];
    row_scale_pointers(P, lane, sp);
    load_group_rows<NW, C, U>(P, 0, tile_byte, lane_byte, wa);
    float s0[U][C];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < C; ++c) s0[u][c] = P.scales[u][blk[c]];
    // (both also when there is only one group: the pointer table is padded, and fetches that
    // depend on nothing later keep this order)
    float st[kRowChunks][C];
    row_scale_loads<C>(sp, blk, st);
    load_group_rows<NW, C, U>(P, U, tile_byte, lane_byte, wb);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (u >= K) break;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if (u == 0) accumulate<BITS, NW, true>(acc[c], wa[u][c], s0[u][c]);
            else accumulate<BITS, NW, false>(acc[c], wa[u][c], s0[u][c]);
        }
    }
    if (n == 1) return false;
    const RowScaleFacts facts = write_row_table<BITS, C>(st, lane, tab);
    if (!facts.exact) {
        // scales of 2^100 and more: every lane decodes with its own scale loads, by convert and multiply
#pragma unroll
        for (int c = 0; c < C; ++c) reduce_peers_plain<BITS, NW>(P, K, elem[c], blk[c], acc[c]);
        return false;
    }
    const float* row_tab = tab + (lane >> 4) * RowTable<BITS, C>::row_pitch;
    for (int g = 1;;) {  // group g is in flight towards wb, wa is free
        if (g + 1 >= n) {
            add_group_rows<BITS, NW, C, U, true>(acc, wb, row_tab, g * U, K - g * U);
            break;
        }
        load_group_rows<NW, C, U>(P, (g + 1) * U, tile_byte, lane_byte, wa);
        add_group_rows<BITS, NW, C, U, false>(acc, wb, row_tab, g * U, U);
        ++g;  // group g is in flight towards wa, wb is free
        if (g + 1 >= n) {
            add_group_rows<BITS, NW, C, U, true>(acc, wa, row_tab, g * U, K - g * U);
            break;
        }
        load_group_rows<NW, C, U>(P, (g + 1) * U, tile_byte, lane_byte, wb);
        add_group_rows<BITS, NW, C, U, false>(acc, wa, row_tab, g * U, U);
        ++g;
    }
    return facts.mid;
}

// Lane geometry of a row-form tile that starts at element `tile` of an m-element tensor.
// m is a multiple of the block and the block of 16 * E, so a row of 16 lanes is inside the
// tensor or outside it as a whole.  Rows outside repeat the addresses of the tile's first
// row (always inside): they load valid data and store nothing.
//
// POW2: the block is 2^log2b elements.  Otherwise it is rows_per_block.d rows of 16 * E elements
// and the tensor has fewer than 2^32 rows, so the block index is a 32-bit division of the row
// index by a divisor prepared on the host.
template <int BITS, int NW, int C, bool POW2>
struct RowGeometry {
    static constexpr int E = EPL<BITS, NW>::value;
    bool ok[C];
    uint32_t lane_byte[C];
    uint64_t elem[C], blk[C];
    __device__ __forceinline__ RowGeometry(uint64_t tile, uint64_t m, int log2b, const FastDiv& rows_per_block, int lane)
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const uint32_t off = (uint32_t)(c * kWave + lane) * E;
            ok[c] = tile + off < m;
            const uint32_t o = ok[c] ? off : (uint32_t)(lane & 15) * E;
            lane_byte[c] = o * BITS / 8;
            elem[c] = tile + o;
            blk[c] = POW2 ? elem[c] >> log2b : (uint64_t)fast_div((uint32_t)(elem[c] / (16 * E)), rows_per_block);
        }
    }
};

// bytes of LDS a wave of a row-form kernel needs: its scale table, and for the inter-node
// stage the 64 x E results of one vector while they are turned for the store
template <int BITS, int NW, int C, bool TURN>
struct RowLds {
    static constexpr int table = RowTable<BITS, C>::floats * 4;
    static constexpr int turn = TURN ? kWave * EPL<BITS, NW>::value * 4 : 0;
    static constexpr int bytes = ((table > turn ? table : turn) + 15) / 16 * 16;
};

// qgz_intra_reduce, power-of-two blocks with EPL <= B <= 64*EPL: a lane owns the EPL
// consecutive output elements of NW code dwords, B/EPL lanes form a block.
template <int BITS, int LOG2B, int NW>
__global__ __launch_bounds__(kThreads) void k_intra_reduce(const PeerTable P, int K, uint64_t m,
                                                           uint8_t* __restrict__ codes_out,
                                                           float* __restrict__ scales_out)
{
    constexpr int E = EPL<BITS, NW>::value;
    constexpr int B = 1 << LOG2B;
    constexpr int G = B / E;
    static_assert(G >= 1 && G <= kWave, "block must fit a wave");
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t wid = (uint64_t)blockIdx.x * kWavesPerWG + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t e = (wid * kWave + lane) * E;
    const bool ok = e < m;  // m % B == 0 and B % E == 0: a lane is all in or all out
    float acc[E];
    if (ok) {
        reduce_peers<BITS, NW, 4>(P, K, e, e >> LOG2B, acc);
    } else {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = 0.0f;
    }
    float a = fabsf(acc[0]);
#pragma unroll
    for (int i = 1; i < E; ++i) a = fmaxf(a, fabsf(acc[i]));
    a = group_max<G>(a);
    float scale, inv;
    block_scale<BITS>(a, scale, inv);
    if (!ok) return;
    if ((lane & (G - 1)) == 0) scales_out[e >> LOG2B] = scale;
    constexpr int FIELDS = 32 / BITS;
    uint32_t o[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) o[j] = pack_dword<BITS>(acc + j * FIELDS, inv);
    uint8_t* dst = codes_out + e * BITS / 8;
    if constexpr (NW == 4) {
        const u32x4 v = {o[0], o[1], o[2], o[3]};
        st_stream(v, reinterpret_cast<u32x4*>(dst));
    } else if constexpr (NW == 2) {
        const u32x2 v = {o[0], o[1]};
        st_stream(v, reinterpret_cast<u32x2*>(dst));
    } else {
        st_stream(o[0], reinterpret_cast<uint32_t*>(dst));
    }
}

// qgz_intra_reduce for any other block size (not a power of two, or large): one wave per
// block, 8 elements per lane and round, R <= 8 rounds
// ((R-1)*64 < B/8 <= R*64).  The sums of the whole block wait in registers between the
// maximum and the encode.  The peers are the outer loop: per peer one scale (the same for the
// whole wave) and one load per round; the next peer's loads are issued before the current
// peer is decoded (two register sets), and nothing inside the loop branches around a load, so
// the wait before a decode covers that peer's loads only.  Lanes past the end of the block
// fetch and decode piece 0 again; their sums are left out of the maximum and not stored.
template <int NW, int R>
__device__ __forceinline__ void load_block_rounds(const uint8_t* __restrict__ src, const uint32_t (&off)[R],
                                                  uint32_t (&w)[R][NW])
{
#pragma unroll
    for (int r = 0; r < R; ++r) load_words<NW>(src + off[r], w[r]);
}

// the fused decode, valid for |s| < 2^100 (the caller redoes the block otherwise)
template <int BITS, int NW, int R, bool FIRST>
__device__ __forceinline__ void add_block_rounds(float (&acc)[R][8], const uint32_t (&w)[R][NW], float s)
{
    if constexpr (BITS == 4) {
        const Dec4 op = dec4_operands(s);
#pragma unroll
        for (int r = 0; r < R; ++r) add_nibbles8<FIRST>(acc[r], w[r][0], op);
    } else {
        const Dec8 op = dec8_operands(s);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            add_bytes4<FIRST>(acc[r], w[r][0], op);
            add_bytes4<FIRST>(acc[r] + 4, w[r][1], op);
        }
    }
}

template <int BITS, int R>
__global__ __launch_bounds__(kThreads) void k_intra_reduce_anyblock(const PeerTable P, int K, uint32_t B,
                                                                    uint64_t blocks,
                                                                    uint8_t* __restrict__ codes_out,
                                                                    float* __restrict__ scales_out)
{
    constexpr int NW = BITS == 4 ? 1 : 2;  // code dwords of 8 elements
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t blk = (uint64_t)blockIdx.x * kWavesPerWG + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (blk >= blocks) return;
    const uint32_t chunks = B / 8;  // 8-element pieces of the block
    const uint64_t base_byte = blk * B * BITS / 8;
    uint32_t off[R];  // byte offset of the lane's piece in each round
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t c = (uint32_t)r * kWave + lane;
        off[r] = (c < chunks ? c : 0u) * (uint32_t)BITS;
    }
    float acc[R][8];
    uint32_t wa[R][NW], wb[R][NW];
    // entries of the table past the last peer repeat it, so peer 1 and the peer fetched ahead
    // in the loop exist for every K
    load_block_rounds<NW, R>(P.codes[0] + base_byte, off, wa);
    float sa = P.scales[0][blk];
    load_block_rounds<NW, R>(P.codes[1] + base_byte, off, wb);
    float sb = P.scales[1][blk];
    add_block_rounds<BITS, NW, R, true>(acc, wa, sa);
    bool exact = fused_decode_ok(sa);  // of all scales so far (same in every lane)
    int k = 1;                    // peers done; peer k waits in wb
    for (; k + 1 < K; k += 2) {
        load_block_rounds<NW, R>(P.codes[k + 1] + base_byte, off, wa);
        sa = P.scales[k + 1][blk];
        add_block_rounds<BITS, NW, R, false>(acc, wb, sb);
        exact &= fused_decode_ok(sb);
        const int ahead = k + 2 < ZPP_MAX_PEERS ? k + 2 : ZPP_MAX_PEERS - 1;
        load_block_rounds<NW, R>(P.codes[ahead] + base_byte, off, wb);
        sb = P.scales[ahead][blk];
        add_block_rounds<BITS, NW, R, false>(acc, wa, sa);
        exact &= fused_decode_ok(sa);
    }
    if (k < K) {
        add_block_rounds<BITS, NW, R, false>(acc, wb, sb);
        exact &= fused_decode_ok(sb);
    }
    if (!exact) {  // a scale of 2^100 or more: the whole block again, by convert and multiply
        load_block_rounds<NW, R>(P.codes[0] + base_byte, off, wa);
        sa = P.scales[0][blk];
#pragma unroll
        for (int r = 0; r < R; ++r) accumulate_plain<BITS, NW, true>(acc[r], wa[r], sa);
        for (k = 1; k < K; ++k) {
            load_block_rounds<NW, R>(P.codes[k] + base_byte, off, wa);
            sa = P.scales[k][blk];
#pragma unroll
            for (int r = 0; r < R; ++r) accumulate_plain<BITS, NW, false>(acc[r], wa[r], sa);
        }
    }
    float a = 0.0f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t c = (uint32_t)r * kWave + lane;
        if (c < chunks) a = fmaxf(a, absmax8(acc[r]));
    }
    a = group_max<kWave>(a);
    float scale, inv;
    block_scale<BITS>(a, scale, inv);
    if (lane == 0) scales_out[blk] = scale;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t c = (uint32_t)r * kWave + lane;
        if (c < chunks) store_codes8<BITS>(codes_out, blk * B + c * 8u, acc[r], inv);
    }
}

// How the inter-node stage divides its sums by the launch's divisor d (same in every lane).
enum DivMode {
    kDivIeee = 0,     // the division instruction sequence
    kDivPow2 = 1,     // d is a power of two: multiplying by its (exact) reciprocal rounds the same real number
    kDivConstant = 2  // y = RN(1/d) prepared on the host, sums known to lie in a middle range: div_by_constant
};

// a / d, correctly rounded, from y = RN(1/d): q = a*y; then twice r = a - d*q (exact in a fused
// multiply-add), q += r*y.  These are the closing steps of the usual division sequence (an
// approximate quotient from a reciprocal good to an ulp, corrected twice by its exact
// remainder); with the reciprocal itself correctly rounded and no scaling needed they are
// all that is left: 5 operations instead of 11.  Valid while nothing under- or overflows: the
// host admits 2^-10 <= d <= 2^16 and the kernel a = 0 or 2^-53 <= |a| < 2^69, so that
// 2^-69 <= |q| < 2^79 and every remainder (a multiple of ulp(d) * ulp(q) >= 2^-125) is
// representable.  zpp_selfcheck_divide compares it with the division for every such a.
__device__ __forceinline__ float div_by_constant(float a, float d, float y)
{
    float q = a * y;
    float r = __builtin_fmaf(-d, q, a);
    q = __builtin_fmaf(r, y, q);
    r = __builtin_fmaf(-d, q, a);
    return __builtin_fmaf(r, y, q);
}

// The wave's 64 x E fp32 results of one vector (acc of lane l = elements l*E .. l*E+E-1 of the
// run that starts at out_run), divided, are turned through LDS so that each store
// instruction writes one contiguous run of 1 KB (lane l, store j: floats 4*(64j + l) .. +4).
// Chunk i of lane l is parked in row l at column i ^ (l % CH): rows are read back whole,
// and lanes writing the same chunk index spread over the columns.  `chunks`: 16-byte
// chunks of the run that exist (the rest lies past the end of the tensor).
template <int E>
__device__ __forceinline__ void store_turned(float (&acc)[E], float divisor, float recip, int mode,
                                             f32x4* __restrict__ turn, float* __restrict__ out_run, uint64_t chunks,
                                             int lane)
{
    constexpr int CH = E / 4;  // 16-byte chunks of results per lane
    if (mode == kDivPow2) {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = acc[i] * recip;
    } else if (mode == kDivConstant) {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = div_by_constant(acc[i], divisor, recip);
    } else {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = acc[i] / divisor;
    }
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        f32x4 v = {acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]};
        turn[lane * CH + (i ^ (lane & (CH - 1)))] = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    f32x4* o = reinterpret_cast<f32x4*>(out_run);
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const uint32_t c = (uint32_t)j * kWave + lane;  // chunk of the run this lane stores now
        const uint32_t src_lane = c / CH, src_i = c % CH;
        const f32x4 v = turn[src_lane * CH + (src_i ^ (src_lane & (CH - 1)))];
        if (c < chunks) st_stream(v, o + c);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Self-check of div_by_constant against the division: every a with 2^-53 <= |a| < 2^69 (both
// signs; 122 exponents x 2^23 mantissas, a grid-stride walk) and a = 0; *count += mismatches.
__global__ __launch_bounds__(kThreads) void k_selfcheck_divide(float d, float y, unsigned long long* __restrict__ count)
{
    const uint32_t lo = (127u - 53u) << 23, hi = (127u + 69u) << 23;  // bit patterns of 2^-53 and 2^69
    unsigned long long bad = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i <= 2ull * (hi - lo); i += (uint64_t)gridDim.x * kThreads) {
        float a = 0.0f;
        if (i > 0) {
            const uint64_t j = i - 1;
            a = as_f32((uint32_t)(lo + (j >> 1)) | ((uint32_t)(j & 1) << 31));
        }
        if (as_u32(div_by_constant(a, d, y)) != as_u32(a / d)) ++bad;
    }
    if (bad) atomicAdd(count, bad);
}

// qgz_inter_reduce, row form: element-wise, the block only selects the scale.  A wave sums
// C vectors of 64 x E elements (a tile of C * 64 * E consecutive elements).
template <int BITS, int NW, int C, int U, bool POW2>
__global__ __launch_bounds__(kThreads) void k_inter_reduce_rows(const PeerTable P, int K, uint64_t m, int log2b,
                                                                FastDiv rows_per_block, float divisor, float recip,
                                                                int recip_kind,
                                                                uint32_t groups_per_xcd, int xcd_shift,
                                                                float* __restrict__ out)
{
    constexpr int E = EPL<BITS, NW>::value;
    __shared__ __align__(16) unsigned char lds[kWavesPerWG][RowLds<BITS, NW, C, true>::bytes];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroup b runs on XCD b % 8.  Tiles are handed out so that a cache line of scales (32
    // consecutive blocks of one peer) is fetched into one XCD's L2, not into all eight: a small
    // grid gives each XCD one contiguous eighth of the tiles (groups_per_xcd > 0), a large one
    // runs of consecutive tiles, with all XCDs moving through the tensor together.
    const uint64_t group = groups_per_xcd ? (uint64_t)(blockIdx.x & 7u) * groups_per_xcd + (blockIdx.x >> 3)
                                          : logical_block(xcd_shift);
    const uint64_t tile = (group * kWavesPerWG + wave) * ((uint64_t)C * kWave * E);
    if (tile >= m) return;
    RowGeometry<BITS, NW, C, POW2> g(tile, m, log2b, rows_per_block, lane);
    float acc[C][E];
    const bool mid = reduce_rows<BITS, NW, C, U>(P, K, tile * BITS / 8, g.lane_byte, g.elem, g.blk, lane,
                                                 reinterpret_cast<float*>(lds[wave]), acc);
    const int mode = recip_kind == kDivConstant && !mid ? kDivIeee : recip_kind;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const uint64_t run = tile + (uint64_t)c * kWave * E;  // same in every lane
        if (run >= m) break;
        store_turned<E>(acc[c], divisor, recip, mode, reinterpret_cast<f32x4*>(lds[wave]), out + run, (m - run) / 4,
                        lane);
    }
}

// qgz_inter_reduce for the remaining block sizes (not a whole number of 16-lane rows): a lane
// sums the 8 (int4) or 4 (int8) consecutive elements of one code dword per peer and fetches
// its own scales.
template <int BITS>
__global__ __launch_bounds__(kThreads) void k_inter_reduce(const PeerTable P, int K, uint64_t m, uint32_t B,
                                                           int log2b, float divisor, float recip, int recip_kind,
                                                           float* __restrict__ out)
{
    constexpr int E = EPL<BITS, 1>::value;
    __shared__ f32x4 turn[kWavesPerWG][kWave * E / 4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t wid = (uint64_t)blockIdx.x * kWavesPerWG + wave;
    const uint64_t tile = wid * kWave * E;
    if (tile >= m) return;
    const uint64_t e = tile + (uint64_t)lane * E;
    const bool ok = e < m;  // m % 32 == 0 and E divides 32: a lane is all in or all out
    float acc[E];
    if (ok) {
        reduce_peers<BITS, 1, 4>(P, K, e, log2b >= 0 ? (e >> log2b) : (e / B), acc);
    } else {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = 0.0f;
    }
    store_turned<E>(acc, divisor, recip, recip_kind == kDivPow2 ? kDivPow2 : kDivIeee, turn[wave], out + tile,
                    (m - tile) / 4, lane);
}

// Plain device copy, one 16-byte vector per lane: the measured bandwidth ceiling the
// kernels above are compared with (the smallest per-workgroup footprint streams
// fastest on this memory system).
__global__ __launch_bounds__(kThreads) void k_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                   uint64_t nvec)
{
    const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < nvec) st_stream(ld_stream(src + i), dst + i);
}

// ---------------------------------------------------------------------------
// host side: argument checks and launches
// ---------------------------------------------------------------------------

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
bool valid_dtype(int d) { return d == ZPP_F16 || d == ZPP_BF16 || d == ZPP_F32; }
bool valid_bits(int b) { return b == 4 || b == 8; }
bool valid_block(int b) { return b >= 32 && b <= 4096 && b % 32 == 0; }
int log2_or_neg(uint32_t b) { return (b & (b - 1)) == 0 ? __builtin_ctz(b) : -1; }

int launch_status()
{
    return hipGetLastError() == hipSuccess ? ZPP_OK : ZPP_ELAUNCH;
}

constexpr uint64_t kMaxGrid = 0x7fffffffull;

// wave slots of the chip at full occupancy: 256 CUs x 4 SIMDs x 8 waves
constexpr uint64_t kWaveSlots = 256ull * 4 * 8;

// Quantize launches of at most this many wave tiles (16 residency rounds) issue all of a tile's
// loads at once.  Measured over 2^23 .. 2^29 elements: with four loads per tile that is 3 to 14 %
// faster up to about this size, the same at twice the size and 3 % slower beyond.
constexpr uint64_t kDeepTilesLimit = 16 * kWaveSlots;

template <int DT, int BITS, int LOG2B>
int launch_quantize_tiled(const void* x, uint8_t* codes, float* scales, uint64_t L, uint64_t slices, uint32_t X,
                          uint32_t Y, hipStream_t st)
{
    constexpr int VMIN = BITS == 8 ? kQuantV8 : kQuantV4;
    constexpr int V = (1 << LOG2B) / 512 > VMIN ? (1 << LOG2B) / 512 : VMIN;
    const uint64_t tps = (L + 512 * V - 1) / (512 * V);
    const uint64_t tiles = tps * slices;
    int xcd_shift;
    const uint64_t grid = plan_grid((tiles + kWavesPerWG - 1) / kWavesPerWG, xcd_shift);
    if (grid > kMaxGrid || tiles >= (1ull << 32) || slices >= (1ull << 32)) return ZPP_EINVAL;
    const FastDiv by_tps = make_fastdiv((uint32_t)tps), byT = make_fastdiv(X * Y), byY = make_fastdiv(Y);
    if (tiles <= kDeepTilesLimit)
        k_quantize<DT, BITS, LOG2B, V, true><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(
            x, codes, scales, L, by_tps, (uint32_t)tiles, X, byT, byY, xcd_shift);
    else
        k_quantize<DT, BITS, LOG2B, V, false><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(
            x, codes, scales, L, by_tps, (uint32_t)tiles, X, byT, byY, xcd_shift);
    return launch_status();
}

template <int DT, int BITS>
int launch_quantize(const void* x, uint8_t* codes, float* scales, uint64_t L, uint64_t slices, uint32_t B,
                    uint32_t X, uint32_t Y, hipStream_t st)
{
    switch (log2_or_neg(B)) {
    case 5: return launch_quantize_tiled<DT, BITS, 5>(x, codes, scales, L, slices, X, Y, st);
    case 6: return launch_quantize_tiled<DT, BITS, 6>(x, codes, scales, L, slices, X, Y, st);
    case 7: return launch_quantize_tiled<DT, BITS, 7>(x, codes, scales, L, slices, X, Y, st);
    case 8: return launch_quantize_tiled<DT, BITS, 8>(x, codes, scales, L, slices, X, Y, st);
    case 9: return launch_quantize_tiled<DT, BITS, 9>(x, codes, scales, L, slices, X, Y, st);
    case 10: return launch_quantize_tiled<DT, BITS, 10>(x, codes, scales, L, slices, X, Y, st);
    case 11: return launch_quantize_tiled<DT, BITS, 11>(x, codes, scales, L, slices, X, Y, st);
    case 12: return launch_quantize_tiled<DT, BITS, 12>(x, codes, scales, L, slices, X, Y, st);
    default: break;
    }
    const uint64_t blocks = L / B * slices;
    const uint64_t grid = ((blocks + kWavesPerWG - 1) / kWavesPerWG);
    if (grid > kMaxGrid) return ZPP_EINVAL;
    if (blocks >= (1ull << 32)) return ZPP_EINVAL;  // more than any device buffer holds; slices and blocks per slice are smaller still
    const uint32_t rounds = (B / 8 + kWave - 1) / kWave;
    const FastDiv by_bps = make_fastdiv((uint32_t)(L / B)), byT = make_fastdiv(X * Y), byY = make_fastdiv(Y);
#define ZPP_QA(R)                                                                                                   \
    k_quantize_anyblock<DT, BITS, R><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(x, codes, scales, L, B, blocks, X, \
                                                                                       Y, by_bps, byT, byY)
    if (rounds <= 2) ZPP_QA(2);
    else if (rounds <= 4) ZPP_QA(4);
    else ZPP_QA(8);
#undef ZPP_QA
    return launch_status();
}

int dispatch_quantize(const void* x, int dtype, int bits, uint8_t* codes, float* scales, uint64_t L,
                      uint64_t slices, uint32_t B, uint32_t X, uint32_t Y, hipStream_t st)
{
#define ZPP_Q(DT, BITS) return launch_quantize<DT, BITS>(x, codes, scales, L, slices, B, X, Y, st)
    if (bits == 8) {
        if (dtype == ZPP_F16) ZPP_Q(ZPP_F16, 8);
        if (dtype == ZPP_BF16) ZPP_Q(ZPP_BF16, 8);
        ZPP_Q(ZPP_F32, 8);
    } else {
        if (dtype == ZPP_F16) ZPP_Q(ZPP_F16, 4);
        if (dtype == ZPP_BF16) ZPP_Q(ZPP_BF16, 4);
        ZPP_Q(ZPP_F32, 4);
    }
#undef ZPP_Q
}

// Code dwords a lane of qgz_intra_reduce takes per peer.  The kernel is bound by the vector
// ALU, and the widest vectors cost the fewest instructions per element; narrower ones (more,
// smaller waves) measured slower at every size.
constexpr int kIntraNW = 4;

template <int BITS>
int launch_intra(const PeerTable& P, int K, uint64_t m, uint32_t B, uint8_t* codes_out, float* scales_out,
                 hipStream_t st)
{
    constexpr int E = EPL<BITS, kIntraNW>::value;
    // Largest power-of-two block that takes the kernel with lane-owned vectors.  From there
    // on one wave per block with the scale in a scalar register is as fast or faster
    // (measured at 2^25 and 2^27 elements: int4 1024 -2 %, 2048 +1 to +8 %; int8 256 -25 %,
    // 512 +4 to +13 %, 1024 +5 to +8 %).
    constexpr int kLaneVectorMaxBlock = BITS == 4 ? 1024 : 256;
    const int l2 = log2_or_neg(B);
    if (m / B > kMaxGrid) return ZPP_EINVAL;
    const uint64_t waves = (m + (uint64_t)kWave * E - 1) / ((uint64_t)kWave * E);
    const uint64_t grid = (waves + kWavesPerWG - 1) / kWavesPerWG;
    if (grid > kMaxGrid) return ZPP_EINVAL;
#define ZPP_I(L2)                                                                                                    \
    case L2:                                                                                                         \
        if constexpr ((1 << L2) >= E && (1 << L2) <= kLaneVectorMaxBlock) {                                          \
            k_intra_reduce<BITS, L2, kIntraNW><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(P, K, m, codes_out, scales_out); \
            return launch_status();                                                                                  \
        }                                                                                                            \
        break
    switch (l2) {  // small power-of-two blocks
        ZPP_I(5);
        ZPP_I(6);
        ZPP_I(7);
        ZPP_I(8);
        ZPP_I(9);
        ZPP_I(10);
    default: break;
    }
#undef ZPP_I
    const uint64_t blocks = m / B, groups = (blocks + kWavesPerWG - 1) / kWavesPerWG;
#define ZPP_IA(R)                                                                                                    \
    case R:                                                                                                          \
        k_intra_reduce_anyblock<BITS, R><<<dim3((uint32_t)groups), dim3(kThreads), 0, st>>>(P, K, B, blocks, codes_out, scales_out); \
        return launch_status()
    switch ((B / 8 + kWave - 1) / kWave) {  // rounds of 64 lanes x 8 elements that cover a block
        ZPP_IA(1);
        ZPP_IA(2);
        ZPP_IA(3);
        ZPP_IA(4);
        ZPP_IA(5);
        ZPP_IA(6);
        ZPP_IA(7);
        ZPP_IA(8);
    default: return ZPP_EINVAL;  // unreachable: blocks have at most 4096 elements
    }
#undef ZPP_IA
}

// divisor of qgz_inter_reduce as the kernels take it
struct Divisor {
    float d, recip;
    int kind;  // DivMode the launch may use
};

Divisor prepare_divisor(float d)
{
    Divisor v = {d, 0.0f, kDivIeee};
    int e = 0;
    if (frexpf(d, &e) == 0.5f && e >= -125) {  // a power of two with a finite, normal reciprocal
        v.recip = 1.0f / d;
        v.kind = kDivPow2;
    } else if (d >= 0x1p-10f && d <= 0x1p16f) {
        v.recip = 1.0f / d;  // correctly rounded
        v.kind = kDivConstant;
    }
    return v;
}

template <int BITS, int NW, int C, int U>
int launch_inter_rows(const PeerTable& P, int K, uint64_t m, uint32_t B, const Divisor& dv, float* out, hipStream_t st)
{
    const int l2 = log2_or_neg(B);
    const FastDiv rows_per_block = make_fastdiv(B / (16 * EPL<BITS, NW>::value));
    constexpr uint64_t tile = (uint64_t)C * kWave * EPL<BITS, NW>::value;
    const uint64_t waves = (m + tile - 1) / tile;
    const uint64_t groups = (waves + kWavesPerWG - 1) / kWavesPerWG;
    // surplus groups of either padded grid exit at once
    int xcd_shift;
    uint64_t per_xcd = 0, grid = plan_grid(groups, xcd_shift);
    if (xcd_shift < 0) {
        per_xcd = (groups + 7) / 8;
        grid = per_xcd * 8;
    }
    if (grid > kMaxGrid) return ZPP_EINVAL;
    if (l2 >= 0)
        k_inter_reduce_rows<BITS, NW, C, U, true><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(
            P, K, m, l2, rows_per_block, dv.d, dv.recip, dv.kind, (uint32_t)per_xcd, xcd_shift, out);
    else
        k_inter_reduce_rows<BITS, NW, C, U, false><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(
            P, K, m, l2, rows_per_block, dv.d, dv.recip, dv.kind, (uint32_t)per_xcd, xcd_shift, out);
    return launch_status();
}

// Vectors per lane (C) for the row form of qgz_inter_reduce over `tiles` wave tiles of 64 x E
// elements.  The kernel is bound by the vector ALU, so what matters is that every SIMD gets the
// same number of tiles and that they all start together: a launch that does not fill more
// than a few residency rounds is cut into waves of C tiles such that all waves are resident
// at once (one round, no second round that runs nearly empty), choosing the C that leaves
// the fewest idle tile slots.  resident[C]: waves of the C-vector kernel a SIMD holds, by its
// registers and LDS.  Larger launches take C = 1 and let the dispatcher balance.
int inter_rows_vectors(uint64_t tiles, const uint64_t (&resident)[4])
{
    constexpr uint64_t simds = 256 * 4;
    if (tiles <= resident[1] * simds || tiles > 3 * resident[3] * simds) return 1;
    int best = 1;
    uint64_t best_cost = ~0ull;
    for (int c = 1; c <= 3; ++c) {
        const uint64_t waves = (tiles + c - 1) / c;
        if (waves > resident[c] * simds) continue;
        const uint64_t cost = (waves + simds - 1) / simds * c;  // tiles the busiest SIMD works through
        if (cost < best_cost) {
            best_cost = cost;
            best = c;
        }
    }
    return best;
}

// The row form with NW code dwords per lane and vector, if the block is a whole number of its
// rows of 16 lanes (blocks that are not powers of two find their scales by a 32-bit division
// of the row index); ZPP_EINVAL if not, and nothing is launched.
template <int BITS, int NW>
int launch_inter_row_form(const PeerTable& P, int K, uint64_t m, uint32_t B, const Divisor& dv, float* out, hipStream_t st)
{
    constexpr uint32_t E = EPL<BITS, NW>::value;
    if (B % (16 * E) != 0 || (log2_or_neg(B) < 0 && m / (16 * E) >= (1ull << 32))) return ZPP_EINVAL;
    // resident waves per SIMD of the kernels with 1, 2, 3 vectors per wave (int4: 57, 91, 102
    // registers; int8 with two dwords per vector: 68, 78, 120; with one: 50, 64, 76)
    constexpr uint64_t resident[4] = {0, BITS == 4 ? 8u : (NW == 2 ? 7u : 8u), BITS == 4 ? 5u : (NW == 2 ? 6u : 8u),
                                      BITS == 4 ? 4u : (NW == 2 ? 4u : 6u)};
    const int c = inter_rows_vectors((m + kWave * E - 1) / (kWave * E), resident);
    // peers per fetch group: 8 where a wave has one vector (more bytes in flight per wave), 4 otherwise
    if (c == 1) return launch_inter_rows<BITS, NW, 1, 8>(P, K, m, B, dv, out, st);
    if (c == 2) return launch_inter_rows<BITS, NW, 2, 4>(P, K, m, B, dv, out, st);
    return launch_inter_rows<BITS, NW, 3, 4>(P, K, m, B, dv, out, st);
}

template <int BITS>
int launch_inter(const PeerTable& P, int K, uint64_t m, uint32_t B, const Divisor& dv, float* out, hipStream_t st)
{
    constexpr uint32_t E = EPL<BITS, 1>::value;
    // A vector is 8 elements where the block allows it (int4: one code dword; int8: two, if the
    // block is a multiple of 128), else the 4 elements of one int8 dword.
    if constexpr (BITS == 8)
        if (B % 128 == 0 && (log2_or_neg(B) >= 0 || m / 128 < (1ull << 32)))
            return launch_inter_row_form<8, 2>(P, K, m, B, dv, out, st);
    if (B % (16 * E) == 0 && (log2_or_neg(B) >= 0 || m / (16 * E) < (1ull << 32)))
        return launch_inter_row_form<BITS, 1>(P, K, m, B, dv, out, st);
    const int l2 = log2_or_neg(B);
    constexpr uint64_t per_wave = (uint64_t)kWave * E;
    const uint64_t waves = (m + per_wave - 1) / per_wave;
    const uint64_t grid = (waves + kWavesPerWG - 1) / kWavesPerWG;
    if (grid > kMaxGrid) return ZPP_EINVAL;
    k_inter_reduce<BITS><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(P, K, m, B, l2, dv.d, dv.recip, dv.kind, out);
    return launch_status();
}

int fill_table(PeerTable& P, const void* const* codes_in, const float* const* scales_in, int K)
{
    if (!codes_in || !scales_in || K < 1 || K > ZPP_MAX_PEERS) return ZPP_EINVAL;
    for (int k = 0; k < K; ++k) {
        if (!codes_in[k] || !scales_in[k] || !aligned(codes_in[k], 16) || !aligned(scales_in[k], 4)) return ZPP_EINVAL;
        P.codes[k] = static_cast<const uint8_t*>(codes_in[k]);
        P.scales[k] = scales_in[k];
    }
    // the unused entries repeat the last peer: kernels that fetch peers in fixed groups may read
    // (and then ignore) them
    for (int k = K; k < ZPP_MAX_PEERS; ++k) {
        P.codes[k] = P.codes[K - 1];
        P.scales[k] = P.scales[K - 1];
    }
    return ZPP_OK;
}

}  // namespace

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------

extern "C" {

size_t zpp_codes_bytes(size_t n, int bits) { return valid_bits(bits) ? n / 8 * (size_t)bits + (n % 8) * (size_t)bits / 8 : 0; }

size_t zpp_scales_count(size_t n, int block) { return block > 0 ? n / (size_t)block : 0; }

const char* zpp_strerror(int code)
{
    switch (code) {
    case ZPP_OK: return "ok";
    case ZPP_EINVAL: return "invalid argument (null or misaligned pointer, size not a multiple of the block, value out of range)";
    case ZPP_ELAUNCH: return "HIP runtime refused the kernel launch";
    default: return "unknown zpp error code";
    }
}

long long zpp_reorder_source_slice(long long p, int X, int Y, int S)
{
    if (X < 1 || Y < 1 || S < 1 || p < 0 || p >= (long long)X * Y * S) return -1;
    if ((long long)X * Y * S < (1ll << 32))  // the same arithmetic the kernels use
        return (long long)source_slice32((uint32_t)p, (uint32_t)X, make_fastdiv((uint32_t)X * (uint32_t)Y),
                                         make_fastdiv((uint32_t)Y));
    return (long long)source_slice((uint64_t)p, (uint32_t)X, (uint32_t)Y);
}

long long zpp_reorder_mapped_slice(long long pid, int X, int Y, int S)
{
    if (X < 1 || Y < 1 || S < 1 || pid < 0 || pid >= (long long)X * Y * S) return -1;
    // inverse permutation: the same transpose with the roles of X and Y exchanged
    if ((long long)X * Y * S < (1ll << 32))
        return (long long)source_slice32((uint32_t)pid, (uint32_t)Y, make_fastdiv((uint32_t)X * (uint32_t)Y),
                                         make_fastdiv((uint32_t)X));
    return (long long)source_slice((uint64_t)pid, (uint32_t)Y, (uint32_t)X);
}

int qwz_quantize(const void* x, int dtype, size_t n, int block, int bits, void* codes, float* scales, void* stream)
{
    if (!valid_dtype(dtype) || !valid_bits(bits) || !valid_block(block) || n % (size_t)block != 0) return ZPP_EINVAL;
    if (n == 0) return ZPP_OK;
    if (!x || !codes || !scales || !aligned(x, 16) || !aligned(codes, 16) || !aligned(scales, 4)) return ZPP_EINVAL;
    return dispatch_quantize(x, dtype, bits, static_cast<uint8_t*>(codes), scales, n, 1, (uint32_t)block, 1, 1,
                             static_cast<hipStream_t>(stream));
}

int qgz_reorder(const void* grad, int dtype, size_t n, int X, int Y, int S, int block, int bits, void* codes,
                float* scales, void* stream)
{
    if (!valid_dtype(dtype) || !valid_bits(bits) || !valid_block(block)) return ZPP_EINVAL;
    if (X < 1 || Y < 1 || S < 1 || X > 65535 || Y > 65535 || S > 65535) return ZPP_EINVAL;
    const uint64_t slices = (uint64_t)X * Y * S;
    if (n % (slices * (uint64_t)block) != 0) return ZPP_EINVAL;
    if (n == 0) return ZPP_OK;
    if (!grad || !codes || !scales || !aligned(grad, 16) || !aligned(codes, 16) || !aligned(scales, 4)) return ZPP_EINVAL;
    return dispatch_quantize(grad, dtype, bits, static_cast<uint8_t*>(codes), scales, n / slices, slices,
                             (uint32_t)block, (uint32_t)X, (uint32_t)Y, static_cast<hipStream_t>(stream));
}

int qwz_dequantize(const void* codes, const float* scales, size_t n, int block, int bits, int out_dtype, void* y,
                   void* stream)
{
    if (!valid_dtype(out_dtype) || !valid_bits(bits) || !valid_block(block) || n % (size_t)block != 0) return ZPP_EINVAL;
    if (n == 0) return ZPP_OK;
    if (!y || !codes || !scales || !aligned(y, 16) || !aligned(codes, 16) || !aligned(scales, 4)) return ZPP_EINVAL;
    constexpr int V = kDeqV;
    const uint64_t waves = (n + 512 * V - 1) / (512 * V);
    int xcd_shift;
    const uint64_t grid = plan_grid((waves + kWavesPerWG - 1) / kWavesPerWG, xcd_shift);
    if (grid > kMaxGrid) return ZPP_EINVAL;
    const uint8_t* c = static_cast<const uint8_t*>(codes);
    const int l2 = log2_or_neg((uint32_t)block);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool one_block = block % (512 * V) == 0;  // a wave's tile inside one block
#define ZPP_D(ODT, BITS)                                                                                          \
    do {                                                                                                          \
        if (l2 >= 0 && one_block)                                                                                 \
            k_dequantize<ODT, BITS, V, true, true><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(c, scales, y, n, (uint32_t)block, l2, xcd_shift);  \
        else if (l2 >= 0)                                                                                         \
            k_dequantize<ODT, BITS, V, true, false><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(c, scales, y, n, (uint32_t)block, l2, xcd_shift);  \
        else                                                                                                      \
            k_dequantize<ODT, BITS, V, false, false><<<dim3((uint32_t)grid), dim3(kThreads), 0, st>>>(c, scales, y, n, (uint32_t)block, l2, xcd_shift); \
    } while (0)
    if (bits == 8) {
        if (out_dtype == ZPP_F16) ZPP_D(ZPP_F16, 8);
        else if (out_dtype == ZPP_BF16) ZPP_D(ZPP_BF16, 8);
        else ZPP_D(ZPP_F32, 8);
    } else {
        if (out_dtype == ZPP_F16) ZPP_D(ZPP_F16, 4);
        else if (out_dtype == ZPP_BF16) ZPP_D(ZPP_BF16, 4);
        else ZPP_D(ZPP_F32, 4);
    }
#undef ZPP_D
    return launch_status();
}

int qgz_intra_reduce(const void* const* codes_in, const float* const* scales_in, int ranks, size_t m, int block,
                     int bits, void* codes_out, float* scales_out, void* stream)
{
    if (!valid_bits(bits) || !valid_block(block) || m % (size_t)block != 0) return ZPP_EINVAL;
    PeerTable P;
    if (fill_table(P, codes_in, scales_in, ranks) != ZPP_OK) return ZPP_EINVAL;
    if (m == 0) return ZPP_OK;
    if (!codes_out || !scales_out || !aligned(codes_out, 16) || !aligned(scales_out, 4)) return ZPP_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bits == 4) return launch_intra<4>(P, ranks, m, (uint32_t)block, static_cast<uint8_t*>(codes_out), scales_out, st);
    return launch_intra<8>(P, ranks, m, (uint32_t)block, static_cast<uint8_t*>(codes_out), scales_out, st);
}

int qgz_inter_reduce(const void* const* codes_in, const float* const* scales_in, int nodes, size_t m, int block,
                     int bits, float divisor, float* out, void* stream)
{
    if (!valid_bits(bits) || !valid_block(block) || m % (size_t)block != 0 || !(divisor > 0.0f)) return ZPP_EINVAL;
    PeerTable P;
    if (fill_table(P, codes_in, scales_in, nodes) != ZPP_OK) return ZPP_EINVAL;
    if (m == 0) return ZPP_OK;
    if (!out || !aligned(out, 16)) return ZPP_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Divisor dv = prepare_divisor(divisor);
    if (bits == 4) return launch_inter<4>(P, nodes, m, (uint32_t)block, dv, out, st);
    return launch_inter<8>(P, nodes, m, (uint32_t)block, dv, out, st);
}

// Diagnostic: compares the short division sequences the encoders use with the plain
// fp32 divisions for every mantissa at one binary exponent.
int zpp_selfcheck_block_scale(int bits, int exponent, unsigned long long* counts, void* stream)
{
    if (!valid_bits(bits) || exponent < -100 || exponent > 99 || !counts || !aligned(counts, 8)) return ZPP_EINVAL;
    const uint32_t eb = (uint32_t)(exponent + 127);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bits == 4) k_selfcheck_block_scale<4><<<dim3((1u << 23) / kThreads), dim3(kThreads), 0, st>>>(eb, counts);
    else k_selfcheck_block_scale<8><<<dim3((1u << 23) / kThreads), dim3(kThreads), 0, st>>>(eb, counts);
    return launch_status();
}

// Diagnostic: compares the short division by a launch-constant divisor that qgz_inter_reduce
// uses with the plain fp32 division, for every dividend the kernel admits to it.
int zpp_selfcheck_divide(float divisor, unsigned long long* count, void* stream)
{
    if (!count || !aligned(count, 8) || !(divisor > 0.0f)) return ZPP_EINVAL;
    const Divisor dv = prepare_divisor(divisor);
    if (dv.kind != kDivConstant) return ZPP_EINVAL;  // such divisors never take the short sequence
    k_selfcheck_divide<<<dim3(256 * 32), dim3(kThreads), 0, static_cast<hipStream_t>(stream)>>>(dv.d, dv.recip, count);
    return launch_status();
}

// Measurement helper (not part of the paper's method): copy `bytes` (a multiple of
// 16) from src to dst with the same access width the kernels use.
int zpp_stream_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (bytes % 16 != 0) return ZPP_EINVAL;
    if (bytes == 0) return ZPP_OK;
    if (!dst || !src || !aligned(dst, 16) || !aligned(src, 16)) return ZPP_EINVAL;
    const uint64_t nvec = bytes / 16;
    const uint64_t grid = (nvec + kThreads - 1) / kThreads;
    if (grid > kMaxGrid) return ZPP_EINVAL;
    k_copy<<<dim3((uint32_t)grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), nvec);
    return launch_status();
}

}  // extern "C"
