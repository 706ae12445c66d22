// Device-side helpers shared by the kernels of libtensair (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32;
typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned short bf16_t;  // raw bfloat16 bits

#define WAVE 64
#define BLOCK 256
#define WAVES_PER_BLOCK (BLOCK / WAVE)

// status word bits (device), reported as TENSAIR_EDATA
#define ST_BAD_ID 1
#define ST_BAD_ORDER 2
#define ST_OVERFLOW 4

// ---------------------------------------------------------------- bf16
__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((u32)h << 16); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    u32 u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// ---------------------------------------------------------------- 4-element chunks of a row
__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ float4 ld4(const bf16_t *p)
{
    uint2 r = *reinterpret_cast<const uint2 *>(p);
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u));
}
__device__ __forceinline__ void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ __forceinline__ void st4(bf16_t *p, float4 v)
{
    uint2 r;
    r.x = (u32)f32_to_bf16(v.x) | ((u32)f32_to_bf16(v.y) << 16);
    r.y = (u32)f32_to_bf16(v.z) | ((u32)f32_to_bf16(v.w) << 16);
    *reinterpret_cast<uint2 *>(p) = r;
}

// Streaming variants: global address space (so that a pointer rebuilt from integers does not
// fall back to flat addressing) and the non-temporal hint, for data that is touched once.
typedef float v4f __attribute__((ext_vector_type(4)));
typedef u32 v2u __attribute__((ext_vector_type(2)));
#define GLOBAL_AS __attribute__((address_space(1)))
__device__ __forceinline__ float4 ld4s(const float *p)
{
    v4f r = __builtin_nontemporal_load((const GLOBAL_AS v4f *)p);
    return make_float4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ float4 ld4s(const bf16_t *p)
{
    v2u r = __builtin_nontemporal_load((const GLOBAL_AS v2u *)p);
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u));
}
__device__ __forceinline__ void st4s(float *p, float4 v)
{
    v4f r = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(r, (GLOBAL_AS v4f *)p);
}
__device__ __forceinline__ void st4s(bf16_t *p, float4 v)
{
    v2u r;
    r.x = (u32)f32_to_bf16(v.x) | ((u32)f32_to_bf16(v.y) << 16);
    r.y = (u32)f32_to_bf16(v.z) | ((u32)f32_to_bf16(v.w) << 16);
    __builtin_nontemporal_store(r, (GLOBAL_AS v2u *)p);
}

// A 4-element chunk as it comes from memory: a float4 for fp32, two words (4 x bfloat16) for bf16.  Where
// several rows are loaded at a time the chunks stay in this form until they are used: a conversion placed
// next to its load makes the compiler wait for the data right there, one round trip per load instead of
// one per batch.
template <typename T> struct Raw4;
template <> struct Raw4<float> { typedef float4 type; };
template <> struct Raw4<bf16_t> { typedef uint2 type; };
__device__ __forceinline__ float4 widen4(float4 v) { return v; }
__device__ __forceinline__ float4 widen4(uint2 r)
{
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u));
}
__device__ __forceinline__ float widen1(float v) { return v; }
__device__ __forceinline__ float widen1(bf16_t v) { return bf16_to_f32(v); }
__device__ __forceinline__ void zero_raw(float4 &v) { v = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void zero_raw(uint2 &v) { v = make_uint2(0u, 0u); }
__device__ __forceinline__ float4 ldraw(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ uint2 ldraw(const bf16_t *p) { return *reinterpret_cast<const uint2 *>(p); }
__device__ __forceinline__ float4 ldraw_s(const float *p) { return ld4s(p); }
__device__ __forceinline__ uint2 ldraw_s(const bf16_t *p)
{
    v2u r = __builtin_nontemporal_load((const GLOBAL_AS v2u *)p);
    return make_uint2(r.x, r.y);
}

// A row of D = 4*C4 elements is held by one wave: lane l owns chunks l, l+64, ...
// (ITERS = ceil(C4/64) chunks per lane, compile-time).
template <typename T, int ITERS>
__device__ __forceinline__ void load_row(float4 (&r)[ITERS], const T *row, int C4, int lane)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int c = lane + WAVE * it;
        r[it] = (c < C4) ? ld4(row + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}
// the same, chunks left as loaded; MODE 0: through the caches, 1: around them (non-temporal), 2: around
// them except for the (at most two) 128-byte lines that the row shares with its neighbours in memory,
// so that the neighbour finds those in the cache
template <typename T, int ITERS, int MODE>
__device__ __forceinline__ void load_row_raw(typename Raw4<T>::type (&r)[ITERS], const T *row, int C4, int lane)
{
    const uintptr_t lo = (uintptr_t)row, hi = lo + (size_t)C4 * 4 * sizeof(T);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int c = lane + WAVE * it;
        zero_raw(r[it]);
        if (c < C4) {
            if (MODE == 0) {
                r[it] = ldraw(row + 4 * c);
            } else if (MODE == 1) {
                r[it] = ldraw_s(row + 4 * c);
            } else {
                const uintptr_t line = (uintptr_t)(row + 4 * c) & ~(uintptr_t)127;
                if (line >= lo && line + 128 <= hi) r[it] = ldraw_s(row + 4 * c);
                else r[it] = ldraw(row + 4 * c);
            }
        }
    }
}
template <int ITERS, typename R>
__device__ __forceinline__ void zero_row_raw(R (&r)[ITERS])
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) zero_raw(r[it]);
}
// acc += x for a row of chunks as loaded
template <int ITERS, typename R>
__device__ __forceinline__ void add_row_raw(float4 (&acc)[ITERS], const R (&x)[ITERS])
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const float4 v = widen4(x[it]);
        acc[it].x += v.x;
        acc[it].y += v.y;
        acc[it].z += v.z;
        acc[it].w += v.w;
    }
}
template <typename T, int ITERS>
__device__ __forceinline__ void store_row(T *row, const float4 (&r)[ITERS], int C4, int lane)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int c = lane + WAVE * it;
        if (c < C4) st4(row + 4 * c, r[it]);
    }
}
template <typename T, int ITERS>
__device__ __forceinline__ void load_row_s(float4 (&r)[ITERS], const T *row, int C4, int lane)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int c = lane + WAVE * it;
        r[it] = (c < C4) ? ld4s(row + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}
template <typename T, int ITERS>
__device__ __forceinline__ void store_row_s(T *row, const float4 (&r)[ITERS], int C4, int lane)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int c = lane + WAVE * it;
        if (c < C4) st4s(row + 4 * c, r[it]);
    }
}
template <int ITERS>
__device__ __forceinline__ void zero_row(float4 (&r)[ITERS])
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) r[it] = make_float4(0.f, 0.f, 0.f, 0.f);
}
template <int ITERS>
__device__ __forceinline__ void add_row(float4 (&acc)[ITERS], const float4 (&x)[ITERS])
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        acc[it].x += x[it].x;
        acc[it].y += x[it].y;
        acc[it].z += x[it].z;
        acc[it].w += x[it].w;
    }
}
template <int ITERS>
__device__ __forceinline__ float dot_partial(const float4 (&a)[ITERS], const float4 (&b)[ITERS])
{
    float s = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        s = fmaf(a[it].x, b[it].x, s);
        s = fmaf(a[it].y, b[it].y, s);
        s = fmaf(a[it].z, b[it].z, s);
        s = fmaf(a[it].w, b[it].w, s);
    }
    return s;
}

// ---------------------------------------------------------------- wave-level primitives
// butterfly sum: every lane ends with the same value, the order of additions is fixed
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, WAVE);
    return x;
}
// The same sum with data-parallel-primitive moves instead of LDS-crossbar shuffles: four
// in-row steps (16 lanes), then the row totals are chained into lane 63 and broadcast.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_get(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum_dpp(float x)
{
    x += dpp_get<0xB1, 0xF>(x);    // quad_perm [1,0,3,2]
    x += dpp_get<0x4E, 0xF>(x);    // quad_perm [2,3,0,1]
    x += dpp_get<0x141, 0xF>(x);   // row_half_mirror
    x += dpp_get<0x140, 0xF>(x);   // row_mirror: every lane of a row holds the row's sum
    x += dpp_get<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
    x += dpp_get<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3: lane 63 holds the total
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ __forceinline__ u32 wave_or(u32 x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x |= (u32)__shfl_xor((int)x, o, WAVE);
    return x;
}
__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }
__device__ __forceinline__ int rd_lane(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ float rd_lane(float v, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ u64 rd_lane64(u64 v, int l)
{
    u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)v, l);
    u32 hi = (u32)__builtin_amdgcn_readlane((int)(u32)(v >> 32), l);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// inclusive scan of one value per lane across the wave
__device__ __forceinline__ u32 wave_incl_scan(u32 x, int lane)
{
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        u32 y = (u32)__shfl_up((int)x, o, WAVE);
        if (lane >= o) x += y;
    }
    return x;
}

// ---------------------------------------------------------------- Philox4x32-10
// Counter-based generator of Salmon et al. (SC'11): 10 rounds, multipliers
// 0xD2511F53 / 0xCD9E8D57, key increments 0x9E3779B9 / 0xBB67AE85.
struct philox_out {
    u32 r0, r1, r2, r3;
};
__device__ __forceinline__ philox_out philox4x32_10(u32 c0, u32 c1, u32 c2, u32 c3, u32 k0, u32 k1)
{
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        u32 hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        u32 hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        u32 n0 = hi1 ^ c1 ^ k0;
        u32 n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return philox_out{c0, c1, c2, c3};
}

// ---------------------------------------------------------------- index of the table update
// start[] and mask[] hold one entry per (source, 64-row word of the vocabulary), source by source
__host__ __device__ __forceinline__ size_t idx_at(i64 words, int k, i64 word) { return (size_t)k * (size_t)words + (size_t)word; }

// ---------------------------------------------------------------- pair arithmetic
// Number of (center, context) pairs of the positions [0, p) in a stream of T tokens with
// window w: position x has min(x, w) contexts on the left and min(T-1-x, w) on the right.
__host__ __device__ __forceinline__ i64 sum_min_below(i64 x, i64 w)
{   // sum_{y=0}^{x-1} min(y, w)
    if (x <= 0) return 0;
    if (x <= w + 1) return x * (x - 1) / 2;
    return w * (w + 1) / 2 + (x - w - 1) * w;
}
__host__ __device__ __forceinline__ i64 pairs_before(i64 p, i64 T, i64 w)
{
    return sum_min_below(p, w) + sum_min_below(T, w) - sum_min_below(T - p, w);
}
