// Device-side helpers shared by the gfx950 kernels of the tolerance engine.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tao {

constexpr int kWave = 64;

// Smallest binary32 value >= v, for v >= 0 (NaN and +inf pass through).  The
// conversion itself rounds to nearest; one step up repairs a round-down.
__device__ __forceinline__ float up32(double v) {
    float f = (float)v;
    if ((double)f < v) f = __uint_as_float(__float_as_uint(f) + 1u);
    return f;
}

// Cheaper upper rounding for the streaming kernels, which also takes the place of the guard
// factor: for v >= 0 the result is a binary32 value >= v (1 + m) and at most one binary32 step
// above the smallest such value, where m is the rounding margin the caller asks for.
//  - Normal results: with mul = 1 + 2^-24 + 2m the product v mul lies above the midpoint of the
//    binary32 neighbours of v (1 + m) (their distance is at most 2^-23 of the lower one), so the
//    conversion's round-to-nearest lands on the upper neighbour or beyond: no compare, no step.
//  - Results below 2^-126 (subnormal, or zero): the spacing is absolute there and one step is a
//    large relative amount, so v (1 + m) is rounded up exactly (sub = 1 + m): the result is the
//    smallest representable value >= v sub, and 0 stays 0.
// The defaults serve the element-wise kernels (a handful of binary64 roundings and, for GELU, an
// exponential accurate to 2^-40); the row kernels pass constants that grow with the row length.
// NaN and +inf pass through.
constexpr double kUpMul = 1.0 + 0x1p-24 + 0x1p-32;
constexpr double kUpSub = 1.0 + 0x1p-36;
__device__ __forceinline__ float up32g(double v, double mul = kUpMul, double sub = kUpSub) {
    float f = (float)(v * mul);
    if (f < 0x1p-126f) {
        const double w = v * sub;
        f = (float)w;
        if ((double)f < w) f = __uint_as_float(__float_as_uint(f) + 1u);
    }
    return f;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ int wave_or(int v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v |= __shfl_xor(v, o, kWave);
    return v;
}

// Streaming 16-byte load: the data is used once, so it is marked non-temporal.
__device__ __forceinline__ float4 ntload4(const float4* p) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

// Streaming 16-byte store of data that is not read again by this kernel.
__device__ __forceinline__ void ntstore4(float4* p, float4 v) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    const v4f t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
}

// 16-byte global load when the caller has established alignment, else four
// guarded scalar loads; elements at or beyond `limit` read as `fill`.
// STREAM: the data is read once by the kernel (non-temporal load).
template <bool STREAM = false>
__device__ __forceinline__ float4 load4(const float* __restrict__ p, long idx, long limit,
                                        bool vec_ok, float fill) {
    float4 r;
    if (vec_ok && idx + 3 < limit) {
        r = STREAM ? ntload4(reinterpret_cast<const float4*>(p + idx))
                   : *reinterpret_cast<const float4*>(p + idx);
    } else {
        r.x = (idx + 0 < limit) ? p[idx + 0] : fill;
        r.y = (idx + 1 < limit) ? p[idx + 1] : fill;
        r.z = (idx + 2 < limit) ? p[idx + 2] : fill;
        r.w = (idx + 3 < limit) ? p[idx + 3] : fill;
    }
    return r;
}
__device__ __forceinline__ void store4(float* __restrict__ p, long idx, long limit, bool vec_ok,
                                       float4 v) {
    if (vec_ok && idx + 3 < limit) {
        ntstore4(reinterpret_cast<float4*>(p + idx), v);      // bounds are written once, never re-read here
    } else {
        if (idx + 0 < limit) p[idx + 0] = v.x;
        if (idx + 1 < limit) p[idx + 1] = v.y;
        if (idx + 2 < limit) p[idx + 2] = v.z;
        if (idx + 3 < limit) p[idx + 3] = v.w;
    }
}

}  // namespace tao
