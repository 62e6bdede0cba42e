// Device-side helpers shared by the liblap kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lap {

constexpr int WAVE = 64;
constexpr uint64_t U64_MAX = ~0ull;

__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }

__device__ __forceinline__ uint64_t shfl64(uint64_t v, int src)
{
    return (uint64_t)__shfl((unsigned long long)v, src, WAVE);
}

__device__ __forceinline__ uint64_t shfl_up64(uint64_t v, unsigned d)
{
    return (uint64_t)__shfl_up((unsigned long long)v, d, WAVE);
}

__device__ __forceinline__ uint64_t shfl_xor64(uint64_t v, int m)
{
    return (uint64_t)__shfl_xor((unsigned long long)v, m, WAVE);
}

__device__ __forceinline__ uint64_t umax64(uint64_t a, uint64_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint64_t umin64(uint64_t a, uint64_t b) { return a < b ? a : b; }

// inclusive prefix maximum over the wave
__device__ __forceinline__ uint64_t wave_scan_max(uint64_t v)
{
    const int l = lane_id();
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        uint64_t t = shfl_up64(v, d);
        if (l >= d) v = umax64(v, t);
    }
    return v;
}

// inclusive prefix sum over the wave
__device__ __forceinline__ uint64_t wave_scan_add(uint64_t v)
{
    const int l = lane_id();
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        uint64_t t = shfl_up64(v, d);
        if (l >= d) v += t;
    }
    return v;
}

__device__ __forceinline__ uint64_t wave_reduce_max(uint64_t v)
{
#pragma unroll
    for (int m = WAVE / 2; m > 0; m >>= 1) v = umax64(v, shfl_xor64(v, m));
    return v;
}

__device__ __forceinline__ uint64_t wave_reduce_add(uint64_t v)
{
#pragma unroll
    for (int m = WAVE / 2; m > 0; m >>= 1) v += shfl_xor64(v, m);
    return v;
}

__device__ __forceinline__ uint32_t wave_reduce_add32(uint32_t v)
{
#pragma unroll
    for (int m = WAVE / 2; m > 0; m >>= 1) v += __shfl_xor(v, m, WAVE);
    return v;
}

__device__ __forceinline__ uint64_t ballot(bool p) { return (uint64_t)__ballot(p); }

// splitmix64 output function on the counter seed + (i+1)*gamma (Steele/Lea/Flood 2014)
__device__ __forceinline__ uint64_t mix64(uint64_t seed, uint32_t i)
{
    uint64_t z = seed + ((uint64_t)i + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

}  // namespace lap
