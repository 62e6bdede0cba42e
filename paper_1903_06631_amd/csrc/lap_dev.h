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

// Data-parallel-primitive lane moves (gfx9 encodings): row_shr:n = 0x110+n shifts within
// rows of 16 lanes, row_bcast:15 / row_bcast:31 = 0x142 / 0x143 copy a row's last lane into
// the following rows, wave_shr:1 = 0x138 shifts the whole wave up by one lane.  Lanes with
// no source lane (or outside row_mask) receive `old`.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t old, uint32_t src)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, CTRL, ROW_MASK, 0xF, false);
}

// lane i receives lane i-1's value; lane 0 receives `carry`
__device__ __forceinline__ uint32_t lane_shift_up(uint32_t v, uint32_t carry) { return dpp_mov<0x138>(carry, v); }

__device__ __forceinline__ uint64_t lane_shift_up64(uint64_t v, uint64_t carry)
{
    const uint32_t lo = lane_shift_up((uint32_t)v, (uint32_t)carry);
    const uint32_t hi = lane_shift_up((uint32_t)(v >> 32), (uint32_t)(carry >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// inclusive prefix maximum of unsigned 32-bit values over the wave (identity 0)
__device__ __forceinline__ uint32_t wave_scan_max_u32(uint32_t v)
{
    v = max(v, dpp_mov<0x111>(0u, v));
    v = max(v, dpp_mov<0x112>(0u, v));
    v = max(v, dpp_mov<0x114>(0u, v));
    v = max(v, dpp_mov<0x118>(0u, v));
    v = max(v, dpp_mov<0x142, 0xA>(0u, v));
    v = max(v, dpp_mov<0x143, 0xC>(0u, v));
    return v;
}

// value of a uniform lane
__device__ __forceinline__ uint32_t read_lane(uint32_t v, int lane)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

__device__ __forceinline__ uint64_t read_lane64(uint64_t v, int lane)
{
    return ((uint64_t)read_lane((uint32_t)(v >> 32), lane) << 32) | read_lane((uint32_t)v, lane);
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
