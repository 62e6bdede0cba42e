// Memory load profile and its peak (Section II Def. 2 and Def. 4, Eq. 1).
//
// The 2N alloc/free events (+size at alloc, -size at free) are binned by their
// time key and reduced in place: delta[t] accumulates every event of step t
// (a counting sort by time whose buckets are summed instead of stored; the
// order of events inside one step does not affect the per-step load).  A
// prefix sum over the T bins gives load[t]; the same pass takes the maximum
// and the earliest step that reaches it.
#include <string.h>

#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

__global__ void k_fill_u64(uint64_t *p, size_t n, uint64_t v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

// A few KB of host values travel to the device inside the kernel arguments: the runtime copies
// the arguments when the launch is enqueued, so the host array may change or vanish as soon as
// the launch call returns, nothing waits, and the launch can be captured in a graph.
constexpr uint32_t PUT_WORDS = 448;             // 32-bit words per launch (1792 B of the 4 KB argument space)
struct PutChunk { uint32_t w[PUT_WORDS]; };
__global__ __launch_bounds__(256) void k_put_words(uint32_t *dst, uint32_t count, PutChunk c)
{
    for (uint32_t i = threadIdx.x; i < count; i += blockDim.x) dst[i] = c.w[i];
}

// Bins kept in LDS per workgroup, flushed once with global atomics.  Arithmetic
// is modulo 2^64; the prefix sums are non-negative so wrap-around cancels.
__global__ __launch_bounds__(256) void k_delta_lds(uint32_t n, uint32_t nbins,
                                                   const uint64_t *__restrict__ size,
                                                   const uint32_t *__restrict__ alloc,
                                                   const uint32_t *__restrict__ free_,
                                                   unsigned long long *delta)
{
    extern __shared__ unsigned long long bins[];
    for (uint32_t i = threadIdx.x; i < nbins; i += blockDim.x) bins[i] = 0;
    __syncthreads();
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint64_t s = size[i];
        atomicAdd(&bins[alloc[i]], (unsigned long long)s);
        atomicAdd(&bins[free_[i]], (unsigned long long)(0ull - s));
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < nbins; i += blockDim.x) {
        const unsigned long long v = bins[i];
        if (v) atomicAdd(&delta[i], v);
    }
}

// Time-local variant for long time lines: a workgroup owns 4096 consecutive variables, reads
// them once (16-byte vector loads, kept in registers), finds the step range their events
// fall into and, when that range fits the LDS bins, accumulates there and flushes the bins
// with global atomics; otherwise it adds to global memory directly.
constexpr int DW_THREADS = 256;
constexpr int DW_GROUPS = 4;                       // groups of 4 variables per thread
constexpr uint32_t DW_PER_BLOCK = DW_THREADS * DW_GROUPS * 4;

__global__ __launch_bounds__(DW_THREADS) void k_delta_window(uint32_t n, uint32_t lds_bins,
                                                             const uint64_t *__restrict__ size,
                                                             const uint32_t *__restrict__ alloc,
                                                             const uint32_t *__restrict__ free_,
                                                             unsigned long long *delta)
{
    extern __shared__ unsigned long long bins[];
    __shared__ uint32_t s_lo, s_hi;
    const uint32_t begin = blockIdx.x * DW_PER_BLOCK;
    if (threadIdx.x == 0) { s_lo = 0xFFFFFFFFu; s_hi = 0; }
    __syncthreads();
    uint64_t sz[DW_GROUPS][4];
    uint32_t al[DW_GROUPS][4], fr[DW_GROUPS][4];
    uint32_t lo = 0xFFFFFFFFu, hi = 0;
#pragma unroll
    for (int g = 0; g < DW_GROUPS; ++g) {
        const uint32_t i0 = begin + (g * DW_THREADS + threadIdx.x) * 4;
        if (i0 + 3 < n) {
            const ulonglong2 s01 = *(const ulonglong2 *)(size + i0);
            const ulonglong2 s23 = *(const ulonglong2 *)(size + i0 + 2);
            const uint4 a4 = *(const uint4 *)(alloc + i0);
            const uint4 f4 = *(const uint4 *)(free_ + i0);
            sz[g][0] = s01.x; sz[g][1] = s01.y; sz[g][2] = s23.x; sz[g][3] = s23.y;
            al[g][0] = a4.x; al[g][1] = a4.y; al[g][2] = a4.z; al[g][3] = a4.w;
            fr[g][0] = f4.x; fr[g][1] = f4.y; fr[g][2] = f4.z; fr[g][3] = f4.w;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool in = i0 + k < n;
                sz[g][k] = in ? size[i0 + k] : 0;          // size 0 marks an empty slot
                al[g][k] = in ? alloc[i0 + k] : 0;
                fr[g][k] = in ? free_[i0 + k] : 0;
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (sz[g][k]) { lo = min(lo, al[g][k]); hi = max(hi, fr[g][k]); }
    }
    for (int m = WAVE / 2; m > 0; m >>= 1) {
        lo = min(lo, (uint32_t)__shfl_xor(lo, m, WAVE));
        hi = max(hi, (uint32_t)__shfl_xor(hi, m, WAVE));
    }
    if ((threadIdx.x & (WAVE - 1)) == 0) { atomicMin(&s_lo, lo); atomicMax(&s_hi, hi); }
    __syncthreads();
    lo = s_lo; hi = s_hi;
    if (lo > hi) return;                               // nothing in this block
    const bool local = (hi - lo + 1) <= lds_bins;
    if (local) {
        const uint32_t nb = hi - lo + 1;
        for (uint32_t i = threadIdx.x; i < nb; i += blockDim.x) bins[i] = 0;
        __syncthreads();
#pragma unroll
        for (int g = 0; g < DW_GROUPS; ++g)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (sz[g][k]) {
                    atomicAdd(&bins[al[g][k] - lo], (unsigned long long)sz[g][k]);
                    atomicAdd(&bins[fr[g][k] - lo], (unsigned long long)(0ull - sz[g][k]));
                }
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < nb; i += blockDim.x) {
            const unsigned long long v = bins[i];
            if (v) atomicAdd(&delta[lo + i], v);
        }
    } else {
#pragma unroll
        for (int g = 0; g < DW_GROUPS; ++g)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (sz[g][k]) {
                    atomicAdd(&delta[al[g][k]], (unsigned long long)sz[g][k]);
                    atomicAdd(&delta[fr[g][k]], (unsigned long long)(0ull - sz[g][k]));
                }
    }
}

// One workgroup: inclusive prefix sum of delta[0..T) -> load, running maximum
// and earliest argmax.  ITEMS consecutive bins per thread, wave scan, LDS
// carry between waves, register carry between tiles.
constexpr int SCAN_THREADS = 1024;
constexpr int SCAN_ITEMS = 4;

__global__ __launch_bounds__(SCAN_THREADS) void k_scan_peak(uint32_t T, const uint64_t *__restrict__ delta,
                                                            uint64_t *__restrict__ load,
                                                            uint64_t *__restrict__ peak, uint32_t *__restrict__ t_peak)
{
    __shared__ uint64_t wsum[SCAN_THREADS / WAVE];
    __shared__ uint64_t wmax[SCAN_THREADS / WAVE];
    __shared__ uint32_t warg[SCAN_THREADS / WAVE];
    const int tid = threadIdx.x, l = tid & (WAVE - 1), w = tid / WAVE;
    uint64_t carry = 0, best = 0;
    uint32_t best_t = 0;
    bool have = false;
    for (uint32_t base = 0; base < T; base += SCAN_THREADS * SCAN_ITEMS) {
        const uint32_t t0 = base + tid * SCAN_ITEMS;
        uint64_t v[SCAN_ITEMS];
        uint64_t sum = 0;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            v[k] = (t0 + k < T) ? delta[t0 + k] : 0;
            sum += v[k];
        }
        const uint64_t incl = wave_scan_add(sum);
        if (l == WAVE - 1) wsum[w] = incl;
        __syncthreads();
        uint64_t pre = carry;
        for (int k = 0; k < w; ++k) pre += wsum[k];
        uint64_t total = 0;
        for (int k = 0; k < SCAN_THREADS / WAVE; ++k) total += wsum[k];
        uint64_t run = pre + incl - sum;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            run += v[k];
            if (t0 + k < T) {
                load[t0 + k] = run;
                if (!have || run > best) { best = run; best_t = t0 + k; have = true; }
            }
        }
        carry += total;
        __syncthreads();
    }
    // (value, earliest step) reduction
    if (!have) { best = 0; best_t = 0xFFFFFFFFu; }
    for (int m = WAVE / 2; m > 0; m >>= 1) {
        const uint64_t ov = shfl_xor64(best, m);
        const uint32_t ot = (uint32_t)__shfl_xor(best_t, m, WAVE);
        if (ov > best || (ov == best && ot < best_t)) { best = ov; best_t = ot; }
    }
    if (l == 0) { wmax[w] = best; warg[w] = best_t; }
    __syncthreads();
    if (tid == 0) {
        for (int k = 1; k < SCAN_THREADS / WAVE; ++k)
            if (wmax[k] > best || (wmax[k] == best && warg[k] < best_t)) { best = wmax[k]; best_t = warg[k]; }
        *peak = best;
        *t_peak = best_t;
    }
}

// Long time lines: the same scan in four small launches, tiles of SCAN_THREADS * SCAN_ITEMS steps.
//   1  every tile scans itself into load[] (the last entry of a tile is the tile's total)
//   2  one workgroup turns the tile totals into tile offsets; delta[] is no longer needed as input
//      and takes them (delta[0 .. nb))
//   3  every tile adds its offset and notes its largest value and the earliest step that has it
//      (delta[nb .. 2nb) and delta[2nb .. 3nb))
//   4  one workgroup reduces those to the peak and the peak step
constexpr uint32_t SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

__global__ __launch_bounds__(SCAN_THREADS) void k_scan_tile_local(uint32_t T, const uint64_t *__restrict__ delta,
                                                                  uint64_t *__restrict__ load)
{
    __shared__ uint64_t wsum[SCAN_THREADS / WAVE];
    const int tid = threadIdx.x, l = tid & (WAVE - 1), w = tid / WAVE;
    const uint32_t t0 = blockIdx.x * SCAN_TILE + tid * SCAN_ITEMS;
    uint64_t v[SCAN_ITEMS], sum = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        v[k] = (t0 + k < T) ? delta[t0 + k] : 0;
        sum += v[k];
    }
    const uint64_t incl = wave_scan_add(sum);
    if (l == WAVE - 1) wsum[w] = incl;
    __syncthreads();
    uint64_t run = incl - sum;
    for (int k = 0; k < w; ++k) run += wsum[k];
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        run += v[k];
        if (t0 + k < T) load[t0 + k] = run;
    }
}

__global__ __launch_bounds__(SCAN_THREADS) void k_scan_tile_offsets(uint32_t T, uint32_t nb,
                                                                    const uint64_t *__restrict__ load,
                                                                    uint64_t *__restrict__ offs)
{
    __shared__ uint64_t wsum[SCAN_THREADS / WAVE];
    const int tid = threadIdx.x, l = tid & (WAVE - 1), w = tid / WAVE;
    uint64_t carry = 0;
    for (uint32_t base = 0; base < nb; base += SCAN_THREADS) {
        const uint32_t j = base + tid;
        const uint64_t tot = j < nb ? load[min(T, (j + 1) * SCAN_TILE) - 1] : 0;
        const uint64_t incl = wave_scan_add(tot);
        if (l == WAVE - 1) wsum[w] = incl;
        __syncthreads();
        uint64_t pre = carry, all = 0;
        for (int k = 0; k < SCAN_THREADS / WAVE; ++k) { if (k < w) pre += wsum[k]; all += wsum[k]; }
        if (j < nb) offs[j] = pre + incl - tot;
        carry += all;
        __syncthreads();
    }
}

__global__ __launch_bounds__(SCAN_THREADS) void k_scan_tile_apply(uint32_t T, uint32_t nb, uint64_t *__restrict__ load,
                                                                  uint64_t *scratch)
{
    __shared__ uint64_t wmax[SCAN_THREADS / WAVE];
    __shared__ uint32_t warg[SCAN_THREADS / WAVE];
    const int tid = threadIdx.x, l = tid & (WAVE - 1), w = tid / WAVE;
    const uint32_t b = blockIdx.x, t0 = b * SCAN_TILE + tid * SCAN_ITEMS;
    const uint64_t off = scratch[b];
    uint64_t best = 0;
    uint32_t best_t = 0xFFFFFFFFu;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (t0 + k < T) {
            const uint64_t x = load[t0 + k] + off;
            load[t0 + k] = x;
            if (best_t == 0xFFFFFFFFu || x > best) { best = x; best_t = t0 + k; }
        }
    }
    for (int m = WAVE / 2; m > 0; m >>= 1) {
        const uint64_t ov = shfl_xor64(best, m);
        const uint32_t ot = (uint32_t)__shfl_xor(best_t, m, WAVE);
        if (ov > best || (ov == best && ot < best_t)) { best = ov; best_t = ot; }
    }
    if (l == 0) { wmax[w] = best; warg[w] = best_t; }
    __syncthreads();
    if (tid == 0) {
        for (int k = 1; k < SCAN_THREADS / WAVE; ++k)
            if (wmax[k] > best || (wmax[k] == best && warg[k] < best_t)) { best = wmax[k]; best_t = warg[k]; }
        scratch[nb + b] = best;
        scratch[2 * nb + b] = best_t;
    }
}

__global__ __launch_bounds__(SCAN_THREADS) void k_scan_tile_peak(uint32_t nb, const uint64_t *__restrict__ scratch,
                                                                 uint64_t *__restrict__ peak,
                                                                 uint32_t *__restrict__ t_peak)
{
    __shared__ uint64_t wmax[SCAN_THREADS / WAVE];
    __shared__ uint32_t warg[SCAN_THREADS / WAVE];
    const int tid = threadIdx.x, l = tid & (WAVE - 1), w = tid / WAVE;
    uint64_t best = 0;
    uint32_t best_t = 0xFFFFFFFFu;
    for (uint32_t j = tid; j < nb; j += SCAN_THREADS) {
        const uint64_t x = scratch[nb + j];
        const uint32_t at = (uint32_t)scratch[2 * nb + j];
        if (x > best || (x == best && at < best_t)) { best = x; best_t = at; }
    }
    for (int m = WAVE / 2; m > 0; m >>= 1) {
        const uint64_t ov = shfl_xor64(best, m);
        const uint32_t ot = (uint32_t)__shfl_xor(best_t, m, WAVE);
        if (ov > best || (ov == best && ot < best_t)) { best = ov; best_t = ot; }
    }
    if (l == 0) { wmax[w] = best; warg[w] = best_t; }
    __syncthreads();
    if (tid == 0) {
        for (int k = 1; k < SCAN_THREADS / WAVE; ++k)
            if (wmax[k] > best || (wmax[k] == best && warg[k] < best_t)) { best = wmax[k]; best_t = warg[k]; }
        *peak = best;
        *t_peak = best_t;
    }
}

// Trace content checks (flags[0] = trace error, flags[1] = a size >= 2^53),
// and the sums the range checks need: sizes split in 32-bit halves so that
// neither partial sum can overflow, max size, and the same for step_ns.
__global__ __launch_bounds__(256) void k_validate(uint32_t n, uint32_t T, const uint64_t *__restrict__ size,
                                                  const uint32_t *__restrict__ alloc,
                                                  const uint32_t *__restrict__ free_,
                                                  const uint32_t *__restrict__ gap_lo,
                                                  const uint32_t *__restrict__ gap_hi,
                                                  const uint64_t *__restrict__ step_ns,
                                                  unsigned long long *out /* [8] zeroed */)
{
    const uint32_t stride = gridDim.x * blockDim.x;
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    unsigned long long bad = 0, big = 0, lo = 0, hi = 0, mx = 0, nlo = 0, nhi = 0;
    for (uint32_t i = g; i < n; i += stride) {
        const uint64_t s = size[i];
        const uint32_t a = alloc[i], f = free_[i];
        if (s == 0 || a >= f || f > T) bad = 1;
        if (gap_lo && (a < f) && (gap_lo[i] < a || gap_hi[i] > f - 1 || gap_lo[i] > gap_hi[i])) bad = 1;
        if (s >= (1ull << 53)) big = 1;
        lo += s & 0xFFFFFFFFull;
        hi += s >> 32;
        mx = s > mx ? s : mx;
    }
    if (step_ns)
        for (uint32_t t = g; t < T; t += stride) {
            const uint64_t ns = step_ns[t];
            if (ns == 0) bad = 1;
            if (ns >= (1ull << 53)) big = 1;
            nlo += ns & 0xFFFFFFFFull;
            nhi += ns >> 32;
        }
    if (bad) atomicOr(&out[0], 1ull);
    if (big) atomicOr(&out[1], 1ull);
    lo = wave_reduce_add(lo); hi = wave_reduce_add(hi); mx = wave_reduce_max(mx);
    nlo = wave_reduce_add(nlo); nhi = wave_reduce_add(nhi);
    if ((threadIdx.x & (WAVE - 1)) == 0) {
        atomicAdd(&out[2], lo); atomicAdd(&out[3], hi); atomicMax(&out[4], mx);
        atomicAdd(&out[5], nlo); atomicAdd(&out[6], nhi);
    }
}

// ---------------------------------------------------------------------------

hipError_t launch_fill_u64(uint64_t *p, size_t n, uint64_t v, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    const int threads = 256;
    const size_t want = (n + threads - 1) / threads;
    const int blocks = (int)(want < 2048 ? want : 2048);
    hipLaunchKernelGGL(k_fill_u64, dim3(blocks), dim3(threads), 0, st, p, n, v);
    return hipGetLastError();
}

hipError_t launch_put_words(void *dst, const void *host_src, size_t n_words, hipStream_t st)
{
    const uint32_t *src = (const uint32_t *)host_src;
    uint32_t *d = (uint32_t *)dst;
    for (size_t done = 0; done < n_words; done += PUT_WORDS) {
        PutChunk c;
        const uint32_t cnt = (uint32_t)(n_words - done < PUT_WORDS ? n_words - done : PUT_WORDS);
        memcpy(c.w, src + done, (size_t)cnt * 4);
        hipLaunchKernelGGL(k_put_words, dim3(1), dim3(256), 0, st, d + done, cnt, c);
    }
    return hipGetLastError();
}

hipError_t launch_delta(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                        uint64_t *delta, hipStream_t st)
{
    const uint32_t nbins = T + 1;
    constexpr uint32_t LDS_BINS = 8192;            // 64 KiB of u64 bins per workgroup
    if (nbins <= LDS_BINS) {
        uint32_t blocks = (n + 256 * 16 - 1) / (256 * 16);
        blocks = blocks < 1 ? 1 : (blocks > 1024 ? 1024 : blocks);
        hipLaunchKernelGGL(k_delta_lds, dim3(blocks), dim3(256), nbins * sizeof(uint64_t), st, n, nbins, size, alloc,
                           free_, (unsigned long long *)delta);
    } else {
        constexpr uint32_t WIN_BINS = 2048;        // 16 KiB of bins: several workgroups per CU
        const uint32_t blocks = (n + DW_PER_BLOCK - 1) / DW_PER_BLOCK;
        hipLaunchKernelGGL(k_delta_window, dim3(blocks), dim3(DW_THREADS), WIN_BINS * sizeof(uint64_t), st, n,
                           WIN_BINS, size, alloc, free_, (unsigned long long *)delta);
    }
    return hipGetLastError();
}

hipError_t launch_scan_peak(uint32_t T, uint64_t *delta, uint64_t *load, uint64_t *peak, uint32_t *t_peak,
                            hipStream_t st)
{
    const uint32_t nb = (T + SCAN_TILE - 1) / SCAN_TILE;
    if (nb < 8) {
        hipLaunchKernelGGL(k_scan_peak, dim3(1), dim3(SCAN_THREADS), 0, st, T, delta, load, peak, t_peak);
        return hipGetLastError();
    }
    // 3 * nb <= T + 1 entries of delta serve as scratch once the tiles have been read
    hipLaunchKernelGGL(k_scan_tile_local, dim3(nb), dim3(SCAN_THREADS), 0, st, T, delta, load);
    hipLaunchKernelGGL(k_scan_tile_offsets, dim3(1), dim3(SCAN_THREADS), 0, st, T, nb, load, delta);
    hipLaunchKernelGGL(k_scan_tile_apply, dim3(nb), dim3(SCAN_THREADS), 0, st, T, nb, load, delta);
    hipLaunchKernelGGL(k_scan_tile_peak, dim3(1), dim3(SCAN_THREADS), 0, st, nb, delta, peak, t_peak);
    return hipGetLastError();
}

hipError_t launch_validate(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                           const uint32_t *gap_lo, const uint32_t *gap_hi, const uint64_t *step_ns, uint64_t *out8,
                           hipStream_t st)
{
    uint32_t blocks = (n + 255) / 256;
    blocks = blocks > 1024 ? 1024 : blocks;
    hipLaunchKernelGGL(k_validate, dim3(blocks), dim3(256), 0, st, n, T, size, alloc, free_, gap_lo, gap_hi, step_ns,
                       (unsigned long long *)out8);
    return hipGetLastError();
}

}  // namespace lap
