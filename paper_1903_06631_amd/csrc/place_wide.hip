// Placement of every variable under many orderings (Section III-C), first-fit or
// best-fit: the 64-bit path, used when byte offsets do not fit 32-bit granules (see
// place_fast.hip for the common case).
//
// One wave (one 64-thread workgroup) per ordering.  Variables are taken in
// the ordering's rank order; each gets the lowest offset at which its block
// does not meet the block of any already-placed variable whose lifetime
// overlaps its own (first-fit: the lowest hole that is large enough, else
// above the highest neighbour, Section III-C).  Best-fit walks on from hole to hole (next_overlap gives a
// hole's end) and keeps the smallest one that fits.
//
// Data structure per ordering: the placed blocks kept SORTED BY OFFSET, as
//   main    (global memory)  off[], end[], life[] (alloc<<32 | free), nm entries
//   recent  (LDS)            the last < RECENT placements, also sorted
// A query sweeps a sorted list once, 64 entries per step: entries that do not
// overlap the variable in time are masked out, a wave prefix-maximum of the
// remaining ends gives "highest occupied address so far", and the first entry
// whose offset leaves a hole of at least `size` above it ends the sweep (early
// exit).  main and recent are swept alternately, each resuming from its own
// cursor, until neither moves the candidate offset.  New blocks are inserted
// into recent; when recent is full it is merged into main in place.
#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

constexpr uint32_t RECENT = 512;

// Lowest offset >= P at which a block of `s` bytes is free with respect to the
// time-overlapping entries of one sorted list.  `cursor` is where the sweep
// starts and where it stopped; every time-overlapping entry before it ends at
// or below the returned offset, so a later call with a larger P may resume.
__device__ __forceinline__ uint64_t sweep(const uint64_t *off, const uint64_t *end, const uint64_t *life,
                                          uint32_t n, uint32_t &cursor, uint64_t P, uint64_t s, uint32_t a,
                                          uint32_t f)
{
    const int l = lane_id();
    uint32_t i = cursor;
    for (;;) {
        const uint32_t idx = i + l;
        uint64_t o = U64_MAX, e = 0;
        if (idx < n) {
            o = off[idx];
            const uint64_t lf = life[idx];
            const uint32_t ea = (uint32_t)(lf >> 32), ef = (uint32_t)lf;
            if (ea < f && a < ef) e = end[idx];
        }
        const uint64_t incl = wave_scan_max(e);
        uint64_t excl = shfl_up64(incl, 1);
        if (l == 0) excl = 0;
        const uint64_t before = umax64(P, excl);
        // lanes past the end of the list carry o = 2^64-1 and always report a hole
        const uint64_t hole = ballot(o >= before + s);
        if (hole) {
            const int first = __ffsll((unsigned long long)hole) - 1;
            cursor = i + first;
            return shfl64(before, first);
        }
        P = umax64(P, shfl64(incl, WAVE - 1));
        i += WAVE;
    }
}

// offset of the first entry at or after index `from` that overlaps [a, f) in time, 2^64-1 if none
__device__ __forceinline__ uint64_t next_overlap(const uint64_t *off, const uint64_t *life, uint32_t n,
                                                 uint32_t from, uint32_t a, uint32_t f)
{
    const int l = lane_id();
    for (uint32_t base = from; base < n; base += WAVE) {
        const uint32_t idx = base + l;
        bool hit = false;
        uint64_t o = 0;
        if (idx < n) {
            const uint64_t lf = life[idx];
            hit = (uint32_t)(lf >> 32) < f && a < (uint32_t)lf;
            o = off[idx];
        }
        const uint64_t m = ballot(hit);
        if (m) return shfl64(o, __ffsll((unsigned long long)m) - 1);
    }
    return U64_MAX;
}

// number of entries of a sorted list with off < key (all lanes get the result)
__device__ __forceinline__ uint32_t count_below(const uint64_t *off, uint32_t n, uint64_t key)
{
    const int l = lane_id();
    uint32_t p = 0;
    for (uint32_t base = 0; base < n; base += WAVE) {
        const uint32_t idx = base + l;
        const uint64_t m = ballot(idx < n && off[idx] < key);
        p += (uint32_t)__popcll(m);
        if (m != ~0ull) break;            // sorted: nothing further can be below
    }
    return p;
}

// insert one entry at position p of a sorted list of n entries (capacity > n); LDS or global
__device__ __forceinline__ void insert_at(uint64_t *off, uint64_t *end, uint64_t *life, uint32_t n, uint32_t p,
                                          uint64_t o, uint64_t e, uint64_t lf)
{
    const int l = lane_id();
    uint32_t hi = n;
    while (hi > p) {
        const uint32_t lo = (hi - p > (uint32_t)WAVE) ? hi - WAVE : p;
        const uint32_t idx = lo + l;
        const bool act = idx < hi;
        uint64_t x = 0, y = 0, z = 0;
        if (act) { x = off[idx]; y = end[idx]; z = life[idx]; }
        __syncthreads();
        if (act) { off[idx + 1] = x; end[idx + 1] = y; life[idx + 1] = z; }
        __syncthreads();
        hi = lo;
    }
    if (l == 0) { off[p] = o; end[p] = e; life[p] = lf; }
    __syncthreads();
}

// Merge the full recent list (LDS, nr entries) into main (global, nm entries, capacity >= nm+nr),
// in place.  Ties: main entries stay below recent entries of equal offset.
__device__ __forceinline__ void merge_recent(uint64_t *m_off, uint64_t *m_end, uint64_t *m_life, uint32_t nm,
                                             const uint64_t *r_off, const uint64_t *r_end, const uint64_t *r_life,
                                             uint32_t nr)
{
    const int l = lane_id();
    constexpr int PER = RECENT / WAVE;
    uint32_t pos[PER];
    // final position of recent[j]: j + number of main entries with off <= its off
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const uint32_t j = k * WAVE + l;
        pos[k] = 0;
        if (j < nr) {
            const uint64_t key = r_off[j];
            uint32_t lo = 0, hi = nm;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (m_off[mid] <= key) lo = mid + 1; else hi = mid;
            }
            pos[k] = lo + j;
        }
    }
    __syncthreads();
    // move main entries up by the number of recent entries strictly below them, top chunk first
    uint32_t hi = nm;
    while (hi > 0) {
        const uint32_t lo = hi > (uint32_t)WAVE ? hi - WAVE : 0;
        const uint32_t idx = lo + l;
        const bool act = idx < hi;
        uint64_t x = 0, y = 0, z = 0;
        uint32_t sh = 0;
        if (act) {
            x = m_off[idx]; y = m_end[idx]; z = m_life[idx];
            uint32_t a = 0, b = nr;
            while (a < b) {
                const uint32_t mid = (a + b) >> 1;
                if (r_off[mid] < x) a = mid + 1; else b = mid;
            }
            sh = a;
        }
        __syncthreads();
        if (act && sh) { m_off[idx + sh] = x; m_end[idx + sh] = y; m_life[idx + sh] = z; }
        __syncthreads();
        hi = lo;
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const uint32_t j = k * WAVE + l;
        if (j < nr) { m_off[pos[k]] = r_off[j]; m_end[pos[k]] = r_end[j]; m_life[pos[k]] = r_life[j]; }
    }
    __syncthreads();
}

__global__ __launch_bounds__(64) void k_place_wide(uint32_t n, const uint64_t *__restrict__ size,
                                              const uint32_t *__restrict__ alloc,
                                              const uint32_t *__restrict__ free_,
                                              const uint32_t *__restrict__ perm_all,
                                              const uint32_t *__restrict__ fits,
                                              const PlanHeader *__restrict__ hdr,
                                              uint64_t *m_off_all, uint64_t *m_end_all, uint64_t *m_life_all,
                                              uint64_t *__restrict__ offs_all, uint64_t *__restrict__ fps,
                                              uint64_t *__restrict__ ticks)
{
    __shared__ uint64_t r_off[RECENT], r_end[RECENT], r_life[RECENT];
    if (hdr->fast) return;                 // the 32-bit granule kernel handles this trace
    const long long t_begin = wall_clock64();
    const uint32_t b = blockIdx.x;
    const int l = lane_id();
    const bool best_fit = fits[b] != 0;
    const uint32_t *perm = perm_all + (size_t)b * n;
    uint64_t *m_off = m_off_all + (size_t)b * n;
    uint64_t *m_end = m_end_all + (size_t)b * n;
    uint64_t *m_life = m_life_all + (size_t)b * n;
    uint64_t *offs = offs_all + (size_t)b * n;

    uint32_t nm = 0, nr = 0;
    uint64_t fp = 0;
    for (uint32_t r = 0; r < n; ++r) {
        const uint32_t v = perm[r];
        const uint64_t s = size[v];
        const uint32_t a = alloc[v], f = free_[v];

        uint64_t o = 0;
        uint32_t cm = 0, cr = 0;
        uint64_t best_gap = U64_MAX, best_off = 0;
        for (;;) {
            // lowest feasible offset >= o
            for (;;) {
                const uint64_t o1 = sweep(m_off, m_end, m_life, nm, cm, o, s, a, f);
                const uint64_t o2 = nr ? sweep(r_off, r_end, r_life, nr, cr, o1, s, a, f) : o1;
                o = o2;
                if (o2 == o1) break;
            }
            if (!best_fit) break;
            // best-fit: o starts a hole that fits; it ends at the next neighbour above (the sweeps
            // stopped at the first entry above the hole).  Smallest hole wins, the first of equals;
            // an exact fit ends the search; no neighbour above: o is the top of the neighbours.
            const uint64_t e = umin64(next_overlap(m_off, m_life, nm, cm, a, f),
                                      next_overlap(r_off, r_life, nr, cr, a, f));
            if (e == U64_MAX) { if (best_gap != U64_MAX) o = best_off; break; }
            const uint64_t gap = e - o;
            if (gap < best_gap) { best_gap = gap; best_off = o; }
            if (gap == s) break;
            o = e;
        }

        if (l == 0) offs[r] = o;                 // by rank: the result arrays are un-permuted afterwards
        fp = umax64(fp, o + s);

        const uint32_t p = count_below(r_off, nr, o);
        insert_at(r_off, r_end, r_life, nr, p, o, o + s, ((uint64_t)a << 32) | f);
        ++nr;
        if (nr == RECENT) {
            merge_recent(m_off, m_end, m_life, nm, r_off, r_end, r_life, nr);
            nm += nr;
            nr = 0;
        }
    }
    if (l == 0) {
        fps[b] = fp;
        ticks[b] = (uint64_t)(wall_clock64() - t_begin);      // how long this ordering took, in timer ticks
    }
}

// best = lowest index among the smallest footprints
__global__ __launch_bounds__(256) void k_select(uint32_t B, const uint64_t *__restrict__ fps,
                                                uint64_t *__restrict__ best_fp, uint32_t *__restrict__ best_idx)
{
    __shared__ uint64_t sv[256];
    __shared__ uint32_t si[256];
    uint64_t v = U64_MAX;
    uint32_t ix = 0xFFFFFFFFu;
    for (uint32_t b = threadIdx.x; b < B; b += blockDim.x) {
        const uint64_t x = fps[b];
        if (x < v || (x == v && b < ix)) { v = x; ix = b; }
    }
    sv[threadIdx.x] = v; si[threadIdx.x] = ix;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st) {
            const uint64_t x = sv[threadIdx.x + st];
            const uint32_t j = si[threadIdx.x + st];
            if (x < sv[threadIdx.x] || (x == sv[threadIdx.x] && j < si[threadIdx.x])) {
                sv[threadIdx.x] = x; si[threadIdx.x] = j;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) { *best_fp = sv[0]; *best_idx = si[0]; }
}

// The placement kernels leave their offsets in rank order (entry r belongs to variable
// perm[r]): stores of neighbouring ranks fall into the same cache lines.  The results asked for
// are put in variable order here: the best ordering's, and all B when the caller wants them.
__global__ __launch_bounds__(256) void k_copy_best(uint32_t n, const uint64_t *__restrict__ offs_rank,
                                                   const uint32_t *__restrict__ perm_all,
                                                   const uint32_t *__restrict__ best_idx,
                                                   uint64_t *__restrict__ best_offsets)
{
    const uint64_t *src = offs_rank + (size_t)(*best_idx) * n;
    const uint32_t *perm = perm_all + (size_t)(*best_idx) * n;
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) best_offsets[perm[i]] = src[i];
}

__global__ __launch_bounds__(256) void k_unpermute(uint32_t n, const uint64_t *__restrict__ offs_rank,
                                                   const uint32_t *__restrict__ perm_all,
                                                   uint64_t *__restrict__ all_offsets)
{
    const size_t b = blockIdx.y;
    const uint64_t *src = offs_rank + b * n;
    const uint32_t *perm = perm_all + b * n;
    uint64_t *dst = all_offsets + b * n;
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[perm[i]] = src[i];
}

hipError_t launch_place_wide(uint32_t n, uint32_t B, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                        const uint32_t *perm, const uint32_t *fits, const PlanHeader *hdr, uint64_t *m_off,
                        uint64_t *m_end, uint64_t *m_life, uint64_t *offs, uint64_t *fps, uint64_t *ticks,
                        hipStream_t st)
{
    hipLaunchKernelGGL(k_place_wide, dim3(B), dim3(WAVE), 0, st, n, size, alloc, free_, perm, fits, hdr, m_off,
                       m_end, m_life, offs, fps, ticks);
    return hipGetLastError();
}

hipError_t launch_select(uint32_t n, uint32_t B, const uint64_t *fps, const uint64_t *offs_rank, const uint32_t *perm,
                         uint64_t *best_fp, uint32_t *best_idx, uint64_t *best_offsets, uint64_t *all_offsets,
                         hipStream_t st)
{
    hipLaunchKernelGGL(k_select, dim3(1), dim3(256), 0, st, B, fps, best_fp, best_idx);
    uint32_t blocks = (n + 255) / 256;
    blocks = blocks > 1024 ? 1024 : blocks;
    hipLaunchKernelGGL(k_copy_best, dim3(blocks), dim3(256), 0, st, n, offs_rank, perm, best_idx, best_offsets);
    if (all_offsets) {
        blocks = blocks > 64 ? 64 : blocks;
        hipLaunchKernelGGL(k_unpermute, dim3(blocks, B), dim3(256), 0, st, n, offs_rank, perm, all_offsets);
    }
    return hipGetLastError();
}

}  // namespace lap
