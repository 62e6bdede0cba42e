// Placement orders (Section III-C sorts by size, largest first; the other
// kinds are the extra heuristic orders evaluated in parallel).
//
// One workgroup per ordering produces perm[b][rank] = variable index: a stable
// least-significant-digit radix sort (8-bit digits) of the indices 0..N-1 by a
// 64-bit key.  The key is a pure function of (ordering, index) and is
// recomputed from the trace on every pass, so only the 4-byte indices move.
// Descending kinds sort the bitwise complement of the key; stability keeps
// equal keys in ascending index order.  A pass whose digit is the same for
// every variable is skipped.  The seeded shuffles' keys are distinct and spread
// over all 64 bits, so only their top 24 bits (32 for very large N, and for the
// shuffle inside size classes, whose top 6 bits are the class) are radix
// sorted; the few runs of variables that share those bits are then put in order
// by their full keys, one thread per run.
#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

__device__ __forceinline__ uint64_t order_key(uint32_t kind, uint64_t seed, uint32_t i,
                                              const uint64_t *__restrict__ size,
                                              const uint32_t *__restrict__ alloc,
                                              const uint32_t *__restrict__ free_)
{
    switch (kind) {
    case 0: return ~size[i];
    case 1: return ~(uint64_t)(free_[i] - alloc[i]);
    case 2: return ~(size[i] * (uint64_t)(free_[i] - alloc[i]));
    case 3: return (uint64_t)alloc[i];
    case 6: {
        // size class (floor(log2 size)) descending in the top 6 bits, then the shuffle key
        const uint64_t c = (uint64_t)__clzll((long long)size[i]);          // 63 - class
        return (c << 58) | (mix64(seed, i) >> 6);
    }
    default: return mix64(seed, i);
    }
}

// full comparison of two variables of a seeded kind (4 or 6): the radix key above drops the
// low bits of the shuffle key, the order does not
__device__ __forceinline__ bool seeded_after(uint32_t kind, uint64_t seed, uint32_t x, uint32_t y,
                                             const uint64_t *__restrict__ size)
{
    if (kind == 6) {
        const int cx = __clzll((long long)size[x]), cy = __clzll((long long)size[y]);
        if (cx != cy) return cx > cy;
    }
    return mix64(seed, x) > mix64(seed, y);
}

constexpr int SW = 4;                    // waves per ordering

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

constexpr uint32_t TS = 4096;            // ranks per tile of a scatter pass
constexpr int SUB = TS / (SW * WAVE);    // 64-rank sub-tiles per wave and tile

// One radix pass = a histogram of the digit over all ranks, then tile after tile of TS ranks:
// every wave counts the digits of its quarter of the tile, the workgroup turns the 4 x 256 counts
// into positions inside the tile (digit-major, wave-minor, sub-tile order within a wave: stable),
// the waves put their indices there in an LDS staging area, and the staged tile -- now grouped by
// digit -- is written out, so that equal digits go to consecutive addresses instead of one
// 4-byte store per cache line.
__global__ __launch_bounds__(SW *WAVE) void k_sort_perm(uint32_t n, const uint64_t *__restrict__ size,
                                                        const uint32_t *__restrict__ alloc,
                                                        const uint32_t *__restrict__ free_,
                                                        const uint32_t *__restrict__ kinds,
                                                        const uint64_t *__restrict__ seeds,
                                                        uint32_t *perm_all, uint32_t *tmp_all)
{
    __shared__ uint32_t hist[SW][256];
    __shared__ uint32_t tile_off[256];       // per digit: address in dst minus position in the staged tile
    __shared__ uint32_t stage[TS];
    __shared__ uint8_t stage_d[TS];          // the digit of every staged index
    __shared__ uint32_t wtot[SW];
    __shared__ uint64_t s_or[SW], s_and[SW];
    __shared__ uint32_t hist_all[8][256];    // the digit counts of all passes, counted in one sweep
    const uint32_t b = blockIdx.x;
    const int l = lane_id();
    const uint32_t tid = threadIdx.x, w = tid / WAVE;
    const uint32_t kind = kinds[b];
    const uint64_t seed = seeds[b];
    uint32_t *perm = perm_all + (size_t)b * n;
    uint32_t *tmp = tmp_all + (size_t)b * n;

    if (kind == 5) {
        // caller-supplied permutation: copy.  Indices are clamped so that a malformed
        // array can never cause an out-of-range access downstream.
        const uint32_t *src = (const uint32_t *)(uintptr_t)seed;
        for (uint32_t i = tid; i < n; i += SW * WAVE) perm[i] = min(src[i], n - 1);
        return;
    }
    // The few orderings by a fixed heuristic need more passes than the many seeded ones that share
    // their compute units, and the launch ends with the slowest workgroup: their waves go first.
    if (kind < 4) __builtin_amdgcn_s_setprio(3);

    // exclusive scan over the 256 digit owners (thread d owns digit d); returns the value before d.
    // The callers pass a workgroup barrier between one call and the next.
    auto scan256 = [&](uint32_t v) -> uint32_t {
        uint32_t incl = v;
#pragma unroll
        for (int dlt = 1; dlt < WAVE; dlt <<= 1) {
            const uint32_t t = __shfl_up(incl, dlt, WAVE);
            if (l >= dlt) incl += t;
        }
        if (l == WAVE - 1) wtot[w] = incl;
        __syncthreads();
        uint32_t run = incl - v;
        for (uint32_t k = 0; k < w; ++k) run += wtot[k];
        return run;
    };

    // cur == nullptr means the identity (no buffer read yet)
    const uint32_t *cur = nullptr;
    uint32_t *dst = perm;
    const uint64_t lt_mask = (1ull << l) - 1ull;
    const int first_pass = (kind == 4) ? (n <= (1u << 22) ? 5 : 4) : (kind == 6) ? 4 : 0;
    // Key bits that differ between variables: a pass whose digit has none of them moves nothing.
    // The seeded kinds sort their top digits whatever the keys are.
    uint64_t vary = ~0ull << (first_pass * 8);
    if (!first_pass) {
        uint64_t o = 0, a = ~0ull;
        for (uint32_t i = tid; i < n; i += SW * WAVE) {
            const uint64_t key = order_key(kind, seed, i, size, alloc, free_);
            o |= key; a &= key;
        }
#pragma unroll
        for (int dlt = 1; dlt < WAVE; dlt <<= 1) {
            o |= (uint64_t)__shfl_xor((unsigned long long)o, dlt, WAVE);
            a &= (uint64_t)__shfl_xor((unsigned long long)a, dlt, WAVE);
        }
        if (l == 0) { s_or[w] = o; s_and[w] = a; }
        __syncthreads();
        o = 0; a = ~0ull;
#pragma unroll
        for (int k = 0; k < SW; ++k) { o |= s_or[k]; a &= s_and[k]; }
        const uint64_t v = o ^ a;               // alike in all lanes: to scalar registers
        vary = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(v >> 32)) << 32) |
               (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    }
    // How often a digit occurs does not depend on the order of the ranks, so the counts of all
    // the passes come from one sweep over the variables in index order (no read of the ranks
    // at all) instead of one sweep per pass.
#pragma unroll
    for (int q = 0; q < 8; ++q) hist_all[q][tid] = 0;
    __syncthreads();
    for (uint32_t i = tid; i < n; i += SW * WAVE) {
        const uint64_t key = order_key(kind, seed, i, size, alloc, free_);
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if ((vary >> (q * 8)) & 255u) atomicAdd(&hist_all[q][(uint32_t)(key >> (q * 8)) & 255u], 1u);
    }
    __syncthreads();
    for (int pass = first_pass; pass < 8; ++pass) {
        const int shift = pass * 8;
        if (!((vary >> shift) & 255u)) continue;      // every key has the same digit: nothing moves
        // thread d keeps, in a register, where the next entry of digit d goes in dst
        uint32_t gb = scan256(hist_all[pass][tid]);

        // ---- tiles
        for (uint32_t tb = 0; tb < n; tb += TS) {
            hist[w][l] = 0; hist[w][l + 64] = 0; hist[w][l + 128] = 0; hist[w][l + 192] = 0;
            wave_lds_sync();
            uint32_t iv[SUB], dv[SUB];
#pragma unroll
            for (int k = 0; k < SUB; ++k) {
                const uint32_t r = tb + (w * SUB + k) * WAVE + l;
                iv[k] = r < n ? (cur ? cur[r] : r) : 0u;
            }
#pragma unroll
            for (int k = 0; k < SUB; ++k) {
                const uint32_t r = tb + (w * SUB + k) * WAVE + l;
                dv[k] = 256u;
                if (r < n) {
                    dv[k] = (uint32_t)(order_key(kind, seed, iv[k], size, alloc, free_) >> shift) & 255u;
                    atomicAdd(&hist[w][dv[k]], 1u);
                }
            }
            __syncthreads();
            // digit owner: where the tile's entries of this digit start, per wave
            uint32_t c[SW], ttot = 0;
#pragma unroll
            for (int k = 0; k < SW; ++k) { c[k] = hist[k][tid]; ttot += c[k]; }
            uint32_t run = scan256(ttot);
            tile_off[tid] = gb - run;
            gb += ttot;
#pragma unroll
            for (int k = 0; k < SW; ++k) { hist[k][tid] = run; run += c[k]; }
            __syncthreads();
            // stable placement of this wave's sub-tiles into the staging area
#pragma unroll
            for (int k = 0; k < SUB; ++k) {
                const uint32_t d = dv[k];
                const bool act = d < 256u;
                uint64_t same = ballot(act);
#pragma unroll
                for (int bit = 0; bit < 8; ++bit) {
                    const uint64_t m = ballot(act && ((d >> bit) & 1u));
                    same &= ((d >> bit) & 1u) ? m : ~m;
                }
                const uint32_t rank = (uint32_t)__popcll(same & lt_mask);
                const uint32_t cnt = (uint32_t)__popcll(same);
                // The first lane of every group of equal digits takes the group's positions.  The LDS unit
                // serves a wave's requests in the order they were issued, so the sub-tiles take theirs in
                // order without waiting for one another.
                uint32_t base = 0;
                if (act && rank == 0) base = atomicAdd(&hist[w][d], cnt);
                const uint32_t pos = (uint32_t)__shfl((int)base, act ? __builtin_ctzll(same) : 0, WAVE) + rank;
                if (act) { stage[pos] = iv[k]; stage_d[pos] = (uint8_t)d; }
                if ((k & 3) == 3) __builtin_amdgcn_sched_barrier(0);     // four sub-tiles in flight, not all
            }
            __syncthreads();
            // The staged tile, grouped by digit, goes out: equal digits to consecutive addresses.  The
            // next tile's first barrier comes before anything read here is written again.
            const uint32_t tn = min(TS, n - tb);
            for (uint32_t p = tid; p < tn; p += SW * WAVE) dst[p + tile_off[stage_d[p]]] = stage[p];
        }
        __syncthreads();                                      // the next pass reads what this one wrote
        cur = dst;
        dst = (dst == perm) ? tmp : perm;
    }
    if (cur == nullptr) {
        for (uint32_t i = threadIdx.x; i < n; i += SW * WAVE) perm[i] = i;
    } else if (cur != perm) {
        for (uint32_t i = threadIdx.x; i < n; i += SW * WAVE) perm[i] = tmp[i];
    }
    if (first_pass == 0) return;
    // Runs of equal sorted bits: the thread at a run's first rank sorts the run by the full
    // key (insertion sort; the shuffle keys of one seed are distinct).  Every entry a run
    // moves keeps the run's sorted bits, so the neighbours' run tests are not disturbed.
    __syncthreads();
    const int pshift = first_pass * 8;
    // A wave looks at 63 ranks per turn: lane 0 only hands the sorted bits of the rank before them to lane 1.
    for (uint32_t base = w * 63u; base < n; base += SW * 63u) {
        const uint32_t r = base + (uint32_t)l - 1u;
        const bool have = r < n;                                                 // not so for rank "-1"
        uint64_t p0 = 0;
        if (have) p0 = order_key(kind, seed, perm[r], size, alloc, free_) >> pshift;
        const uint64_t before = (uint64_t)__shfl_up((unsigned long long)p0, 1, WAVE);
        if (l == 0 || !have) continue;
        if (r > 0 && before == p0) continue;                                     // not a run's first rank
        uint32_t m = 1;
        while (r + m < n && (order_key(kind, seed, perm[r + m], size, alloc, free_) >> pshift) == p0) ++m;
        for (uint32_t x = 1; x < m; ++x) {
            const uint32_t vi = perm[r + x];
            uint32_t y = x;
            while (y > 0 && seeded_after(kind, seed, perm[r + y - 1], vi, size)) { perm[r + y] = perm[r + y - 1]; --y; }
            perm[r + y] = vi;
        }
    }
}

// A caller-supplied order must be a permutation of 0..N-1.  One that is not (an index out of
// range, or one used twice) is replaced by the identity order, so that every variable is
// still placed exactly once.  tmp is free after the sort and serves as the "seen" marks.
__global__ __launch_bounds__(256) void k_sanitize_explicit(uint32_t n, const uint32_t *__restrict__ kinds,
                                                           const uint64_t *__restrict__ seeds, uint32_t *perm_all,
                                                           uint32_t *tmp_all)
{
    const uint32_t b = blockIdx.x;
    if (kinds[b] != 5) return;
    __shared__ uint32_t s_bad;
    const uint32_t *src = (const uint32_t *)(uintptr_t)seeds[b];
    uint32_t *perm = perm_all + (size_t)b * n;
    uint32_t *seen = tmp_all + (size_t)b * n;
    if (threadIdx.x == 0) s_bad = 0;
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) seen[i] = 0;
    __syncthreads();
    bool bad = false;
    for (uint32_t r = threadIdx.x; r < n; r += blockDim.x) {
        const uint32_t v = src[r];
        if (v >= n) bad = true;
        else if (atomicAdd(&seen[v], 1u) != 0) bad = true;
    }
    if (bad) s_bad = 1;
    __syncthreads();
    if (s_bad)
        for (uint32_t r = threadIdx.x; r < n; r += blockDim.x) perm[r] = r;
}

hipError_t launch_sort_perm(uint32_t n, uint32_t B, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                            const uint32_t *kinds, const uint64_t *seeds, uint32_t *perm, uint32_t *tmp,
                            bool any_explicit, hipStream_t st)
{
    hipLaunchKernelGGL(k_sort_perm, dim3(B), dim3(SW * WAVE), 0, st, n, size, alloc, free_, kinds, seeds, perm, tmp);
    if (any_explicit)
        hipLaunchKernelGGL(k_sanitize_explicit, dim3(B), dim3(256), 0, st, n, kinds, seeds, perm, tmp);
    return hipGetLastError();
}

}  // namespace lap
