// The swap schedule under a memory-load limit (Section IV-E): a Malloc that would exceed the limit
// waits until enough has been swapped out, a swap-in starts only when its bytes fit.  One iteration
// is replayed as a discrete-event machine with three actors (compute, the swap-out stream, the
// swap-in stream); the result is the time lost against the plain iteration.
//
// The machine is sequential; the parallel dimension is the set of (swap list prefix, limit) pairs to
// evaluate -- a sweep of limits, several priority orders -- one wave each, lane 0 running the
// machine.  Shared by all of them and built by data-parallel kernels: bytes allocated and freed per
// step, and the listed variables in swap-out order and in swap-in order (positions in the list, so
// that "the first k of the list" is a filter).
#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

constexpr int SIM_THREADS = 1024;
constexpr int SIM_WAVES = SIM_THREADS / WAVE;
constexpr uint32_t SIM_NONE = 0xFFFFFFFFu;

__global__ __launch_bounds__(256) void k_sim_steps(uint32_t n, const uint64_t *__restrict__ size,
                                                   const uint32_t *__restrict__ alloc,
                                                   const uint32_t *__restrict__ free_, unsigned long long *need,
                                                   unsigned long long *rel)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    atomicAdd(&need[alloc[i]], (unsigned long long)size[i]);
    atomicAdd(&rel[free_[i] - 1], (unsigned long long)size[i]);
}

// several lists, one row of n entries each: position map of list r = row r.  Row r lists the first
// n_listed[0] entries of its row of `lists`.
__global__ __launch_bounds__(256) void k_sim_mark_rows(uint32_t n, const uint32_t *__restrict__ lists,
                                                       const uint32_t *__restrict__ n_listed,
                                                       uint32_t *__restrict__ posmap)
{
    const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x, r = blockIdx.y;
    if (j < *n_listed) posmap[(size_t)r * n + min(lists[(size_t)r * n + j], n - 1)] = j;
}

// jobs[0..m) = list positions of the listed variables that have an idle gap, in the order of perm;
// one workgroup per list (rows of n entries of posmap and jobs, one count each)
__global__ __launch_bounds__(SIM_THREADS) void k_sim_jobs(uint32_t n, const uint32_t *__restrict__ perm,
                                                          const uint32_t *__restrict__ posmap_all,
                                                          const uint32_t *__restrict__ step_lo,
                                                          const uint32_t *__restrict__ step_hi, uint32_t hi_minus,
                                                          uint32_t *__restrict__ jobs_all,
                                                          uint32_t *__restrict__ m_all)
{
    __shared__ uint32_t wsum[SIM_WAVES];
    const uint32_t *posmap = posmap_all + (size_t)blockIdx.x * n;
    uint32_t *jobs = jobs_all + (size_t)blockIdx.x * n;
    uint32_t *m_out = m_all + blockIdx.x;
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    uint32_t carry = 0;
    for (uint32_t base = 0; base < n; base += SIM_THREADS) {
        const uint32_t r = base + tid;
        uint32_t pos = SIM_NONE;
        if (r < n) {
            const uint32_t v = perm[r];
            pos = posmap[v];
            if (pos != SIM_NONE && step_hi[v] - hi_minus <= step_lo[v]) pos = SIM_NONE;
        }
        const uint64_t mine = ballot(pos != SIM_NONE);
        const uint32_t before = (uint32_t)__popcll(mine & ((1ull << lane) - 1ull));
        if (lane == 0) wsum[wave] = (uint32_t)__popcll(mine);
        __syncthreads();
        uint32_t pre = 0, tot = 0;
        for (int q = 0; q < SIM_WAVES; ++q) { const uint32_t x = wsum[q]; if (q < (int)wave) pre += x; tot += x; }
        __syncthreads();
        if (pos != SIM_NONE) jobs[carry + pre + before] = pos;
        carry += tot;
    }
    if (tid == 0) *m_out = carry;
}

struct SimArgs {
    uint32_t n, T, Q, kmax;
    const uint64_t *size;
    const uint32_t *step_lo, *step_hi;
    uint32_t hi_minus;
    const uint64_t *C;
    const unsigned long long *need, *rel;
    const uint32_t *list;
    const uint32_t *jobs_lo, *jobs_hi, *m;
    const uint32_t *prefix;            // [Q]
    const uint64_t *limits;            // [Q]
    uint32_t *kb;                      // [Q][kmax] issue boundary of a swap-in, by list position
    uint8_t *out_done;                 // [Q][kmax]
    uint32_t per_run_lists;            // 1: run q has its own list (row q of list / jobs / m), 0: all share row 0
    uint64_t bpus;
    uint64_t *total_ns, *overhead_ns, *peak_resident;
    uint32_t *forced;
};

__global__ __launch_bounds__(WAVE) void k_sim_run(SimArgs A)
{
    if (threadIdx.x != 0) return;
    const uint32_t q = blockIdx.x;
    const size_t row = A.per_run_lists ? (size_t)q * A.n : 0;
    A.list += row;
    A.jobs_lo += row;
    A.jobs_hi += row;
    const uint32_t k = A.prefix[q], m = A.m[A.per_run_lists ? q : 0], T = A.T;
    const uint64_t limit = A.limits[q];
    uint32_t *kb = A.kb + (size_t)q * A.kmax;
    uint8_t *odone = A.out_done + (size_t)q * A.kmax;
    auto dur = [&](uint32_t v) { return (A.size[v] * 1000ull + A.bpus - 1) / A.bpus; };
    auto lo_of = [&](uint32_t pos) { return A.step_lo[A.list[pos]]; };
    auto hi_of = [&](uint32_t pos) { return A.step_hi[A.list[pos]] - A.hi_minus; };

    // the plan's swap-in starts, from the last access backwards; each gives the step boundary at
    // which the swap-in is issued
    {
        long long next_start = (1ll << 62);
        for (uint32_t jj = m; jj-- > 0;) {
            const uint32_t pos = A.jobs_hi[jj];
            if (pos >= k) continue;
            const uint32_t v = A.list[pos], th = hi_of(pos);
            const long long due = (long long)A.C[th];
            const long long st = (due < next_start ? due : next_start) - (long long)dur(v);
            next_start = st;
            uint32_t l0 = 0, h0 = th;                      // last t <= th with C[t] <= st (0 if none)
            while (l0 < h0) { const uint32_t mid = (l0 + h0 + 1) >> 1; if ((long long)A.C[mid] <= st) l0 = mid; else h0 = mid - 1; }
            kb[pos] = max(l0, lo_of(pos) + 1);
            odone[pos] = 0;
        }
    }

    uint64_t now = 0, R = 0, peak = 0;
    uint32_t t = 0, nforced = 0, boundary = 0;
    bool step_run = false, out_run = false, in_run = false;
    uint64_t step_end = 0, out_end = 0, in_end = 0;
    uint32_t o_iss = 0, o_next = 0, i_iss = 0, i_next = 0;   // indices into jobs_lo / jobs_hi
    auto skip_lo = [&](uint32_t p) { while (p < m && A.jobs_lo[p] >= k) ++p; return p; };
    auto skip_hi = [&](uint32_t p) { while (p < m && A.jobs_hi[p] >= k) ++p; return p; };
    auto issue_ins = [&]() {
        while (i_iss < m && (A.jobs_hi[i_iss] >= k || kb[A.jobs_hi[i_iss]] <= boundary)) ++i_iss;
    };
    o_next = skip_lo(0);
    i_next = skip_hi(0);
    issue_ins();
    for (;;) {
        // ends at this instant
        if (step_run && step_end == now) {
            step_run = false;
            R -= A.rel[t];
            while (o_iss < m && (A.jobs_lo[o_iss] >= k || lo_of(A.jobs_lo[o_iss]) <= t)) ++o_iss;
            ++t;
            boundary = t;
            issue_ins();
        }
        if (out_run && out_end == now) {
            out_run = false;
            const uint32_t pos = A.jobs_lo[o_next];
            R -= A.size[A.list[pos]];
            odone[pos] = 1;
            o_next = skip_lo(o_next + 1);
        }
        if (in_run && in_end == now) {
            in_run = false;
            i_next = skip_hi(i_next + 1);
        }
        if (t == T && !step_run) break;
        // starts: swap-out, step, swap-in
        if (!out_run && o_next < o_iss) {
            out_run = true;
            out_end = now + dur(A.list[A.jobs_lo[o_next]]);
        }
        bool step_blocked = false, in_blocked = false;
        if (!step_run && t < T && (i_next >= m || hi_of(A.jobs_hi[i_next]) > t)) {
            const uint64_t nd = A.need[t];
            if (nd == 0 || R + nd <= limit) {
                step_run = true; R += nd; step_end = now + (A.C[t + 1] - A.C[t]);
                peak = umax64(peak, R);
            } else step_blocked = true;
        }
        if (!in_run && i_next < i_iss && odone[A.jobs_hi[i_next]]) {
            const uint32_t v = A.list[A.jobs_hi[i_next]];
            if (R + A.size[v] <= limit) {
                in_run = true; R += A.size[v]; in_end = now + dur(v);
                peak = umax64(peak, R);
            } else in_blocked = true;
        }
        if (!step_run && !out_run && !in_run) {
            // nothing will change by itself: the limit is overridden once
            ++nforced;
            if (step_blocked) {
                step_run = true; R += A.need[t]; step_end = now + (A.C[t + 1] - A.C[t]);
            } else if (in_blocked) {
                const uint32_t v = A.list[A.jobs_hi[i_next]];
                in_run = true; R += A.size[v]; in_end = now + dur(v);
            } else {
                nforced = SIM_NONE;           // an inconsistent trace; leave rather than spin
                break;
            }
            peak = umax64(peak, R);
        }
        uint64_t nx = U64_MAX;
        if (step_run) nx = umin64(nx, step_end);
        if (out_run) nx = umin64(nx, out_end);
        if (in_run) nx = umin64(nx, in_end);
        now = nx;
    }
    A.total_ns[q] = now;
    A.overhead_ns[q] = now - A.C[T];
    A.peak_resident[q] = peak;
    A.forced[q] = nforced;
}

hipError_t launch_simulate_swaps(uint32_t n, uint32_t T, uint32_t Q, uint32_t kmax, const uint64_t *size,
                                 const uint32_t *alloc, const uint32_t *free_, const uint32_t *step_lo,
                                 const uint32_t *step_hi, uint32_t hi_minus, const uint64_t *C, uint64_t *need,
                                 uint64_t *rel, const uint32_t *list, const uint32_t *perm_lo,
                                 const uint32_t *perm_hi, const uint32_t *posmap, uint32_t *jobs_lo,
                                 uint32_t *jobs_hi, uint32_t *m, const uint32_t *prefix, const uint64_t *limits,
                                 uint32_t *kb, uint8_t *out_done, uint64_t bpus, uint64_t *total_ns,
                                 uint64_t *overhead_ns, uint64_t *peak_resident, uint32_t *forced, hipStream_t st,
                                 uint32_t n_lists, const uint32_t *n_listed)
{
    // n_listed given: run q replays row q of `list` (n_lists rows of n entries, *n_listed valid entries
    // each); the caller has cleared the n_lists position maps, they are filled here
    if (n_listed)
        hipLaunchKernelGGL(k_sim_mark_rows, dim3((n + 255) / 256, n_lists), dim3(256), 0, st, n, list, n_listed,
                           const_cast<uint32_t *>(posmap));
    hipLaunchKernelGGL(k_sim_steps, dim3((n + 255) / 256), dim3(256), 0, st, n, size, alloc, free_,
                       (unsigned long long *)need, (unsigned long long *)rel);
    hipLaunchKernelGGL(k_sim_jobs, dim3(n_lists), dim3(SIM_THREADS), 0, st, n, perm_lo, posmap, step_lo, step_hi,
                       hi_minus, jobs_lo, m);
    hipLaunchKernelGGL(k_sim_jobs, dim3(n_lists), dim3(SIM_THREADS), 0, st, n, perm_hi, posmap, step_lo, step_hi,
                       hi_minus, jobs_hi, m);
    SimArgs A{n, T, Q, kmax, size, step_lo, step_hi, hi_minus, C, (const unsigned long long *)need,
              (const unsigned long long *)rel, list, jobs_lo, jobs_hi, m, prefix, limits, kb, out_done,
              n_listed ? 1u : 0u, bpus,
              total_ns, overhead_ns, peak_resident, forced};
    hipLaunchKernelGGL(k_sim_run, dim3(Q), dim3(WAVE), 0, st, A);
    return hipGetLastError();
}

}  // namespace lap
