// Swap-candidate filter and priority scores (Section IV-A, IV-B).
//
// Prefix arrays over the T steps are built once by a single workgroup:
//   C[t]  wall-clock start of step t (prefix sum of step_ns), C[T] = total
//   S[t]  sum of load over steps < t (area under the load curve)
//   PM[t] max load over steps < t,   SM[t] max load over steps >= t
// A sparse table over load answers range-maximum queries in O(1).  Then one
// thread per variable evaluates its scores with two binary searches over C.
#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

constexpr int PFX_THREADS = 1024;

__device__ __forceinline__ uint64_t block_scan(uint64_t v, bool is_max, uint64_t *wtmp, uint64_t &total)
{
    // inclusive scan over the workgroup (sum or max); total = reduction of all
    const int tid = threadIdx.x, l = tid & (WAVE - 1), w = tid / WAVE;
    uint64_t incl = is_max ? wave_scan_max(v) : wave_scan_add(v);
    if (l == WAVE - 1) wtmp[w] = incl;
    __syncthreads();
    uint64_t pre = 0, tot = 0;
    for (int k = 0; k < PFX_THREADS / WAVE; ++k) {
        const uint64_t x = wtmp[k];
        if (is_max) { if (k < w) pre = umax64(pre, x); tot = umax64(tot, x); }
        else        { if (k < w) pre += x;             tot += x; }
    }
    __syncthreads();
    total = tot;
    return is_max ? umax64(pre, incl) : pre + incl;
}

__global__ __launch_bounds__(PFX_THREADS) void k_swap_prefix(uint32_t T, const uint64_t *__restrict__ load,
                                                             const uint64_t *__restrict__ step_ns,
                                                             uint64_t *__restrict__ C, uint64_t *__restrict__ S,
                                                             uint64_t *__restrict__ PM, uint64_t *__restrict__ SM,
                                                             uint64_t *__restrict__ peak_out,
                                                             uint32_t *__restrict__ tpeak_out)
{
    __shared__ uint64_t wtmp[PFX_THREADS / WAVE];
    __shared__ uint64_t s_peak;
    const uint32_t tid = threadIdx.x;
    uint64_t cC = 0, cS = 0, cM = 0, tot;
    if (tid == 0) { C[0] = 0; S[0] = 0; PM[0] = 0; SM[T] = 0; }
    for (uint32_t base = 0; base < T; base += PFX_THREADS) {
        const uint32_t t = base + tid;
        const bool in = t < T;
        const uint64_t ns = in ? (step_ns ? step_ns[t] : 1000000ull) : 0;
        const uint64_t ld = in ? load[t] : 0;
        const uint64_t c = cC + block_scan(ns, false, wtmp, tot); cC += tot;
        const uint64_t s = cS + block_scan(ld, false, wtmp, tot); cS += tot;
        const uint64_t m = umax64(cM, block_scan(ld, true, wtmp, tot)); cM = umax64(cM, tot);
        if (in) { C[t + 1] = c; S[t + 1] = s; PM[t + 1] = m; }
    }
    if (tid == 0) s_peak = cM;
    // suffix maxima: scan the reversed array
    uint64_t cR = 0;
    for (uint32_t base = 0; base < T; base += PFX_THREADS) {
        const uint32_t k = base + tid;             // k-th element from the end
        const bool in = k < T;
        const uint64_t ld = in ? load[T - 1 - k] : 0;
        const uint64_t m = umax64(cR, block_scan(ld, true, wtmp, tot)); cR = umax64(cR, tot);
        if (in) SM[T - 1 - k] = m;
    }
    __syncthreads();
    // earliest step that attains the peak
    const uint64_t pk = s_peak;
    uint32_t first = 0xFFFFFFFFu;
    for (uint32_t t = tid; t < T; t += PFX_THREADS)
        if (load[t] == pk) { first = t; break; }
    __shared__ uint32_t s_first;
    if (tid == 0) s_first = 0xFFFFFFFFu;
    __syncthreads();
    if (first != 0xFFFFFFFFu) atomicMin(&s_first, first);
    __syncthreads();
    if (tid == 0) { *peak_out = pk; *tpeak_out = s_first; }
}

// level k of the sparse table: M[k][t] = max load[t .. t + 2^k)
__global__ void k_sparse_level(uint32_t T, uint32_t half, const uint64_t *__restrict__ prev, uint64_t *__restrict__ cur)
{
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const uint64_t a = prev[t];
    const uint64_t b = (t + half < T) ? prev[t + half] : 0;
    cur[t] = umax64(a, b);
}

__global__ __launch_bounds__(256) void k_score(uint32_t n, uint32_t T, const uint64_t *__restrict__ size,
                                               const uint32_t *__restrict__ alloc, const uint32_t *__restrict__ free_,
                                               const uint32_t *__restrict__ gap_lo, const uint32_t *__restrict__ gap_hi,
                                               uint64_t bpus, uint64_t min_bytes,
                                               const uint64_t *__restrict__ load, const uint64_t *__restrict__ C,
                                               const uint64_t *__restrict__ S, const uint64_t *__restrict__ PM,
                                               const uint64_t *__restrict__ SM, const uint64_t *__restrict__ table,
                                               const uint64_t *__restrict__ peak_p, const uint32_t *__restrict__ tpeak_p,
                                               uint8_t *__restrict__ cand, int64_t *__restrict__ doa,
                                               double *__restrict__ aoa, uint64_t *__restrict__ wdoa,
                                               uint64_t *__restrict__ cut, uint32_t *__restrict__ win_lo,
                                               uint32_t *__restrict__ win_hi)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint64_t peak = *peak_p;
    const uint32_t t_peak = *tpeak_p;
    const uint64_t s = size[i];
    const uint32_t a = alloc[i], f = free_[i];
    const uint32_t tl = gap_lo ? gap_lo[i] : a;
    const uint32_t th = gap_hi ? gap_hi[i] : f - 1;
    uint8_t c = 0; int64_t d = 0; double ar = 0.0; uint64_t w = 0, pc = 0;
    uint32_t wl = 0, wh = 0;          // whole steps [wl, wh) during which a swapped variable is away
    if (th > tl) {
        c = (s >= min_bytes && a <= t_peak && t_peak < f) ? 1 : 0;
        const uint64_t delta = (s * 1000ull + bpus - 1) / bpus;
        const uint64_t idle_from = C[tl + 1], idle_to = C[th];
        d = (int64_t)(idle_to - idle_from) - 2 * (int64_t)delta;
        ar = d >= 0 ? (double)d * (double)s : (double)d / (double)s;
        w = S[th] - S[tl + 1];
        if (d >= 0) {
            const uint64_t out_done = idle_from + delta, in_start = idle_to - delta;
            // lo = first t with C[t] >= out_done ; hi = last t with C[t] <= in_start   (t in [0, T])
            uint32_t l0 = 0, h0 = T;
            while (l0 < h0) { const uint32_t m = (l0 + h0) >> 1; if (C[m] < out_done) l0 = m + 1; else h0 = m; }
            const uint32_t lo = l0;
            l0 = 0; h0 = T;
            while (l0 < h0) { const uint32_t m = (l0 + h0 + 1) >> 1; if (C[m] <= in_start) l0 = m; else h0 = m - 1; }
            const uint32_t hi = l0;
            if (hi > lo) {
                wl = lo; wh = hi;
                const uint32_t len = hi - lo;
                const uint32_t k = 31 - __clz(len);
                const uint64_t *lvl = table + (size_t)k * T;
                const uint64_t inside = umax64(lvl[lo], lvl[hi - (1u << k)]);
                const uint64_t np = umax64(umax64(PM[lo], SM[hi]), inside - s);
                pc = peak - np;
            }
        }
    }
    cand[i] = c; doa[i] = d; aoa[i] = ar; wdoa[i] = w; cut[i] = pc;
    if (win_lo) { win_lo[i] = wl; win_hi[i] = wh; }
}

hipError_t launch_swap_prefix(uint32_t T, const uint64_t *load, const uint64_t *step_ns, uint64_t *C, uint64_t *S,
                              uint64_t *PM, uint64_t *SM, uint64_t *peak, uint32_t *t_peak, hipStream_t st)
{
    hipLaunchKernelGGL(k_swap_prefix, dim3(1), dim3(PFX_THREADS), 0, st, T, load, step_ns, C, S, PM, SM, peak, t_peak);
    return hipGetLastError();
}

// table holds levels 1.. ; level 0 is `load` itself, so table level k lives at table + (k) * T with
// level 0 copied in by the first launch (half = 0 copies).
hipError_t launch_sparse_table(uint32_t T, const uint64_t *load, uint64_t *table, uint32_t levels, hipStream_t st)
{
    const uint32_t blocks = (T + 255) / 256;
    hipLaunchKernelGGL(k_sparse_level, dim3(blocks), dim3(256), 0, st, T, T /* no partner */, load, table);
    for (uint32_t k = 1; k < levels; ++k)
        hipLaunchKernelGGL(k_sparse_level, dim3(blocks), dim3(256), 0, st, T, 1u << (k - 1),
                           table + (size_t)(k - 1) * T, table + (size_t)k * T);
    return hipGetLastError();
}

hipError_t launch_score(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                        const uint32_t *gap_lo, const uint32_t *gap_hi, uint64_t bpus, uint64_t min_bytes,
                        const uint64_t *load, const uint64_t *C, const uint64_t *S, const uint64_t *PM,
                        const uint64_t *SM, const uint64_t *table, const uint64_t *peak, const uint32_t *t_peak,
                        uint8_t *cand, int64_t *doa, double *aoa, uint64_t *wdoa, uint64_t *cut, uint32_t *win_lo,
                        uint32_t *win_hi, hipStream_t st)
{
    const uint32_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(k_score, dim3(blocks), dim3(256), 0, st, n, T, size, alloc, free_, gap_lo, gap_hi, bpus,
                       min_bytes, load, C, S, PM, SM, table, peak, t_peak, cand, doa, aoa, wdoa, cut, win_lo, win_hi);
    return hipGetLastError();
}

}  // namespace lap
