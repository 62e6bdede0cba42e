// Swap schedule (Section IV-E): one stream carries the swap-outs in access order, each as soon
// as its access is over and the stream is free; a second stream carries the swap-ins in the
// order of the next accesses, each as late as its access and the swap-in after it allow.
//
// Both are scans.  A stream that serves job j (ready r_j, duration d_j) after it is free at x is
// free again at f_j(x) = max(x, r_j) + d_j = max(x + d_j, r_j + d_j); such functions compose as
// (a, b) pairs -- f(x) = max(x + a, b), (f2 o f1) = (a1 + a2, max(b1 + a2, b2)) -- so the end
// times of all swap-outs are one inclusive scan in (max, +), and the start times of all swap-ins
// the mirror image in (min, -) taken from the last job backwards.  The variables arrive sorted
// by access step (a radix sort of all variables, the swap list marks which ones take part), so
// unselected variables are the identity of the scan.
#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

constexpr int SC_THREADS = 1024;
constexpr int SC_WAVES = SC_THREADS / WAVE;
constexpr long long SC_NEG = -(1ll << 62), SC_POS = (1ll << 62);
constexpr uint32_t SC_NONE = 0xFFFFFFFFu;

__global__ __launch_bounds__(256) void k_sched_mark(uint32_t n, uint32_t k, const uint32_t *__restrict__ list,
                                                    uint32_t *__restrict__ posmap)
{
    const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < k) posmap[min(list[j], n - 1)] = j;
}

struct Fn {
    long long a, b;
};
// OUT: f(x) = max(x + a, b), `then` applied after `first`
__device__ __forceinline__ Fn then_max(const Fn &first, const Fn &then)
{
    const long long t = first.b + then.a;
    return Fn{first.a + then.a, t > then.b ? t : then.b};
}
// IN: g(y) = min(y - a, b)
__device__ __forceinline__ Fn then_min(const Fn &first, const Fn &then)
{
    const long long t = first.b - then.a;
    return Fn{first.a + then.a, t < then.b ? t : then.b};
}

template <bool OUT>
__device__ __forceinline__ Fn block_scan_fn(Fn v, Fn &carry, Fn *wtmp)
{
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    const Fn ident{0, OUT ? SC_NEG : SC_POS};
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        Fn o;
        o.a = (long long)shfl_up64((uint64_t)v.a, d);
        o.b = (long long)shfl_up64((uint64_t)v.b, d);
        if (lane >= d) v = OUT ? then_max(o, v) : then_min(o, v);
    }
    if (lane == WAVE - 1) wtmp[wave] = v;
    __syncthreads();
    Fn pre = carry, tot = carry;
    for (int q = 0; q < SC_WAVES; ++q) {
        const Fn x = wtmp[q];
        if (q < wave) pre = OUT ? then_max(pre, x) : then_min(pre, x);
        tot = OUT ? then_max(tot, x) : then_min(tot, x);
    }
    __syncthreads();
    carry = tot;
    (void)ident;
    return OUT ? then_max(pre, v) : then_min(pre, v);
}

struct SchedArgs {
    uint32_t n, T, k;
    const uint64_t *size;
    const uint32_t *step_lo, *step_hi;   // access steps: gap_lo or alloc, gap_hi or free (see hi_minus)
    uint32_t hi_minus;                   // 1 when step_hi holds free (the access is step free - 1)
    const uint64_t *C;                   // [T+1] start time of every step
    const uint32_t *perm_lo, *perm_hi;   // all variables by (step_lo, index) and by (step_hi, index)
    const uint32_t *posmap;              // variable -> position in the swap list, or none
    const uint32_t *list;
    uint64_t bpus;
    long long *out_start, *out_end, *in_start, *in_end;
    unsigned long long *diff;            // [T+1] what leaves the load curve (difference array)
    unsigned long long *late;            // [1]
};

__global__ __launch_bounds__(SC_THREADS) void k_sched_streams(SchedArgs A)
{
    __shared__ Fn wtmp[SC_WAVES];
    const uint32_t tid = threadIdx.x, n = A.n;
    // swap-outs, first to last
    Fn carry{0, SC_NEG};
    for (uint32_t base = 0; base < n; base += SC_THREADS) {
        const uint32_t r = base + tid;
        Fn f{0, SC_NEG};
        uint32_t pos = SC_NONE;
        long long d = 0;
        if (r < n) {
            const uint32_t v = A.perm_lo[r];
            pos = A.posmap[v];
            if (pos != SC_NONE) {
                d = (long long)((A.size[v] * 1000ull + A.bpus - 1) / A.bpus);
                f = Fn{d, (long long)A.C[A.step_lo[v] + 1] + d};
            }
        }
        const Fn g = block_scan_fn<true>(f, carry, wtmp);
        if (pos != SC_NONE) { A.out_end[pos] = g.b; A.out_start[pos] = g.b - d; }
    }
    // swap-ins, last to first
    carry = Fn{0, SC_POS};
    for (uint32_t base = 0; base < n; base += SC_THREADS) {
        const uint32_t rr = base + tid;
        Fn f{0, SC_POS};
        uint32_t pos = SC_NONE;
        long long d = 0;
        if (rr < n) {
            const uint32_t v = A.perm_hi[n - 1 - rr];
            pos = A.posmap[v];
            if (pos != SC_NONE) {
                d = (long long)((A.size[v] * 1000ull + A.bpus - 1) / A.bpus);
                f = Fn{d, (long long)A.C[A.step_hi[v] - A.hi_minus] - d};
            }
        }
        const Fn g = block_scan_fn<false>(f, carry, wtmp);
        if (pos != SC_NONE) { A.in_start[pos] = g.b; A.in_end[pos] = g.b + d; }
    }
    __syncthreads();
    // what each selected variable takes out of the load curve: the whole steps between the end of
    // its swap-out and the start of its swap-in; transfers that overlap are counted as late
    unsigned long long late = 0;
    for (uint32_t j = tid; j < A.k; j += SC_THREADS) {
        const long long eo = A.out_end[j], si = A.in_start[j];
        if (eo > si) { late += (unsigned long long)(eo - si); continue; }
        const uint32_t T = A.T;
        uint32_t l0 = 0, h0 = T;                  // first t with C[t] >= eo
        while (l0 < h0) { const uint32_t m = (l0 + h0) >> 1; if ((long long)A.C[m] < eo) l0 = m + 1; else h0 = m; }
        const uint32_t lo = l0;
        l0 = 0; h0 = T;                           // last t with C[t] <= si
        while (l0 < h0) { const uint32_t m = (l0 + h0 + 1) >> 1; if ((long long)A.C[m] <= si) l0 = m; else h0 = m - 1; }
        const uint32_t hi = l0;
        if (hi > lo) {
            const unsigned long long s = A.size[min(A.list[j], n - 1)];
            atomicAdd(&A.diff[lo], s);
            atomicAdd(&A.diff[hi], 0ull - s);
        }
    }
    late = wave_reduce_add(late);
    if ((tid & (WAVE - 1)) == 0 && late) atomicAdd(A.late, late);
}

__global__ __launch_bounds__(SC_THREADS) void k_sched_load(uint32_t T, const uint64_t *__restrict__ load,
                                                           const unsigned long long *__restrict__ diff,
                                                           uint64_t *__restrict__ load_sched,
                                                           uint64_t *__restrict__ peak)
{
    __shared__ uint64_t wsum[SC_WAVES], wmax[SC_WAVES];
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    uint64_t carry = 0, mx = 0;
    for (uint32_t base = 0; base < T; base += SC_THREADS) {
        const uint32_t t = base + tid;
        const uint64_t d = t < T ? diff[t] : 0;
        const uint64_t incl = wave_scan_add(d);
        if (lane == WAVE - 1) wsum[wave] = incl;
        __syncthreads();
        uint64_t pre = 0, tot = 0;
        for (int q = 0; q < SC_WAVES; ++q) { const uint64_t x = wsum[q]; if (q < (int)wave) pre += x; tot += x; }
        __syncthreads();
        if (t < T) {
            const uint64_t v = load[t] - (carry + pre + incl);
            load_sched[t] = v;
            mx = umax64(mx, v);
        }
        carry += tot;
    }
    mx = wave_reduce_max(mx);
    if (lane == 0) wmax[wave] = mx;
    __syncthreads();
    if (tid == 0) {
        uint64_t m = 0;
        for (int q = 0; q < SC_WAVES; ++q) m = umax64(m, wmax[q]);
        *peak = m;
    }
}

hipError_t launch_sched_mark(uint32_t n, uint32_t k, const uint32_t *list, uint32_t *posmap, hipStream_t st)
{
    if (k) hipLaunchKernelGGL(k_sched_mark, dim3((k + 255) / 256), dim3(256), 0, st, n, k, list, posmap);
    return hipGetLastError();
}

hipError_t launch_schedule_swaps(uint32_t n, uint32_t T, uint32_t k, const uint64_t *size, const uint32_t *step_lo,
                                 const uint32_t *step_hi, uint32_t hi_minus, const uint64_t *C,
                                 const uint32_t *perm_lo, const uint32_t *perm_hi, uint32_t *posmap,
                                 const uint32_t *list, uint64_t bpus, int64_t *out_start, int64_t *out_end,
                                 int64_t *in_start, int64_t *in_end, uint64_t *diff, uint64_t *late,
                                 const uint64_t *load, uint64_t *load_sched, uint64_t *peak, hipStream_t st)
{
    if (k) hipLaunchKernelGGL(k_sched_mark, dim3((k + 255) / 256), dim3(256), 0, st, n, k, list, posmap);
    SchedArgs A{n, T, k, size, step_lo, step_hi, hi_minus, C, perm_lo, perm_hi, posmap, list, bpus,
                (long long *)out_start, (long long *)out_end, (long long *)in_start, (long long *)in_end,
                (unsigned long long *)diff, (unsigned long long *)late};
    hipLaunchKernelGGL(k_sched_streams, dim3(1), dim3(SC_THREADS), 0, st, A);
    hipLaunchKernelGGL(k_sched_load, dim3(1), dim3(SC_THREADS), 0, st, T, load, (const unsigned long long *)diff,
                       load_sched, peak);
    return hipGetLastError();
}

}  // namespace lap
