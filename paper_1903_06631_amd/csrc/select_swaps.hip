// Selection of swap variables down to a load limit (Section IV-D), for K priority scores at
// once, including the submodular WDOA order of Section IV-B (iv), and load_min (Section VI-B1).
//
// The walk is sequential by nature: every addition changes the curve the next decision sees.
// One workgroup of 1024 threads runs one score kind.  Thread i owns the steps t = i (mod 1024)
// of the current load curve and the candidate slots c = i (mod 1024); one iteration applies the
// previous winner to the owned steps, re-scores the owned slots (SWDOA only, in closed form: a
// slot's area drops by size * |idle steps of the slot that the winner leaves|), and finds the
// new peak and the best remaining slot with a single fused reduction and one barrier.
#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / WAVE;
constexpr uint32_t NONE = 0xFFFFFFFFu;

// slot list of the candidates (any order: ties are decided on the variable index) and the
// difference array of what leaves the curve when every candidate is away on all its idle steps
__global__ __launch_bounds__(256) void k_sel_gather(SelectArgs a)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.n || !a.cand[i]) return;
    const uint32_t tl = a.gap_lo ? a.gap_lo[i] : a.alloc[i];
    const uint32_t th = a.gap_hi ? a.gap_hi[i] : a.free_[i] - 1;
    const uint32_t slot = atomicAdd(a.nc, 1u);
    a.cidx[slot] = i;
    a.c_ilo[slot] = tl + 1;
    a.c_ihi[slot] = th;
    const unsigned long long s = a.size[i];
    if (th > tl + 1) {
        atomicAdd((unsigned long long *)&a.dmin[tl + 1], s);
        atomicAdd((unsigned long long *)&a.dmin[th], 0ull - s);
    }
}

// order-preserving map of a score to an unsigned key (larger = higher priority)
__device__ __forceinline__ uint64_t score_key(const SelectArgs &a, uint32_t kind, uint32_t v)
{
    switch (kind) {
    case 0: return (uint64_t)a.doa[v] ^ (1ull << 63);
    case 1: {
        const uint64_t b = (uint64_t)__double_as_longlong(a.aoa[v]);
        return (b >> 63) ? ~b : (b | (1ull << 63));
    }
    case 4: return a.cut[v];
    default: return a.wdoa[v];
    }
}

__device__ __forceinline__ uint64_t custom_key(double x)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    return (b >> 63) ? ~b : (b | (1ull << 63));
}

struct Best {
    uint64_t score;
    uint32_t var, slot;
};
__device__ __forceinline__ bool better(const Best &x, const Best &y)
{
    return x.score > y.score || (x.score == y.score && x.var < y.var);
}

__global__ __launch_bounds__(SEL_THREADS) void k_sel_walk(SelectArgs a)
{
    __shared__ uint64_t p_peak[2][SEL_WAVES], p_score[2][SEL_WAVES];
    __shared__ uint32_t p_var[2][SEL_WAVES], p_slot[2][SEL_WAVES];
    const uint32_t ks = blockIdx.x, kind = a.kinds[ks];
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const uint32_t n = a.n, T = a.T, nc = *a.nc;
    uint64_t *rs = a.r_score + (size_t)ks * n;
    uint32_t *rv = a.r_var + (size_t)ks * n;
    uint64_t *lc = a.l_cur + (size_t)ks * T;
    uint32_t *order = a.order + (size_t)ks * n;
    uint32_t *rank = a.rank ? a.rank + (size_t)ks * n : nullptr;
    uint64_t *peaks = a.peaks + (size_t)ks * ((size_t)n + 1);

    for (uint32_t c = tid; c < nc; c += SEL_THREADS) {
        const uint32_t v = a.cidx[c];
        rv[c] = v;
        rs[c] = kind == 5 ? custom_key(a.custom[(size_t)ks * n + v]) : score_key(a, kind, v);
    }
    for (uint32_t t = tid; t < T; t += SEL_THREADS) lc[t] = a.load[t];
    if (rank)
        for (uint32_t i = tid; i < n; i += SEL_THREADS) rank[i] = NONE;
    if (ks == 0 && tid == 0) *a.n_cand = nc;

    bool has_w = false;
    uint32_t w_slot = 0, w_lo = 0, w_hi = 0;
    uint64_t w_size = 0;
    for (uint32_t k = 0;; ++k) {
        // the previous winner leaves the owned steps; running maximum of the owned steps
        uint64_t mx = 0;
        for (uint32_t t = tid; t < T; t += SEL_THREADS) {
            uint64_t x = lc[t];
            if (has_w && t >= w_lo && t < w_hi) { x -= w_size; lc[t] = x; }
            mx = umax64(mx, x);
        }
        // best remaining owned slot (SWDOA: after re-scoring on the reduced curve)
        Best b{0, NONE, NONE};
        for (uint32_t c = tid; c < nc; c += SEL_THREADS) {
            const uint32_t v = rv[c];
            if (v == NONE) continue;
            if (has_w && c == w_slot) { rv[c] = NONE; continue; }
            uint64_t s = rs[c];
            if (kind == 3 && has_w) {
                const uint32_t lo = max(a.c_ilo[c], w_lo), hi = min(a.c_ihi[c], w_hi);
                if (hi > lo) { s -= w_size * (uint64_t)(hi - lo); rs[c] = s; }
            }
            const Best x{s, v, c};
            if (better(x, b)) b = x;
        }
#pragma unroll
        for (int d = 1; d < WAVE; d <<= 1) {
            mx = umax64(mx, shfl_xor64(mx, d));
            const Best o{shfl_xor64(b.score, d), (uint32_t)__shfl_xor((int)b.var, d, WAVE),
                         (uint32_t)__shfl_xor((int)b.slot, d, WAVE)};
            if (better(o, b)) b = o;
        }
        const int buf = k & 1;
        if (lane == 0) { p_peak[buf][wave] = mx; p_score[buf][wave] = b.score; p_var[buf][wave] = b.var; p_slot[buf][wave] = b.slot; }
        __syncthreads();
        mx = 0;
        b = Best{0, NONE, NONE};
#pragma unroll
        for (int q = 0; q < SEL_WAVES; ++q) {
            mx = umax64(mx, p_peak[buf][q]);
            const Best o{p_score[buf][q], p_var[buf][q], p_slot[buf][q]};
            if (better(o, b)) b = o;
        }
        if (tid == 0) {
            peaks[k] = mx;
            if (b.var != NONE) {
                order[k] = b.var;
                if (rank) rank[b.var] = k;
                if (kind == 3 && a.pick_wdoa) a.pick_wdoa[b.var] = b.score;
            }
        }
        if (b.var == NONE) break;        // k == nc: nothing left
        has_w = true;
        w_slot = b.slot;
        w_size = a.size[b.var];
        w_lo = a.win_lo[b.var];
        w_hi = a.win_hi[b.var];
    }
    __syncthreads();
    // every limit: the shortest prefix of the order whose peak is within the limit
    for (uint32_t q = tid; q < a.L; q += SEL_THREADS) {
        const uint64_t lim = a.limits[q];
        uint32_t lo = 0, hi = nc;        // first k in [0, nc] with peaks[k] <= lim, else nc
        while (lo < hi) {
            const uint32_t m = (lo + hi) >> 1;
            if (peaks[m] <= lim) hi = m; else lo = m + 1;
        }
        a.n_selected[(size_t)ks * a.L + q] = lo;
        a.peak_after[(size_t)ks * a.L + q] = peaks[lo];
    }
}

// load_min: prefix sum of the difference array = load that leaves each step; one workgroup
__global__ __launch_bounds__(SEL_THREADS) void k_load_min(uint32_t T, const uint64_t *__restrict__ load,
                                                         const uint64_t *__restrict__ dmin,
                                                         uint64_t *__restrict__ out)
{
    __shared__ uint64_t wsum[SEL_WAVES], wmax[SEL_WAVES];
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    uint64_t carry = 0, mx = 0;
    for (uint32_t base = 0; base < T; base += SEL_THREADS) {
        const uint32_t t = base + tid;
        const uint64_t d = t < T ? dmin[t] : 0;
        const uint64_t incl = wave_scan_add(d);
        if (lane == WAVE - 1) wsum[wave] = incl;
        __syncthreads();
        uint64_t pre = 0, tot = 0;
        for (int q = 0; q < SEL_WAVES; ++q) { const uint64_t x = wsum[q]; if (q < (int)wave) pre += x; tot += x; }
        __syncthreads();
        if (t < T) mx = umax64(mx, load[t] - (carry + pre + incl));
        carry += tot;
    }
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) mx = umax64(mx, shfl_xor64(mx, d));
    if (lane == 0) wmax[wave] = mx;
    __syncthreads();
    if (tid == 0) {
        uint64_t m = 0;
        for (int q = 0; q < SEL_WAVES; ++q) m = umax64(m, wmax[q]);
        *out = m;
    }
}

hipError_t launch_select_swaps(const SelectArgs &a, bool gather, hipStream_t st)
{
    if (gather) {
        hipLaunchKernelGGL(k_sel_gather, dim3((a.n + 255) / 256), dim3(256), 0, st, a);
        hipLaunchKernelGGL(k_load_min, dim3(1), dim3(SEL_THREADS), 0, st, a.T, a.load, a.dmin, a.load_min);
    }
    hipLaunchKernelGGL(k_sel_walk, dim3(a.K), dim3(SEL_THREADS), 0, st, a);
    return hipGetLastError();
}

// Section IV-C, Eq. 3 on the raw scores: one binary64 expression per (weight vector, variable),
// evaluated left to right without contraction
__global__ __launch_bounds__(256) void k_weighted_scores(uint32_t n, uint32_t W, const double *__restrict__ weights,
                                                         const double *__restrict__ aoa,
                                                         const int64_t *__restrict__ doa,
                                                         const uint64_t *__restrict__ wdoa,
                                                         const uint64_t *__restrict__ swdoa, double *__restrict__ bo)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x, w = blockIdx.y;
    if (i >= n) return;
    const double a = weights[4 * w], b = weights[4 * w + 1], c = weights[4 * w + 2], d = weights[4 * w + 3];
    const double t1 = a * aoa[i], t2 = b * (double)doa[i];
    const double t3 = t1 + t2, t4 = c * (double)wdoa[i];
    const double t5 = t3 + t4, t6 = d * (double)swdoa[i];
    bo[(size_t)w * n + i] = t5 + t6;
}

hipError_t launch_weighted_scores(uint32_t n, uint32_t W, const double *weights, const double *aoa, const int64_t *doa,
                                  const uint64_t *wdoa, const uint64_t *swdoa, double *bo, hipStream_t st)
{
    hipLaunchKernelGGL(k_weighted_scores, dim3((n + 255) / 256, W), dim3(256), 0, st, n, W, weights, aoa, doa, wdoa,
                       swdoa, bo);
    return hipGetLastError();
}

// index of the smallest of n values, the lowest index among equals (n is small)
__global__ __launch_bounds__(WAVE) void k_argmin_u64(uint32_t n, const uint64_t *__restrict__ v, uint32_t *best)
{
    if (threadIdx.x != 0) return;
    uint32_t b = 0;
    for (uint32_t i = 1; i < n; ++i)
        if (v[i] < v[b]) b = i;
    *best = b;
}

hipError_t launch_argmin_u64(uint32_t n, const uint64_t *v, uint32_t *best, hipStream_t st)
{
    hipLaunchKernelGGL(k_argmin_u64, dim3(1), dim3(WAVE), 0, st, n, v, best);
    return hipGetLastError();
}

}  // namespace lap
