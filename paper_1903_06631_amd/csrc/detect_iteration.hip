// Iteration detection on a recorded request stream (Section V): the list ends with two equal
// consecutive subsequences of length p; the smallest such p (>= min_period) is reported.
//
// One workgroup.  A polynomial hash of every prefix (mod 2^64, odd base) is built with a block
// scan; the two halves of a candidate p then compare in O(1):
//     (P[M-p] - P[M-2p]) * r^p == P[M] - P[M-p]
// Candidates are tested 1024 at a time in ascending order; the first one whose hashes agree is
// checked element by element by the whole workgroup (hashes mod 2^64 can collide, the answer
// never depends on them), and the search resumes behind it if the check fails.
#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

constexpr int DI_THREADS = 1024;
constexpr int DI_WAVES = DI_THREADS / WAVE;
constexpr uint64_t DI_BASE = 0x9E3779B97F4A7C15ull | 1ull;

__device__ __forceinline__ uint64_t pow_base(uint32_t e)
{
    uint64_t r = 1, b = DI_BASE;
    while (e) { if (e & 1u) r *= b; b *= b; e >>= 1; }
    return r;
}

__device__ __forceinline__ uint64_t tok_hash(uint64_t x)
{
    x ^= x >> 31; x *= 0xBF58476D1CE4E5B9ull; x ^= x >> 29; x *= 0x94D049BB133111EBull; x ^= x >> 32;
    return x | 1ull;
}

__global__ __launch_bounds__(DI_THREADS) void k_detect_iteration(const uint64_t *__restrict__ tok, uint32_t M,
                                                                 uint32_t min_period, uint64_t *P,
                                                                 uint32_t *__restrict__ period)
{
    __shared__ uint64_t wsum[DI_WAVES];
    __shared__ uint32_t s_first, s_bad;
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;

    // P[i] = sum over j < i of hash(tok[j]) * r^j
    uint64_t carry = 0;
    if (tid == 0) P[0] = 0;
    for (uint32_t base = 0; base < M; base += DI_THREADS) {
        const uint32_t j = base + tid;
        const uint64_t v = j < M ? tok_hash(tok[j]) * pow_base(j) : 0;
        const uint64_t incl = wave_scan_add(v);
        if (lane == WAVE - 1) wsum[wave] = incl;
        __syncthreads();
        uint64_t pre = 0, tot = 0;
        for (int q = 0; q < DI_WAVES; ++q) { const uint64_t x = wsum[q]; if (q < (int)wave) pre += x; tot += x; }
        __syncthreads();
        if (j < M) P[j + 1] = carry + pre + incl;
        carry += tot;
    }
    __syncthreads();

    const uint32_t pmax = M / 2;
    uint32_t lo = min_period, found = 0;
    while (lo <= pmax) {
        // first candidate of this batch whose halves hash alike
        if (tid == 0) { s_first = 0xFFFFFFFFu; s_bad = 0; }
        __syncthreads();
        const uint32_t p = lo + tid;
        if (p >= lo && p <= pmax) {
            const uint64_t a = P[M - p] - P[M - 2 * p], b = P[M] - P[M - p];
            if (a * pow_base(p) == b) atomicMin(&s_first, p);
        }
        __syncthreads();
        const uint32_t c = s_first;
        __syncthreads();                 // everyone has read the batch result before it is reset
        if (c == 0xFFFFFFFFu) {
            if (pmax - lo < (uint32_t)DI_THREADS) break;
            lo += DI_THREADS;
            continue;
        }
        // exact check of candidate c
        bool bad = false;
        for (uint32_t i = tid; i < c && !bad; i += DI_THREADS) bad = tok[M - 2 * c + i] != tok[M - c + i];
        if (bad) s_bad = 1;
        __syncthreads();
        if (!s_bad) { found = c; break; }
        lo = c + 1;
        __syncthreads();
    }
    if (tid == 0) *period = found;
}

hipError_t launch_detect_iteration(const uint64_t *tokens, uint32_t M, uint32_t min_period, uint64_t *P,
                                   uint32_t *period, hipStream_t st)
{
    hipLaunchKernelGGL(k_detect_iteration, dim3(1), dim3(DI_THREADS), 0, st, tokens, M, min_period, P, period);
    return hipGetLastError();
}

}  // namespace lap
