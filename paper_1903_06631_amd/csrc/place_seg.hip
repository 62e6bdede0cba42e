// First-fit placement of every variable under many orderings (Section III-C): the path for
// traces whose variables live long (dense interval graphs), where neither
// per-step free lists (every block would have to be entered at every step of its life) nor a
// sweep over all placed blocks (half of them are neighbours) is affordable.
//
// The time line is cut into segments of w = 2^shift steps.  Free address ranges ("holes") are
// kept, sorted, in three families of lists (seg_core.h):
//   all[k]    free with respect to every block whose lifetime meets segment k
//   cover[k]  free with respect to the blocks that live through all of segment k
//   step[t]   free with respect to the blocks alive at step t that do not live through all of
//             t's segment
// A variable with lifetime [a, f) meets, in time, exactly the blocks of all[k] for the segments
// it lives through entirely, and of cover[k] and step[t] for its steps t in the (at most two)
// segments it lives through partly.  Its first fit is the lowest address that is free in all
// of these lists: every thread of the workgroup asks one list for its lowest fit at or above
// the candidate, the maximum becomes the next candidate, until no list moves it (two to three
// rounds in practice, because every list is the union of everything that matters in its
// segment, so few of its holes are filled by blocks of another list).  The placed block is then
// taken out of all[k] of every segment it touches, cover[k] of the segments it lives through,
// and step[t] of its other steps: one list per thread again.  A block enters about
// lifetime / w + w lists instead of `lifetime` per-step lists; w is chosen per trace to make
// the total smallest.
//
// One workgroup of 256 threads works on one ordering at a time in its own slot of the list
// pool and then takes the next ordering from a common counter; the number of slots is what the
// workspace has room for.  Results are identical to placing the variables one by one in rank
// order (same fixed point: the lowest address free of every time-overlapping block).
// Best-fit orderings of such a trace stay with the sweep over the sorted blocks (place_fast.hip):
// best-fit looks at every hole that fits, which a sweep does in one pass and a fixed point per
// hole does not.
#include "lap_dev.h"
#include "lap_kernels.h"
#define LAP_HD __device__
#include "seg_core.h"

namespace lap {

constexpr int SEG_THREADS = 256;
constexpr int SEG_WAVES = SEG_THREADS / WAVE;
constexpr int SEG_MEMO = 2;        // lists per thread whose last answer is kept between rounds

__device__ __forceinline__ uint32_t seg_wave_max(uint32_t v) { return read_lane(wave_scan_max_u32(v), WAVE - 1); }

// ---------------------------------------------------------------------------
// preparation: how many blocks every list will see (= its capacity - 1), list starts
// ---------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_seg_count(uint32_t n, uint32_t T, const uint32_t *__restrict__ alloc,
                                                   const uint32_t *__restrict__ free_, const PlanHeader *hdr,
                                                   uint32_t *cnt)
{
    if (!hdr->mode2) return;
    const SegGeom g{hdr->seg_shift, hdr->seg_K, T};
    // one wave per variable: its lanes share the variable's lists
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) / WAVE, nwaves = gridDim.x * blockDim.x / WAVE;
    for (uint32_t v = wave; v < n; v += nwaves) {
        const SegSpan sp = seg_span(g, alloc[v], free_[v]);
        const uint32_t nu = sp.n_update();
        for (uint32_t i = lane; i < nu; i += WAVE) atomicAdd(&cnt[seg_update_list(g, sp, i)], 1u);
    }
}

constexpr int SEG_SCAN_THREADS = 1024;

// lst[j] = sum over lists before j of (cnt + 1): every list has room for one range more than
// the blocks it will see (a block adds at most one range)
__global__ __launch_bounds__(SEG_SCAN_THREADS) void k_seg_scan(uint32_t T, uint32_t B, PlanHeader *hdr,
                                                               const uint32_t *__restrict__ cnt, uint32_t *lst,
                                                               uint64_t pool_entries)
{
    __shared__ uint64_t wtmp[SEG_SCAN_THREADS / WAVE];
    if (!hdr->mode2) return;
    const uint32_t nl = 2 * hdr->seg_K + T + 1;
    const uint32_t tid = threadIdx.x, l = tid & (WAVE - 1), w = tid / WAVE;
    uint64_t carry = 0;
    for (uint32_t base = 0; base < nl; base += SEG_SCAN_THREADS) {
        const uint32_t j = base + tid;
        const uint64_t v = j < nl ? (uint64_t)cnt[j] + 1 : 0;
        const uint64_t incl = wave_scan_add(v);
        if (l == WAVE - 1) wtmp[w] = incl;
        __syncthreads();
        uint64_t pre = 0, tot = 0;
        for (int k = 0; k < SEG_SCAN_THREADS / WAVE; ++k) {
            const uint64_t x = wtmp[k];
            if ((uint32_t)k < w) pre += x;
            tot += x;
        }
        __syncthreads();
        if (j < nl) lst[j] = (uint32_t)(carry + pre + incl - v);
        carry += tot;
    }
    if (tid == 0) {
        // the slots are laid out with what the lists really take (the estimate that chose the
        // segment width counts the same blocks another way)
        const uint64_t slots = pool_entries / carry;
        lst[nl] = (uint32_t)carry;
        hdr->seg_need = carry;
        hdr->seg_slots = (uint32_t)(slots < B ? slots : B);
        if (slots == 0 || carry >= 0xFFFFFFFFull) hdr->mode2 = 0;
    }
}

// ---------------------------------------------------------------------------
// the placement kernel
// ---------------------------------------------------------------------------

struct SegArgs {
    uint32_t n, T, B;
    const uint4 *vrec;           // [n] (first step, end of life, size in granules, -)
    const uint32_t *perm;        // [B][n]
    const uint32_t *fits;        // [B]
    PlanHeader *hdr;
    const uint32_t *lst;         // [n_lists + 1] start of every list inside a slot
    uint64_t *pool;              // [slots][seg_need]
    uint32_t *lens;              // [slots][dir_cap]
    uint32_t dir_cap;
    uint64_t *offs;              // [B][n] in rank order
    uint64_t *fps;               // [B]
    uint64_t *ticks;             // [B] duration of every ordering in timer ticks
    int trial_b;                 // >= 0: trial run on the first ranks of this ordering, one workgroup
    uint32_t trial_percent;
};

// Whether these lists pay depends on how the searches converge, which depends on the trace: with
// nested lifetimes and a tight packing (a training iteration) two to three rounds, with lifetimes
// at random six to eight, and then the sweep over the sorted blocks is the faster way.  So the
// first ranks of one ordering are placed ahead of time by one workgroup (TRIAL = true), counting
// the rounds of the multi-step variables; above `trial_percent` / 100 rounds per variable the
// trace is handed back to the sweep (mode2 = 0), before any placement kernel looks at that flag.
constexpr uint32_t SEG_TRIAL_RANKS = 2048;

template <bool TRIAL>
__global__ __launch_bounds__(SEG_THREADS) void k_place_seg(SegArgs A)
{
    __shared__ uint32_t s_max[2][SEG_WAVES];
    __shared__ uint32_t s_next;

    PlanHeader *hdr = A.hdr;
    if (!hdr->mode2) return;
    const uint32_t slots = TRIAL ? 1u : hdr->seg_slots;
    if (blockIdx.x >= slots) return;
    const SegGeom g{hdr->seg_shift, hdr->seg_K, A.T};
    const uint32_t nl = g.n_lists();
    const uint32_t sh = hdr->shift;
    const uint32_t n = TRIAL ? min(A.n, SEG_TRIAL_RANKS) : A.n;
    const uint32_t tid = threadIdx.x, l = tid & (WAVE - 1), wave = tid / WAVE;
    uint32_t trial_rounds = 0, trial_vars = 0;
    uint64_t *pool = A.pool + (size_t)blockIdx.x * hdr->seg_need;
    uint32_t *lens = A.lens + (size_t)blockIdx.x * A.dir_cap;
    const uint32_t *__restrict__ lst = A.lst;

    // The workgroups take orderings from a common counter, so that one that drew quick orderings goes
    // on to the next instead of idling (orderings differ by a factor of two in their time).
    for (;;) {
        uint32_t b = (uint32_t)A.trial_b;
        if (!TRIAL) {
            if (tid == 0) s_next = atomicAdd(&hdr->seg_next, 1u);
            __syncthreads();
            b = s_next;
            __syncthreads();
        }
        if (b >= A.B) break;
        if (A.fits[b] != 0) {                        // best-fit orderings: the sweep kernel places them
            if (TRIAL) break;
            continue;
        }
        const long long t_begin = wall_clock64();
        const uint32_t *perm = A.perm + (size_t)b * A.n;
        uint64_t *offs = A.offs + (size_t)b * A.n;
        // every list starts as one range: the whole address space
        for (uint32_t j = tid; j < nl; j += SEG_THREADS) {
            pool[lst[j]] = seg_pack(0u, SEG_INF);
            lens[j] = 1;
        }
        __syncthreads();
        uint32_t fp = 0, flip = 0;
        for (uint32_t r0 = 0; r0 < n; r0 += WAVE) {
            // every wave holds the records of ranks r0 .. r0 + 63, lane i that of rank r0 + i
            uint4 rec = make_uint4(0u, 1u, 1u, 0u);
            if (r0 + l < n) rec = A.vrec[perm[r0 + l]];
            const uint32_t wn = min((uint32_t)WAVE, n - r0);
            for (uint32_t p = 0; p < wn; ++p) {
                const uint32_t a = read_lane(rec.x, (int)p), f = read_lane(rec.y, (int)p), s = read_lane(rec.z, (int)p);
                const SegSpan sp = seg_span(g, a, f);
                const uint32_t nq = sp.n_query(), nu = sp.n_update();
                const bool longv = f - a > 1;         // long-lived blocks end up high, one-step ones low
                // lowest address that is free in every list of the variable: every thread asks its
                // lists for their lowest fit at or above the candidate, the maximum is the next
                // candidate, until no list moves it
                uint32_t memo[SEG_MEMO];
                bool have = false;
                uint32_t o = 0;
                for (;;) {
                    uint32_t best = o, j = 0;
                    for (uint32_t i = tid; i < nq; i += SEG_THREADS, ++j) {
                        const uint32_t id = seg_query_list(g, sp, i);
                        const uint32_t len = lens[id];
                        // Where to look first.  The first round asks from address 0 and is answered
                        // low in the list.  Later rounds: where this list answered before, or, for a
                        // long-lived variable whose candidate has jumped up, further up at the
                        // place the candidate would have if the holes were spread evenly below the
                        // list's top (one read for the top; it saves most of the climb: a third
                        // fewer list reads in all).
                        const uint64_t *L = pool + lst[id];
                        uint32_t idx = 0, he;
                        if (have) {
                            if (j < SEG_MEMO) idx = memo[j];
                            if (longv && len > 8) {
                                const uint32_t top = seg_start(L[len - 1]);
                                if (top) {
                                    const uint64_t at = (uint64_t)len * ((uint64_t)o + s) / top;
                                    idx = max(idx, (uint32_t)(at < len - 1 ? at : len - 1));
                                }
                            }
                        }
                        const uint32_t x = seg_fit(L, len, o, s, idx, he);
                        if (j < SEG_MEMO) memo[j] = idx;
                        best = max(best, x);
                    }
                    have = true;
                    best = seg_wave_max(best);
                    if (l == 0) s_max[flip][wave] = best;
                    __syncthreads();
                    best = max(max(s_max[flip][0], s_max[flip][1]), max(s_max[flip][2], s_max[flip][3]));
                    flip ^= 1;
                    if (TRIAL && longv) ++trial_rounds;
                    if (best == o) break;             // every list accepts o
                    o = best;
                }
                if (TRIAL && longv) ++trial_vars;
                const uint32_t en = o + s;
                fp = max(fp, en);
                if (tid == 0) offs[r0 + p] = (uint64_t)o << sh;      // rank order; un-permuted at the end
                for (uint32_t i = tid; i < nu; i += SEG_THREADS) {
                    const uint32_t id = seg_update_list(g, sp, i);
                    const uint32_t base = lst[id], cap = lst[id + 1] - base;
                    uint32_t len = lens[id];
                    // a list never outgrows its room (it sees at most cap - 1 blocks); the check
                    // keeps the stores inside the list whatever happens
                    if (seg_carve(pool + base, len, cap, o, en, longv ? len - 1 : 0u)) lens[id] = len;
                }
                __syncthreads();
            }
        }
        if (tid == 0 && !TRIAL) {
            A.fps[b] = (uint64_t)fp << sh;
            A.ticks[b] = (uint64_t)(wall_clock64() - t_begin);
        }
        __syncthreads();
        if (TRIAL) break;
    }
    if (TRIAL && tid == 0) {
        hdr->seg_trial_rounds = trial_rounds;
        hdr->seg_trial_vars = trial_vars;
        // (a handful of variables says nothing: then the lists stay)
        if (trial_vars >= 32 && (uint64_t)trial_rounds * 100 > (uint64_t)trial_vars * A.trial_percent) hdr->mode2 = 0;
    }
}

hipError_t launch_seg_prep(uint32_t n, uint32_t T, uint32_t B, const uint32_t *alloc, const uint32_t *free_,
                           PlanHeader *hdr, uint32_t *cnt, uint32_t *lst, uint32_t dir_cap, uint64_t pool_entries,
                           hipStream_t st)
{
    hipError_t e = launch_fill_u64((uint64_t *)cnt, ((size_t)dir_cap + 2) / 2, 0, st);
    if (e != hipSuccess) return e;
    uint32_t blocks = (n + 3) / 4;                 // 4 waves per block, one variable per wave and pass
    blocks = blocks < 1 ? 1 : (blocks > 2048 ? 2048 : blocks);
    hipLaunchKernelGGL(k_seg_count, dim3(blocks), dim3(256), 0, st, n, T, alloc, free_, hdr, cnt);
    hipLaunchKernelGGL(k_seg_scan, dim3(1), dim3(SEG_SCAN_THREADS), 0, st, T, B, hdr, cnt, lst, pool_entries);
    return hipGetLastError();
}

hipError_t launch_seg_trial(uint32_t n, uint32_t T, uint32_t B, const uint32_t *perm, const uint32_t *fits,
                            int trial_b, uint32_t trial_percent, PlanHeader *hdr, const void *vrec, const uint32_t *lst,
                            uint64_t *pool, uint32_t *lens, uint32_t dir_cap, uint64_t *offs, uint64_t *fps,
                            uint64_t *ticks, hipStream_t st)
{
    if (trial_b < 0 || trial_percent == 0) return hipSuccess;
    SegArgs A{n, T, B, (const uint4 *)vrec, perm, fits, hdr, lst, pool, lens, dir_cap, offs, fps, ticks, trial_b,
              trial_percent};
    hipLaunchKernelGGL(k_place_seg<true>, dim3(1), dim3(SEG_THREADS), 0, st, A);
    return hipGetLastError();
}

hipError_t launch_place_seg(uint32_t n, uint32_t T, uint32_t B, const uint32_t *perm, const uint32_t *fits,
                            bool any_first, PlanHeader *hdr, const void *vrec, const uint32_t *lst,
                            uint64_t *pool, uint32_t *lens, uint32_t dir_cap, uint64_t *offs, uint64_t *fps,
                            uint64_t *ticks, hipStream_t st)
{
    SegArgs A{n, T, B, (const uint4 *)vrec, perm, fits, hdr, lst, pool, lens, dir_cap, offs, fps, ticks, -1, 0};
    if (any_first) hipLaunchKernelGGL(k_place_seg<false>, dim3(B), dim3(SEG_THREADS), 0, st, A);
    return hipGetLastError();
}

}  // namespace lap
