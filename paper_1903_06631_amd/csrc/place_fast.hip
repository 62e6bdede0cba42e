// Placement of every variable under many orderings (Section III-C), first-fit or
// best-fit: the 32-bit granule path.
//
// Offsets are multiples of g = 2^shift, the largest power of two dividing every
// size (an offset is a sum of sizes).  When sum(size)/g < 2^32 every offset and
// block end fits 32 bits and a placed block packs into one 64-bit word
// (off << 32 | end), so sorting words sorts by offset.
//
// One workgroup of PW waves per ordering.  Two families of lists:
//
//   ALL    placed blocks with their lifetimes, sorted by offset: `main` and
//          `recent` (global memory, two buffers each, merged out of place) and
//          `pending` (LDS, unsorted, the newest).  Queried by variables that
//          live for more than one step: all waves sweep a sorted list together,
//          64 entries per wave step -- blocks that do not overlap the variable
//          in time are masked, a wave prefix-max of the remaining ends gives the
//          highest occupied address so far, and the first entry whose offset
//          leaves a hole of at least `size` above it ends the sweep (first-fit,
//          Section III-C: the lowest hole that is large enough).
//   L[t]   (only when the sum of all lifetimes, plus one per step, is at most
//          CL*N) the FREE address ranges ("holes") at step t, sorted by start,
//          packed (start << 32 | size), the last one reaching to 2^32-1;
//          followed by an unsorted tail of multi-step blocks that were placed
//          since and still have to be carved out.  A variable that lives for
//          exactly one step t only meets blocks live at t, so its first fit is
//          the first hole of L[t] that is large enough; taking it only shrinks
//          that hole in place (a fit always starts at a hole's start), and a hole
//          that is used up leaves the list.  The wave that works on step t holds
//          L[t] in its LDS slice.  With these lists in use, one-step blocks never
//          enter ALL: a multi-step variable asks the hole lists of its steps
//          instead (steps_fit_pass), in turn with the ALL sweeps, until neither
//          moves the candidate offset.
//
// Without the L[t] lists every variable queries ALL (the sweep).  First-fit orderings of large
// traces whose variables live long may instead be placed by free lists per time segment
// (place_seg.hip); k_plan_prep2 and a trial run decide, and this kernel then leaves them alone.
//
// One-step variables of different steps never interact, so between two
// multi-step variables of the rank order the waves work in parallel: wave w
// owns the steps t with t % PW == w.  Multi-step variables are handled by all
// waves between workgroup barriers.  The result is identical to placing the
// variables one by one in rank order.
#include "lap_dev.h"
#include "lap_kernels.h"

namespace lap {

constexpr int PW = 4;               // waves per ordering
constexpr uint32_t PEND = 128;      // room for the pending (unsorted) entries in LDS
constexpr uint32_t PEND_FLUSH = 32; // pending entries at which they are sorted into `recent`
constexpr uint32_t REC = PLAN_REC;  // recent (sorted) entries per buffer, global memory
constexpr uint32_t PACE_RANKS = 512; // a workgroup reports its progress every this many ranks (power of two)
constexpr uint32_t LH = 768;        // entries of a per-step list a wave can hold in LDS
constexpr uint32_t CL = PLAN_CL;    // per-step lists need sum of lifetimes <= CL * N

// orders this wave's earlier LDS / global accesses before its later ones (no barrier)
__device__ __forceinline__ void wave_fence() { __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup"); }

// orders this wave's LDS accesses for the compiler; the LDS unit serves a wave in order
__device__ __forceinline__ void lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ uint64_t pk(uint32_t off, uint32_t end) { return ((uint64_t)off << 32) | end; }

// A value every lane holds alike (all read the same address, or reduced it together), moved to
// scalar registers: what is computed from it, loop bounds and branch conditions above all,
// is then known to be the same in all lanes.
__device__ __forceinline__ uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ uint64_t uniform64(uint64_t v)
{
    return ((uint64_t)uniform((uint32_t)(v >> 32)) << 32) | uniform((uint32_t)v);
}

// A block's lifetime [alloc, free) next to its packed addresses: 64 bits in general, 32 bits
// (16 + 16) when the time line has at most 65535 steps -- a quarter less list traffic.
template <class LT> struct Life;
template <> struct Life<uint64_t> {
    static __device__ __forceinline__ uint64_t mk(uint32_t a, uint32_t f) { return ((uint64_t)a << 32) | f; }
    static __device__ __forceinline__ uint32_t a(uint64_t lf) { return (uint32_t)(lf >> 32); }
    static __device__ __forceinline__ uint32_t f(uint64_t lf) { return (uint32_t)lf; }
    static __device__ __forceinline__ uint64_t lane(uint64_t v, int l) { return read_lane64(v, l); }
};
template <> struct Life<uint32_t> {
    static __device__ __forceinline__ uint32_t mk(uint32_t a, uint32_t f) { return (a << 16) | f; }
    static __device__ __forceinline__ uint32_t a(uint32_t lf) { return lf >> 16; }
    static __device__ __forceinline__ uint32_t f(uint32_t lf) { return lf & 0xFFFFu; }
    static __device__ __forceinline__ uint32_t lane(uint32_t v, int l) { return read_lane(v, l); }
};

__device__ __forceinline__ uint32_t wave_scan_max32(uint32_t v) { return wave_scan_max_u32(v); }
__device__ __forceinline__ uint32_t wave_reduce_max32(uint32_t v) { return read_lane(wave_scan_max_u32(v), WAVE - 1); }

// ---------------------------------------------------------------------------
// preparation: granule shift, lifetime statistics, per-step list layout
// ---------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_plan_prep1(uint32_t n, uint32_t T, const uint64_t *__restrict__ size,
                                                    const uint32_t *__restrict__ alloc,
                                                    const uint32_t *__restrict__ free_, uint32_t *cntd,
                                                    PlanHeader *hdr)
{
    const uint32_t stride = gridDim.x * blockDim.x;
    unsigned long long orv = 0, sum = 0;
    unsigned long long seg[PLAN_SEG_CAND];
#pragma unroll
    for (uint32_t c = 0; c < PLAN_SEG_CAND; ++c) seg[c] = 0;
    uint32_t multi = 0;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint64_t s = size[i];
        const uint32_t a = alloc[i], f = free_[i];
        orv |= s;
        sum += s;
        multi += (f - a > 1) ? 1u : 0u;
        atomicAdd(&cntd[a], 1u);
        atomicAdd(&cntd[f], 0xFFFFFFFFu);          // -1 modulo 2^32
        // lists the block would enter with segments of 2^sh steps: one per segment it touches,
        // one more per segment it lives through, one per step in the others
#pragma unroll
        for (uint32_t c = 0; c < PLAN_SEG_CAND; ++c) {
            const uint32_t sh = PLAN_SEG_SHIFT0 + c, w = 1u << sh, K = (uint32_t)(((uint64_t)T + w - 1) >> sh);
            const uint32_t k0 = a >> sh, k1 = (f - 1) >> sh;
            const uint32_t kf0 = (uint32_t)(((uint64_t)a + w - 1) >> sh), kf1 = f == T ? K : f >> sh;
            const uint32_t nf = kf1 > kf0 ? kf1 - kf0 : 0;
            uint32_t steps = f - a;
            if (nf) {
                const uint64_t hi = (uint64_t)kf1 << sh;
                steps -= (uint32_t)((hi < T ? hi : (uint64_t)T) - ((uint64_t)kf0 << sh));
            }
            seg[c] += 1ull + (k1 - k0 + 1) + nf + steps;      // (the first: the list of everything)
        }
    }
    for (int m = WAVE / 2; m > 0; m >>= 1) orv |= shfl_xor64(orv, m);
    sum = wave_reduce_add(sum);
    multi = wave_reduce_add32(multi);
#pragma unroll
    for (uint32_t c = 0; c < PLAN_SEG_CAND; ++c) seg[c] = wave_reduce_add(seg[c]);
    if ((threadIdx.x & (WAVE - 1)) == 0) {
        atomicOr((unsigned long long *)&hdr->or_sizes, orv);
        atomicAdd((unsigned long long *)&hdr->sum_sizes, sum);
        atomicAdd(&hdr->n_multi, multi);
#pragma unroll
        for (uint32_t c = 0; c < PLAN_SEG_CAND; ++c) atomicAdd(&hdr->seg_tot[c], seg[c]);
    }
}

constexpr int PREP_THREADS = 1024;

__device__ __forceinline__ uint64_t prep_block_scan(uint64_t v, uint64_t *wtmp, uint64_t &total)
{
    const int tid = threadIdx.x, l = tid & (WAVE - 1), w = tid / WAVE;
    const uint64_t incl = wave_scan_add(v);
    if (l == WAVE - 1) wtmp[w] = incl;
    __syncthreads();
    uint64_t pre = 0, tot = 0;
    for (int k = 0; k < PREP_THREADS / WAVE; ++k) {
        const uint64_t x = wtmp[k];
        if (k < w) pre += x;
        tot += x;
    }
    __syncthreads();
    total = tot;
    return pre + incl;
}

// live[t] = number of variables live at step t; lstart = exclusive prefix sum of live + 1
__global__ __launch_bounds__(PREP_THREADS) void k_plan_prep2(uint32_t n, uint32_t T, uint32_t B,
                                                             const uint32_t *__restrict__ cntd,
                                                             uint32_t *__restrict__ lstart, PlanHeader *hdr,
                                                             uint64_t seg_pool_entries, uint64_t seg_min_vars)
{
    __shared__ uint64_t wtmp[PREP_THREADS / WAVE];
    const uint32_t tid = threadIdx.x;
    uint64_t c1 = 0, c2 = 0, tot;
    for (uint32_t base = 0; base < T; base += PREP_THREADS) {
        const uint32_t t = base + tid;
        const bool in = t < T;
        const uint64_t d = in ? (uint64_t)(int64_t)(int32_t)cntd[t] : 0;     // signed delta
        const uint64_t live = c1 + prep_block_scan(d, wtmp, tot); c1 += tot;
        // room for the holes: blocks + 1, rounded up to 16 entries so that every list starts on a
        // 128-byte line (a fetch of n entries then touches ceil(n / 16) lines, not one more)
        const uint64_t lv = in ? ((live + 1 + 15) & ~15ull) : 0;
        const uint64_t incl = c2 + prep_block_scan(lv, wtmp, tot);
        if (in) lstart[t] = (uint32_t)(incl - lv);
        c2 += tot;
    }
    if (tid == 0) {
        lstart[T] = (uint32_t)c2;
        const uint64_t orv = hdr->or_sizes, sum = hdr->sum_sizes;
        const uint32_t shift = orv ? (uint32_t)__ffsll((unsigned long long)orv) - 1 : 0;
        const bool fast = (sum >> shift) < (1ull << 32);
        const bool lists = fast && c2 <= (uint64_t)CL * n;
        hdr->shift = shift;
        hdr->fast = fast ? 1u : 0u;
        hdr->mode1 = lists ? 1u : 0u;
        // Segment lists: the width that enters the fewest blocks into lists; every list has one
        // entry more than the blocks it sees.  Taken when per-step lists are not, the trace has
        // enough variables for them to pay (below that, sweeping the sorted blocks is faster), the
        // list directory and one ordering fit 32-bit indices, addresses stay below the end marker
        // of the top range, and the pool has room for at least one ordering.
        uint32_t best_c = 0;
        uint64_t best_need = ~0ull;
        for (uint32_t c = 0; c < PLAN_SEG_CAND; ++c) {
            const uint32_t sh = PLAN_SEG_SHIFT0 + c;
            const uint64_t K = ((uint64_t)T + (1ull << sh) - 1) >> sh;
            const uint64_t need = hdr->seg_tot[c] + 2 * K + T + 1;
            if (need < best_need) { best_need = need; best_c = c; }
        }
        // ... or rather the narrowest width within an eighth of that: narrower segments mean fewer
        // lists per variable (a variable asks about lifetime / w + w of them)
        for (uint32_t c = 0; c < best_c; ++c) {
            const uint32_t sh = PLAN_SEG_SHIFT0 + c;
            const uint64_t K = ((uint64_t)T + (1ull << sh) - 1) >> sh;
            const uint64_t need = hdr->seg_tot[c] + 2 * K + T + 1;
            if (need <= best_need + best_need / 8) { best_need = need; best_c = c; break; }
        }
        const uint32_t ssh = PLAN_SEG_SHIFT0 + best_c;
        const uint64_t K = ((uint64_t)T + (1ull << ssh) - 1) >> ssh;
        const uint64_t slots = best_need ? seg_pool_entries / best_need : 0;
        const bool seg = fast && !lists && n >= seg_min_vars && (sum >> shift) < 0xFFFFFFFEull &&
                         best_need < 0xFFFFFFFFull && T < 0x7FFF0000u && slots >= 1;
        hdr->mode2 = seg ? 1u : 0u;
        hdr->seg_shift = ssh;
        hdr->seg_K = (uint32_t)K;
        hdr->seg_slots = (uint32_t)(slots < B ? slots : B);
        hdr->seg_need = best_need;
    }
}

// What the placement kernel reads of a variable, in one 16-byte record (one gather per rank
// instead of three): first step, end of life, size in granules.  Only meaningful on the
// 32-bit path (size >> shift fits 32 bits there).
__global__ __launch_bounds__(256) void k_plan_pack(uint32_t n, const uint64_t *__restrict__ size,
                                                   const uint32_t *__restrict__ alloc,
                                                   const uint32_t *__restrict__ free_, const PlanHeader *hdr,
                                                   uint4 *__restrict__ vrec)
{
    if (!hdr->fast) return;
    const uint32_t sh = hdr->shift;
    for (uint32_t v = blockIdx.x * 256 + threadIdx.x; v < n; v += gridDim.x * 256)
        vrec[v] = make_uint4(alloc[v], free_[v], (uint32_t)(size[v] >> sh), 0u);
}

// ---------------------------------------------------------------------------
// sorted lists of packed blocks (global memory or LDS), one wave
// ---------------------------------------------------------------------------

// insert (x, lf) at position p of a sorted list of n entries; `life` may be null
__device__ __forceinline__ void insert_at32(uint64_t *oe, uint64_t *life, uint32_t n, uint32_t p, uint64_t x,
                                            uint64_t lf)
{
    const int l = lane_id();
    uint32_t hi = n;
    while (hi > p) {
        const uint32_t lo = (hi - p > (uint32_t)WAVE) ? hi - WAVE : p;
        const uint32_t idx = lo + l;
        const bool act = idx < hi;
        uint64_t y = 0, z = 0;
        if (act) { y = oe[idx]; if (life) z = life[idx]; }
        // the stores carry the loaded values, so they issue after every lane's load; the
        // next iteration reads strictly lower indices than any store so far
        if (act) { oe[idx + 1] = y; if (life) life[idx + 1] = z; }
        hi = lo;
    }
    if (l == 0) { oe[p] = x; if (life) life[p] = lf; }
    wave_fence();
}

// index of the first of the nh holes of a list in memory with size >= s
__device__ __forceinline__ uint32_t mem_first_fit(const uint64_t *Lt, uint32_t nh, uint32_t s)
{
    const int l = lane_id();
    for (uint32_t base = 0; base < nh; base += WAVE) {
        const uint32_t idx = base + l;
        const uint64_t m = ballot(idx < nh && (uint32_t)Lt[idx < nh ? idx : 0] >= s);
        if (m) return base + __ffsll((unsigned long long)m) - 1;
    }
    return nh - 1;
}

// index of the hole of a list in memory that contains address o
__device__ __forceinline__ uint32_t mem_find_hole(const uint64_t *Lt, uint32_t nh, uint32_t o)
{
    const int l = lane_id();
    for (uint32_t base = 0; base < nh; base += WAVE) {
        const uint32_t idx = base + l;
        const uint64_t x = Lt[idx < nh ? idx : 0];
        const uint32_t st = (uint32_t)(x >> 32), sz = (uint32_t)x;
        const uint64_t m = ballot(idx < nh && st <= o && o - st < sz);
        if (m) return base + __ffsll((unsigned long long)m) - 1;
    }
    return nh - 1;
}

// bitonic sort of m (power of two, >= 64) packed entries with their lifetimes, in LDS, by the
// whole workgroup (a workgroup barrier after every compare-exchange stage)
template <class LT>
__device__ __forceinline__ void bitonic_sort(uint64_t *oe, LT *life, uint32_t m)
{
    for (uint32_t k = 2; k <= m; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = threadIdx.x; i < m / 2; i += PW * WAVE) {
                const uint32_t lo = ((i / j) * (j << 1)) + (i % j);
                const uint32_t hi = lo + j;
                const bool up = (lo & k) == 0;
                const uint64_t x = oe[lo], y = oe[hi];
                if ((x > y) == up) {
                    oe[lo] = y; oe[hi] = x;
                    const LT u = life[lo], v = life[hi];
                    life[lo] = v; life[hi] = u;
                }
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------
// a per-step hole list held in LDS by one wave (packed start << 32 | size, sorted by start)
// ---------------------------------------------------------------------------


// index of the first of the nh holes with size >= s (there always is one: the top hole)
__device__ __forceinline__ uint32_t h_first_fit(const uint64_t *hl, uint32_t nh, uint32_t s)
{
    const int l = lane_id();
    for (uint32_t base = 0; base < nh; base += 2 * WAVE) {
        const uint32_t i0 = base + l, i1 = base + WAVE + l;
        const uint32_t z0 = i0 < nh ? (uint32_t)hl[i0] : 0u;
        const uint32_t z1 = i1 < nh ? (uint32_t)hl[i1] : 0u;
        const uint64_t m0 = ballot(z0 >= s);                 // s >= 1, empty slots read as size 0
        if (m0) return base + __ffsll((unsigned long long)m0) - 1;
        const uint64_t m1 = ballot(z1 >= s);
        if (m1) return base + WAVE + __ffsll((unsigned long long)m1) - 1;
    }
    return nh - 1;
}

// Best-fit: index of the smallest of the nh-1 bounded holes with size >= s (the lowest of
// equally small ones); the unbounded top hole, the last entry, when none fits
__device__ __forceinline__ uint32_t h_best_fit(const uint64_t *hl, uint32_t nh, uint32_t s)
{
    const int l = lane_id();
    uint64_t best = U64_MAX;
    for (uint32_t base = 0; base + 1 < nh; base += WAVE) {
        const uint32_t idx = base + l;
        if (idx + 1 < nh) {
            const uint32_t z = (uint32_t)hl[idx];
            if (z >= s) best = umin64(best, ((uint64_t)z << 32) | idx);
        }
    }
#pragma unroll
    for (int m = WAVE / 2; m > 0; m >>= 1) best = umin64(best, shfl_xor64(best, m));
    return uniform(best == U64_MAX ? nh - 1 : (uint32_t)best);
}

// index of the hole that contains address o (start <= o < start + size); x receives the hole.
// Searched from the top chunk down: the blocks carved out of a list are those of multi-step
// variables, which mostly sit high.
__device__ __forceinline__ uint32_t h_find_hole(const uint64_t *hl, uint32_t nh, uint32_t o, uint64_t &x)
{
    const int l = lane_id();
    for (uint32_t base = (nh - 1) & ~(uint32_t)(WAVE - 1);; base -= WAVE) {
        const uint32_t idx = base + l;
        const uint64_t y = idx < nh ? hl[idx] : 0ull;
        const uint32_t st = (uint32_t)(y >> 32), sz = (uint32_t)y;
        const uint64_t m = ballot(st <= o && o - st < sz);
        if (m) {
            const int j = __ffsll((unsigned long long)m) - 1;
            x = read_lane64(y, j);
            return base + j;
        }
        if (base == 0) break;
    }
    x = uniform64(hl[nh - 1]);
    return nh - 1;
}

// entries [p, n) move up by one, x goes to position p
__device__ __forceinline__ void h_insert(uint64_t *hl, uint32_t n, uint32_t p, uint64_t x)
{
    const int l = lane_id();
    uint32_t hi = n;
    while (hi > p) {
        const uint32_t lo = (hi - p > (uint32_t)WAVE) ? hi - WAVE : p;
        const uint32_t idx = lo + l;
        uint64_t y = 0;
        if (idx < hi) y = hl[idx];
        lds_sync();
        if (idx < hi) hl[idx + 1] = y;
        hi = lo;
    }
    lds_sync();
    if (l == 0) hl[p] = x;
    lds_sync();
}

// entries (p, n) move down by one: entry p disappears
__device__ __forceinline__ void h_delete(uint64_t *hl, uint32_t n, uint32_t p)
{
    const int l = lane_id();
    for (uint32_t lo = p + 1; lo < n; lo += WAVE) {
        const uint32_t idx = lo + l;
        uint64_t y = 0;
        if (idx < n) y = hl[idx];
        lds_sync();
        if (idx < n) hl[idx - 1] = y;
        lds_sync();
    }
}

// Remove the block [o, en) from the nh free ranges in hl: it lies inside exactly one hole.
// Returns the number of holes afterwards; [lo, hi) is extended to the entries that changed.
// The top 64 holes are looked at first (multi-step blocks sit high); if the hole is among
// them, everything that has to move is already in registers: one LDS read in all.
__device__ __forceinline__ uint32_t h_carve(uint64_t *hl, uint32_t nh, uint32_t o, uint32_t en, uint32_t &lo,
                                            uint32_t &hi)
{
    const int l = lane_id();
    {
        const uint32_t base = (nh - 1) & ~(uint32_t)(WAVE - 1);
        const uint32_t idx = base + l;
        const uint64_t y = idx < nh ? hl[idx] : 0ull;
        const uint32_t yst = (uint32_t)(y >> 32), ysz = (uint32_t)y;
        const uint64_t m = ballot(yst <= o && o - yst < ysz);
        if (m) {
            const int j = __ffsll((unsigned long long)m) - 1;
            const uint64_t x = read_lane64(y, j);
            const uint32_t h = base + j, st = (uint32_t)(x >> 32), hend = st + (uint32_t)x;
            lo = min(lo, h);
            uint32_t left;
            if (o == st && en == hend) {            // used up: the holes above move down
                if (idx > h && idx < nh) hl[idx - 1] = y;
                hi = max(hi, nh - 1);
                left = nh - 1;
            } else if (o == st) {                   // shrinks from below
                if (l == j) hl[h] = pk(en, hend - en);
                hi = max(hi, h + 1);
                left = nh;
            } else if (en == hend) {                // shrinks from above
                if (l == j) hl[h] = pk(st, o - st);
                hi = max(hi, h + 1);
                left = nh;
            } else {                                // split: the holes above move up
                if (idx > h && idx < nh) hl[idx + 1] = y;
                if (l == j) { hl[h] = pk(st, o - st); hl[h + 1] = pk(en, hend - en); }
                hi = max(hi, nh + 1);
                left = nh + 1;
            }
            lds_sync();
            return left;
        }
    }
    uint64_t x;
    const uint32_t h = h_find_hole(hl, nh, o, x);
    const uint32_t st = (uint32_t)(x >> 32), hend = st + (uint32_t)x;
    lo = min(lo, h);
    lds_sync();
    if (o == st && en == hend) {         // the hole is used up: it leaves the list
        h_delete(hl, nh, h);
        hi = max(hi, nh - 1);
        return nh - 1;
    }
    if (o == st) {                       // block at the hole's start: the hole shrinks from below
        if (l == 0) hl[h] = pk(en, hend - en);
        lds_sync();
        hi = max(hi, h + 1);
        return nh;
    }
    if (l == 0) hl[h] = pk(st, o - st);  // lower part stays
    lds_sync();
    if (en == hend) { hi = max(hi, h + 1); return nh; }
    h_insert(hl, nh, h + 1, pk(en, hend - en));   // upper part: a new hole after it
    hi = max(hi, nh + 1);
    return nh + 1;
}

// ---------------------------------------------------------------------------
// the placement kernel
// ---------------------------------------------------------------------------

struct FastArgs {
    uint32_t n, T;
    const uint64_t *size;
    const uint32_t *alloc, *free_;
    const uint4 *vrec;           // [n] (first step, end of life, size in granules, -)
    const uint32_t *perm;        // [B][n]
    const uint32_t *fits;        // [B] 0 = first-fit, 1 = best-fit
    PlanHeader *hdr;
    const uint32_t *lstart;      // [T+1]
    uint64_t *m_oe[2];           // [B][n] x 2  ALL main list, two buffers (merges ping-pong)
    void *m_life[2];             //             lifetimes of its entries (32- or 64-bit words)
    uint64_t *r_oe[2];           // [B][REC] x 2  ALL recent list, two buffers
    void *r_life[2];
    uint64_t *L;                 // [B][capL]   per-step lists, packed blocks
    uint32_t *l_ns, *l_nu;       // [B][T]      sorted / unsorted entry counts; behind l_nu, [B][T] again: where
                                 //             the top (unbounded) hole of every list starts
    uint64_t capL;
    uint64_t *offs;              // [B][n] in rank order
    uint64_t *fps;               // [B]
    uint64_t *ticks;             // [B] duration of every ordering in timer ticks
};

constexpr int COOP_U = 4;                    // chunks per wave in one cooperative round
constexpr int ROUND_CH = PW * COOP_U;        // chunks per round
constexpr uint32_t NONE32 = 0xFFFFFFFFu;

// Lowest offset >= P at which `s` granules are free with respect to the time-overlapping
// entries of a short UNSORTED list: while some entry meets [P, P+s), move P to the highest
// end among those that do.
template <class LT>
__device__ __forceinline__ uint32_t fit_unsorted(const uint64_t *oe, const LT *life, uint32_t n, uint32_t P,
                                                 uint32_t s, uint32_t a, uint32_t f)
{
    const int l = lane_id();
    for (;;) {
        uint32_t top = 0;
        for (uint32_t base = 0; base < n; base += WAVE) {
            const uint32_t idx = base + l;
            if (idx < n) {
                const uint64_t x = oe[idx];
                const LT lf = life[idx];
                const uint32_t o = (uint32_t)(x >> 32), e = (uint32_t)x;
                const uint32_t ea = Life<LT>::a(lf), ef = Life<LT>::f(lf);
                if (ea < f && a < ef && e > P && o < P + s) top = max(top, e);   // P + s < 2^32
            }
        }
        top = wave_scan_max32(top);
        top = read_lane(top, WAVE - 1);
        if (top == 0) return P;
        P = top;
    }
}

// Readers of the smaller list of a merge: entry j for a wave-uniform, mostly ascending j.
template <class LT> struct LdsList {                 // the list sits in LDS
    const uint64_t *oe;
    const LT *life;
    __device__ __forceinline__ uint64_t key(uint32_t j) { return oe[j]; }
    __device__ __forceinline__ LT lifev(uint32_t j) { return life[j]; }
    // first index >= from (< n) whose key is not below `bound`
    __device__ __forceinline__ uint32_t advance(uint32_t from, uint32_t n, uint64_t bound)
    {
        uint32_t lo = from, hi = n;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (oe[mid] < bound) lo = mid + 1; else hi = mid;
        }
        return lo;
    }
};
template <class LT> struct GlobalWindow {   // the list sits in global memory: 64 entries at a time in registers
    const uint64_t *oe;
    const LT *life;
    uint32_t n, base;
    uint64_t w_oe;
    LT w_life;
    __device__ __forceinline__ void load(uint32_t b)
    {
        base = b;
        const uint32_t idx = b + lane_id();
        w_oe = idx < n ? oe[idx] : U64_MAX;
        w_life = idx < n ? life[idx] : 0;
    }
    __device__ __forceinline__ uint64_t key(uint32_t j)
    {
        if (j - base >= (uint32_t)WAVE) load(j & ~(uint32_t)(WAVE - 1));
        return read_lane64(w_oe, (int)(j - base));
    }
    __device__ __forceinline__ LT lifev(uint32_t j)
    {
        if (j - base >= (uint32_t)WAVE) load(j & ~(uint32_t)(WAVE - 1));
        return Life<LT>::lane(w_life, (int)(j - base));
    }
    __device__ __forceinline__ uint32_t advance(uint32_t from, uint32_t cnt, uint64_t bound)
    {
        while (from < cnt && key(from) < bound) ++from;
        return from;
    }
};

// Merge a sorted small list (ns entries, read through `sm`) and a sorted big list (global,
// nb entries) into another global buffer, with all PW waves; chunk c of the big list belongs
// to wave c % PW and chunks are independent.  A chunk moves its own entries up by the number
// of small-list entries below each, and writes the small-list entries whose place is inside
// it (after big-list entries of equal key).  No barrier inside; the caller synchronises
// before reading dst.
template <class LT, class Small>
__device__ __forceinline__ void coop_merge(const uint64_t *src_oe, const LT *src_life, uint32_t nb, Small sm,
                                           uint32_t ns, uint64_t *dst_oe, LT *dst_life, uint32_t wave)
{
    const int l = lane_id();
    const uint32_t nch = nb ? (nb + WAVE - 1) / WAVE : 1;
    uint32_t jp = 0;
    for (uint32_t c0 = wave; c0 < nch; c0 += 2 * PW) {
        uint64_t key[2], prevlast[2];
        LT lf[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t c = c0 + u * PW;
            const uint32_t idx = c * WAVE + l;
            key[u] = U64_MAX; lf[u] = 0; prevlast[u] = 0;
            if (c < nch) {
                if (idx < nb) { key[u] = src_oe[idx]; lf[u] = src_life[idx]; }
                if (c) prevlast[u] = src_oe[c * WAVE - 1];
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t c = c0 + u * PW;
            if (c < nch) {
                const uint32_t idx = c * WAVE + l;
                const bool valid = idx < nb;
                const bool last = c == nch - 1;
                const uint64_t lastkey = read_lane64(key[u], WAVE - 1);
                jp = sm.advance(jp, ns, prevlast[u]);
                uint32_t sh = jp, j = jp;
                while (j < ns) {
                    const uint64_t rk = sm.key(j);
                    if (!last && !(rk < lastkey)) break;
                    const LT rl = sm.lifev(j);
                    const uint32_t below = (uint32_t)__popcll(ballot(valid && key[u] <= rk));
                    if (l == 0) {
                        dst_oe[c * WAVE + below + j] = rk;
                        dst_life[c * WAVE + below + j] = rl;
                    }
                    sh += (valid && rk < key[u]) ? 1u : 0u;
                    ++j;
                }
                if (valid) { dst_oe[idx + sh] = key[u]; dst_life[idx + sh] = lf[u]; }
            }
        }
    }
}

// One sweep over a long sorted list with all PW waves: chunk q of a round belongs to wave
// q % PW.  Every wave scans its chunks, the chunk maxima are exchanged through LDS, each
// wave then tests its chunks for the first hole with the right carry, and the lowest hole
// of the round wins.  Two workgroup barriers per round; the next round's loads are issued
// before the current round is processed.  All waves pass the same arguments and get the
// same result.
template <class LT>
__device__ __forceinline__ uint32_t coop_sweep(const uint64_t *oe, const LT *life, uint32_t n,
                                               uint32_t &cursor, uint32_t P, uint32_t s, uint32_t a, uint32_t f,
                                               uint32_t wave, uint32_t *s_cmax, uint32_t *s_hq, uint32_t *s_hans)
{
    const int l = lane_id();
    uint32_t i = cursor;
    uint64_t x[COOP_U], nx[COOP_U];
    LT lf[COOP_U], nlf[COOP_U];
#pragma unroll
    for (int k = 0; k < COOP_U; ++k) {
        const uint32_t idx = i + (k * PW + wave) * WAVE + l;
        nx[k] = 0; nlf[k] = 0;
        if (idx < n) { nx[k] = oe[idx]; nlf[k] = life[idx]; }
    }
    for (;;) {
#pragma unroll
        for (int k = 0; k < COOP_U; ++k) { x[k] = nx[k]; lf[k] = nlf[k]; }
#pragma unroll
        for (int k = 0; k < COOP_U; ++k) {
            const uint32_t idx = i + ROUND_CH * WAVE + (k * PW + wave) * WAVE + l;
            nx[k] = 0; nlf[k] = 0;
            if (idx < n) { nx[k] = oe[idx]; nlf[k] = life[idx]; }
        }
        uint32_t incl[COOP_U];
#pragma unroll
        for (int k = 0; k < COOP_U; ++k) {
            const uint32_t idx = i + (k * PW + wave) * WAVE + l;
            uint32_t e = (uint32_t)x[k];
            const uint32_t ea = Life<LT>::a(lf[k]), ef = Life<LT>::f(lf[k]);
            if (idx >= n || !(ea < f && a < ef)) e = 0;
            incl[k] = wave_scan_max32(e);
            if (l == WAVE - 1) s_cmax[k * PW + wave] = incl[k];
        }
        __syncthreads();
        const uint32_t cm = (l < ROUND_CH) ? s_cmax[l] : 0;
        const uint32_t pin = wave_scan_max32(cm);
        const uint32_t total = read_lane(pin, ROUND_CH - 1);
        uint32_t best_q = NONE32, best_ans = 0;
#pragma unroll
        for (int k = 0; k < COOP_U; ++k) {
            const uint32_t q = k * PW + wave;
            const uint32_t idx = i + q * WAVE + l;
            const uint32_t carry = max(P, q ? (uint32_t)__shfl(pin, (int)q - 1, WAVE) : 0u);
            const uint32_t excl = lane_shift_up(incl[k], 0u);
            const uint32_t before = max(carry, excl);
            const uint32_t o = (uint32_t)(x[k] >> 32);
            const uint64_t hole = ballot(idx >= n || (o >= before && o - before >= s));
            if (hole && best_q == NONE32) {
                const int first = __ffsll((unsigned long long)hole) - 1;
                best_q = q * WAVE + first;
                best_ans = read_lane(before, first);
            }
        }
        if (l == 0) { s_hq[wave] = best_q; s_hans[wave] = best_ans; }
        __syncthreads();
        uint32_t hq = NONE32, ha = 0;
#pragma unroll
        for (int w = 0; w < PW; ++w) {
            const uint32_t q = s_hq[w];
            if (q < hq) { hq = q; ha = s_hans[w]; }
        }
        if (hq != NONE32) {
            cursor = i + hq;
            return ha;
        }
        P = max(P, total);
        i += ROUND_CH * WAVE;
    }
}

// One pass of a multi-step variable over the per-step hole lists of its lifetime [a, f):
// every thread takes steps a + tid, a + tid + 256, ... and finds the lowest offset >= o at
// which s granules fit into a hole of that step (binary search on the hole ends, which
// ascend with the starts, then a short walk); returns the largest such offset over the
// thread's steps.  Only the sorted part of a list (the holes) is read: blocks still waiting
// in a list's tail belong to multi-step variables, which the ALL list covers.  The topmost
// hole of every list is unbounded, so every search ends.
// Passes over unchanged lists with a rising o (valid0 / valid_rest say whether the thread's first
// step / its other steps have been asked before for this variable) reuse
// what the last search of a step found, kept for the thread's first FIT_MEMO steps in the
// wave's LDS slice `memo` (5 words per step, lane-interleaved; the slice holds no hole list
// while a multi-step variable is being placed): its answer, the end of the hole it lies in,
// that hole's index, and where the step's list starts and ends (so that a later search goes
// straight to the holes).  An answer at or above the new o still stands; below it, the same
// hole may still hold [o, o + s); otherwise the search resumes just above that hole, where
// the next answer is usually a few holes away.
constexpr uint32_t FIT_MEMO = 4;
constexpr uint32_t FIT_WORDS = 5;   // per step: answer, end of its hole, its index, list start, index of the top hole
static_assert(FIT_MEMO * FIT_WORDS * WAVE * sizeof(uint32_t) <= LH * sizeof(uint64_t), "the memo must fit the wave's list slice");
__device__ __forceinline__ uint32_t steps_fit_pass(const uint64_t *__restrict__ L, const uint32_t *__restrict__ lstart,
                                                   const uint32_t *l_ns, const uint32_t *l_top, uint32_t a, uint32_t f, uint32_t o,
                                                   uint32_t s, bool &valid0, bool &valid_rest, uint32_t *memo)
{
    // oq: the offset asked for, need = oq + s; from: holes below this index are known to end
    // below need; gallop: the answer is expected close above `from` (doubling steps first, then
    // the binary search between)
    auto search = [&](uint32_t base, uint32_t top, uint32_t oq, uint32_t need, uint32_t from_idx, bool gallop,
                      uint32_t &hole_idx, uint32_t &hole_end) -> uint32_t {
        const uint64_t *Lt = L + base;
        uint32_t lo = min(from_idx, top), hi = top;
        uint64_t xhi = 0;               // entry hi, once a probe has set hi
        bool have = false;
        if (gallop) {
            uint32_t step = 1;
            while (lo < hi) {
                const uint32_t p = min(lo + step - 1, hi - 1);
                const uint64_t x = Lt[p];
                if ((uint32_t)(x >> 32) + (uint32_t)x >= need) { hi = p; xhi = x; have = true; break; }
                lo = p + 1;
                step <<= 1;
            }
        }
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            const uint64_t x = Lt[mid];
            if ((uint32_t)(x >> 32) + (uint32_t)x >= need) { hi = mid; xhi = x; have = true; } else lo = mid + 1;
        }
        // lo == hi: the first hole that ends high enough (or the top one); walk up from it to
        // the first that fits
        uint64_t x = have ? xhi : Lt[lo];
        for (;;) {
            const uint32_t st = (uint32_t)(x >> 32), from = max(oq, st);
            if (st + (uint32_t)x - from >= s) {
                hole_idx = lo;
                hole_end = lo >= top ? NONE32 : st + (uint32_t)x;
                return from;
            }
            ++lo;
            x = Lt[lo];
        }
    };
    // The thread's steps are taken in rounds of 256 steps (64 per wave); after each round the
    // wave's highest answer becomes the offset asked for in the next, so that a pass over a long
    // lifetime climbs as far as two or three passes over a short one.  (Any offset up to the
    // pass's result is a valid question: the final answer lies at or above it.)
    uint32_t best = o;
    uint32_t *mm = memo + lane_id();
    const uint32_t rounds = (f - a + PW * WAVE - 1) / (PW * WAVE);
    // ... and the wave goes over its own steps again until they all accept its answer: an offset
    // that fails among 64 * rounds steps is dropped without asking the other three quarters.
    // A thread's steps are neighbours (step a + tid * rounds + k in round k), so round 0 alone
    // is a sample of the whole lifetime, every rounds-th step: the wave first settles on an
    // offset among those (a lower bound that is cheap to raise, and for a small variable that
    // lives long it takes dozens of sweeps to raise it), then among all its steps.
    for (uint32_t kmax = rounds > 1 ? 1 : rounds; ; kmax = rounds) {
    for (;;) {
    const uint32_t sweep_from = best;
    for (uint32_t k = 0; k < kmax; ++k) {
        const uint32_t t = a + threadIdx.x * rounds + k;
        uint32_t at = best;
        if (t < f) {
            const uint32_t oq = best, need = oq + s;
            const bool kept = k < FIT_MEMO;
            uint32_t *mk = mm + k * FIT_WORDS * WAVE;
            uint32_t from_idx = 0, base, top;
            bool done = false;
            if (kept && (k == 0 ? valid0 : valid_rest)) {
                const uint32_t m_at = mk[0], m_end = mk[WAVE], m_lo = mk[2 * WAVE];
                if (m_at >= oq) { at = m_at; done = true; }
                else if (m_end >= need) done = true;        // fits at oq itself
                else { from_idx = m_lo + 1; base = mk[3 * WAVE]; top = mk[4 * WAVE]; }
            }
            if (!done) {
                if (from_idx == 0) {
                    base = lstart[t];
                    top = max(l_ns[t], 1u) - 1;
                    if (kept) { mk[3 * WAVE] = base; mk[4 * WAVE] = top; }
                }
                uint32_t idx, end;
                if (oq >= l_top[t]) {           // inside the top hole, where multi-step blocks nearly always go: no list read
                    at = oq;
                    idx = top;
                    end = NONE32;
                } else {
                    at = search(base, top, oq, need, from_idx, from_idx != 0, idx, end);
                }
                if (kept) { mk[0] = at; mk[WAVE] = end; mk[2 * WAVE] = idx; }
            }
        }
        best = wave_reduce_max32(at);
    }
    valid0 = true;                          // the notes of the steps just asked now hold
    if (kmax == rounds) valid_rest = true;
    if (best == sweep_from) break;
    }
    if (kmax == rounds) break;
    }
    return best;
}

// Best-fit needs the size of the hole that starts at a feasible offset p.  In the hole lists:
// the lowest end, over the steps of [a, f), of the hole that holds p (0xFFFFFFFF = unbounded).
// p comes from a fixed point of steps_fit_pass, whose last pass found, for every step, the
// hole that holds [p, p + s): its end is still in `memo` for the thread's first FIT_MEMO
// steps; later steps look their hole up (the first whose end lies above p).
__device__ __forceinline__ uint32_t steps_extent_pass(const uint64_t *__restrict__ L,
                                                      const uint32_t *__restrict__ lstart, const uint32_t *l_ns,
                                                      uint32_t a, uint32_t f, uint32_t p, const uint32_t *memo)
{
    uint32_t e = NONE32;
    const uint32_t *mm = memo + lane_id();
    const uint32_t rounds = (f - a + PW * WAVE - 1) / (PW * WAVE);     // same steps per thread as steps_fit_pass
    for (uint32_t k = 0; k < rounds; ++k) {
        const uint32_t t = a + threadIdx.x * rounds + k;
        if (t >= f) break;
        if (k < FIT_MEMO) {
            e = min(e, mm[(k * FIT_WORDS + 1) * WAVE]);
            continue;
        }
        const uint64_t *Lt = L + lstart[t];
        uint32_t lo = 0, hi = max(l_ns[t], 1u) - 1;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            const uint64_t x = Lt[mid];
            if ((uint32_t)(x >> 32) + (uint32_t)x > p) hi = mid; else lo = mid + 1;
        }
        const uint64_t x = Lt[lo];
        e = min(e, (uint32_t)(x >> 32) + (uint32_t)x);
    }
    return e;
}

// In a sorted list: offset of the first entry at or after index `from` that overlaps [a, f) in
// time, 0xFFFFFFFF if there is none.  All waves call it with the same arguments.
template <class LT>
__device__ __forceinline__ uint32_t coop_next_overlap(const uint64_t *oe, const LT *life, uint32_t n, uint32_t from,
                                                      uint32_t a, uint32_t f, uint32_t wave, uint32_t *s_x)
{
    const int l = lane_id();
    for (uint32_t base = from; base < n; base += PW * WAVE) {
        const uint32_t idx = base + wave * WAVE + l;
        bool hit = false;
        uint32_t off = 0;
        if (idx < n) {
            const uint64_t x = oe[idx];
            const LT lf = life[idx];
            hit = Life<LT>::a(lf) < f && a < Life<LT>::f(lf);
            off = (uint32_t)(x >> 32);
        }
        const uint64_t m = ballot(hit);
        uint32_t first = NONE32;
        if (m) first = read_lane(off, __ffsll((unsigned long long)m) - 1);
        if (l == 0) s_x[wave] = first;
        __syncthreads();
        uint32_t r = NONE32;
#pragma unroll
        for (int w = PW - 1; w >= 0; --w)
            if (s_x[w] != NONE32) r = s_x[w];         // the lowest wave's chunk comes first in the list
        __syncthreads();
        if (r != NONE32) return r;
    }
    return NONE32;
}

// A list of `tot` entries moves between global memory, registers (entry i in register i / 64
// of lane i % 64) and LDS in chunks of 64; the chain of tests ends at the first chunk that
// lies beyond the list, so a short list costs few branches.
template <int C>
__device__ __forceinline__ void regs_from_global(uint64_t (&r)[LH / WAVE], const uint64_t *src, uint32_t tot, int l)
{
    if constexpr (C < (int)(LH / WAVE)) {
        if ((uint32_t)C * WAVE < tot) {
            const uint32_t idx = C * WAVE + l;
            r[C] = idx < tot ? src[idx] : 0ull;
            regs_from_global<C + 1>(r, src, tot, l);
        }
    }
}
template <int C>
__device__ __forceinline__ void lds_from_regs(uint64_t *hl, const uint64_t (&r)[LH / WAVE], uint32_t tot, int l)
{
    if constexpr (C < (int)(LH / WAVE)) {
        if ((uint32_t)C * WAVE < tot) {
            const uint32_t idx = C * WAVE + l;
            if (idx < tot) hl[idx] = r[C];
            lds_from_regs<C + 1>(hl, r, tot, l);
        }
    }
}

template <class LT, bool BEST>
__global__ __launch_bounds__(PW *WAVE, 4) void k_place_fast(FastArgs A)
{
    __shared__ uint64_t p_oe[PEND];
    __shared__ LT p_life[PEND];
    __shared__ uint64_t s_h[PW][LH];         // per-wave hole list
    __shared__ uint32_t s_fp[PW], s_hq[PW], s_hans[PW];
    __shared__ uint32_t s_cmax[ROUND_CH];
    __shared__ uint32_t s_sf[2][PW];
    __shared__ uint32_t s_prio;              // wave priority in force for this workgroup

    if (!A.hdr->fast) return;               // the 64-bit kernel handles this trace
    if (A.hdr->mode2 && !BEST) return;      // the segment kernel places the first-fit orderings of this trace
    const uint32_t b = blockIdx.x;
    if ((A.fits[b] != 0) != BEST) return;   // the other instantiation handles this ordering
    const long long t_begin = wall_clock64();
    const bool mode1 = A.hdr->mode1 != 0;
    const uint32_t sh = A.hdr->shift;
    const int l = lane_id();
    const uint32_t wave = threadIdx.x / WAVE;

    const uint32_t n = A.n, T = A.T;
    const uint32_t *perm = A.perm + (size_t)b * n;
    uint64_t *m_oe[2] = {A.m_oe[0] + (size_t)b * n, A.m_oe[1] + (size_t)b * n};
    LT *m_life[2] = {(LT *)A.m_life[0] + (size_t)b * n, (LT *)A.m_life[1] + (size_t)b * n};
    uint64_t *r_oe[2] = {A.r_oe[0] + (size_t)b * REC, A.r_oe[1] + (size_t)b * REC};
    LT *r_life[2] = {(LT *)A.r_life[0] + (size_t)b * REC, (LT *)A.r_life[1] + (size_t)b * REC};
    uint64_t *hl = s_h[wave];
    uint64_t *L = A.L + (size_t)b * A.capL;
    uint32_t *l_ns = A.l_ns + (size_t)b * T;
    uint32_t *l_nu = A.l_nu + (size_t)b * T;
    uint32_t *l_top = A.l_nu + (size_t)gridDim.x * T + (size_t)b * T;
    uint64_t *offs = A.offs + (size_t)b * n;

    // variables that will still query ALL: every one when there are no per-step lists
    uint32_t multi_left = mode1 ? A.hdr->n_multi : n;
    // ALL list state, identical in every wave: main / recent buffer in use, their counts
    uint32_t mb = 0, rb = 0, nm = 0, nr = 0;
    uint32_t np_multi = 0;      // pending entries (they come from ALL queries and tend to stack)
    uint32_t fp = 0;
    // Pacing.  The launch ends with its slowest ordering, and orderings differ: by what they
    // hold (some need more passes), and by where their workgroup sits (the hardware issues
    // older waves first, so the workgroup that reached a CU last runs about a tenth slower).
    // Every 512 ranks a workgroup adds one to a global count and compares its own progress
    // with the mean over all: behind the mean it raises the issue priority of its waves,
    // ahead of it it lowers it.  That evens out the second effect; the first remains (pausing
    // the orderings that are ahead does not speed up the ones behind).
    uint32_t *g_part = &A.hdr->part[BEST ? 1 : 0], *g_prog = &A.hdr->progress[BEST ? 1 : 0];
    if (threadIdx.x == 0) {
        atomicAdd(g_part, 1u);
        s_prio = 1;
    }
    if (mode1) {
        // every step starts with one hole covering the whole address space
        for (uint32_t t = threadIdx.x; t < T; t += PW * WAVE) {
            L[A.lstart[t]] = pk(0u, NONE32);
            l_ns[t] = 1;
            l_top[t] = 0;
        }
    }
    __syncthreads();

    // this wave's register-resident per-step list: step, entries, hole count, range of
    // indices not yet written back; wmask remembers (hashed) which lists were stored since
    // the last fence
    uint32_t cur_t = NONE32, cur_base = 0, cnt = 0, wb_from = NONE32, wb_to = 0;
    // one more changed entry outside that range: a hole shrunk low in the list, while the range
    // covers what carving changed high up (one range over both would rewrite the whole list)
    uint32_t wb_one = NONE32;
    uint64_t wmask = 0;
    // per lane, for the one-step variable of this lane's rank: list start, sorted and
    // unsorted entry counts of its step (kept current by the code below)
    uint32_t plb = 0, pns = 0, pnu = 0;

    auto writeback = [&](uint32_t a_lane) {
        if (cur_t != NONE32 && (wb_from != NONE32 || wb_one != NONE32)) {
            uint64_t *Lt = L + cur_base;
            for (uint32_t idx = wb_from + l; idx < wb_to; idx += WAVE) Lt[idx] = hl[idx];
            if (l == 0) {
                if (wb_one != NONE32 && (wb_one < wb_from || wb_one >= wb_to)) Lt[wb_one] = hl[wb_one];
                l_ns[cur_t] = cnt;
                l_nu[cur_t] = 0;
                l_top[cur_t] = (uint32_t)(hl[cnt - 1] >> 32);
            }
            wmask |= 1ull << ((cur_t / PW) & 63);
        }
        if (cur_t != NONE32 && a_lane == cur_t) { pns = cnt; pnu = 0; }
        wb_from = NONE32;
        wb_to = 0;
        wb_one = NONE32;
    };

    // pending -> recent, and recent -> main when recent cannot take it (all waves call it)
    auto flush = [&](uint32_t np) {
        if (np == 0) return;
        if (nr + np > REC) {
            GlobalWindow<LT> gw{r_oe[rb], r_life[rb], nr, 0, 0, 0};
            gw.load(0);
            coop_merge(m_oe[mb], m_life[mb], nm, gw, nr, m_oe[mb ^ 1], m_life[mb ^ 1], wave);
            mb ^= 1;
            nm += nr;
            nr = 0;
            __syncthreads();
        }
        uint32_t m = WAVE;
        while (m < np) m <<= 1;
        for (uint32_t i = np + threadIdx.x; i < m; i += PW * WAVE) { p_oe[i] = U64_MAX; p_life[i] = 0; }
        __syncthreads();
        bitonic_sort(p_oe, p_life, m);
        coop_merge(r_oe[rb], r_life[rb], nr, LdsList<LT>{p_oe, p_life}, np, r_oe[rb ^ 1], r_life[rb ^ 1], wave);
        rb ^= 1;
        nr += np;
        np_multi = 0;
        __syncthreads();
    };

    uint32_t prio_now = 1;
    __builtin_amdgcn_s_setprio(1);
    // The variables of a window come through two dependent loads (rank -> variable -> record).
    // They are fetched ahead: while a window is worked on, the records of the next one and the
    // variable numbers of the one after are on their way, so a window starts with its records
    // in registers.
    uint4 rec_next = make_uint4(0u, 1u, 0u, 0u);
    uint32_t v_next = 0;
    if ((uint32_t)l < n) rec_next = A.vrec[perm[l]];
    if ((uint32_t)l + WAVE < n) v_next = perm[l + WAVE];
    for (uint32_t r0 = 0; r0 < n; r0 += WAVE) {
        if (r0 && (r0 & (PACE_RANKS - 1)) == 0) {
            if (threadIdx.x == 0) {
                const uint32_t done = atomicAdd(g_prog, 1u) + 1u;
                const uint32_t started = max(*(volatile uint32_t *)g_part, 1u);
                const int lag = (int)(done / started) - (int)(r0 / PACE_RANKS);
                *(volatile uint32_t *)&s_prio = lag >= 2 ? 3u : lag >= 0 ? 2u : lag >= -2 ? 1u : 0u;
            }
            const uint32_t want = uniform(*(volatile uint32_t *)&s_prio);
            if (want != prio_now) {
                prio_now = want;
                if (want == 0) __builtin_amdgcn_s_setprio(0);
                else if (want == 1) __builtin_amdgcn_s_setprio(1);
                else if (want == 2) __builtin_amdgcn_s_setprio(2);
                else __builtin_amdgcn_s_setprio(3);
            }
        }
        const uint32_t ridx = r0 + l;
        const bool in = ridx < n;
        uint32_t a = 0, f = 1, s = 0;
        if (in) {
            a = rec_next.x;
            f = rec_next.y;
            s = rec_next.z;
        }
        if (ridx + WAVE < n) rec_next = A.vrec[v_next];
        if (ridx + 2 * WAVE < n) v_next = perm[ridx + 2 * WAVE];
        const uint64_t im = ballot(in);
        const uint64_t mm = ballot(in && (!mode1 || f - a > 1));
        const uint32_t wn = (uint32_t)__popcll(im);
        const bool one_step = in && mode1 && f - a == 1;
        const bool own = one_step && (a % PW) == wave;       // only the owner of a step looks at its list
        if (own) { plb = A.lstart[a]; pns = l_ns[a]; pnu = l_nu[a]; }
        if (cur_t != NONE32 && one_step && a == cur_t) { pns = cnt; pnu = 0; }   // the cached list is newer
        uint32_t p = 0;
        while (p < wn) {
            if ((mm >> p) & 1ull) {
                // ---- a variable that queries ALL: every wave sweeps, wave 0 keeps recent ----
                if (cur_t != NONE32) { writeback(one_step ? a : NONE32); cur_t = NONE32; }
                __syncthreads();
                const uint32_t va = __shfl(a, (int)p, WAVE);
                const uint32_t vf = __shfl(f, (int)p, WAVE), vs = __shfl(s, (int)p, WAVE);
                // pending stays unsorted and is checked directly, unless many of its entries come
                // from ALL queries: those stack on each other and would be climbed one by one
                uint32_t np = np_multi;             // every pending entry comes from a query like this one
                if (np >= PEND_FLUSH) {
                    flush(np);
                    np = 0;
                }
                uint32_t cm = 0, cr = 0;
                // no hole-list pass yet for this variable (the lists do not change and the candidate
                // only rises while it is being placed, so later passes may build on earlier ones)
                bool valid0 = false, valid_rest = false;   // (per thread: of its first step, of its other steps)
                // lowest offset >= `from` that is free of every neighbour: the sorted lists, the
                // pending entries and (with per-step lists) the hole lists are asked in turn until
                // none of them moves the candidate
                auto fit_from = [&](uint32_t from) -> uint32_t {
                    uint32_t o = from;
                    bool steps_hold = false;         // the hole lists have confirmed the current candidate
                    uint32_t flip = 0;
                    for (;;) {
                        // the block lists: lowest offset >= o that is free of their time-overlapping entries
                        uint32_t o1 = o;
                        if (nm) o1 = coop_sweep(m_oe[mb], m_life[mb], nm, cm, o, vs, va, vf, wave, s_cmax, s_hq, s_hans);
                        else __syncthreads();      // (keeps this pass's exchange slots apart from the last one's)
                        uint32_t o2 = o1;
                        if (nr)
                            o2 = coop_sweep(r_oe[rb], r_life[rb], nr, cr, o1, vs, va, vf, wave, s_cmax, s_hq, s_hans);
                        // the few pending entries: every wave checks them by itself (same data, same answer)
                        if (np) o2 = fit_unsorted(p_oe, p_life, np, o2, vs, va, vf);
                        if (!mode1) {
                            if (o2 == o1) return o2;             // recent and pending agree with main's answer
                            o = o2;
                            continue;
                        }
                        if (o2 == o && steps_hold) return o;     // nothing moved since the hole lists agreed
                        // one-step variables are not in ALL: the hole lists of the steps it lives through
                        // stand for them.  Passes repeat until no step moves the candidate.
                        uint32_t os = o2;
                        for (;;) {
                            uint32_t c = steps_fit_pass(L, A.lstart, l_ns, l_top, va, vf, os, vs, valid0, valid_rest, (uint32_t *)hl);
                            c = wave_reduce_max32(c);
                            if (l == 0) s_sf[flip][wave] = c;
                            __syncthreads();
                            c = max(max(s_sf[flip][0], s_sf[flip][1]), max(s_sf[flip][2], s_sf[flip][3]));
                            flip ^= 1;
                            if (c == os) break;
                            os = c;
                        }
                        // o2 == o1: recent and pending left main's answer alone, so all block lists accept o2;
                        // os == o2: so do the hole lists
                        if (os == o2 && o2 == o1) return os;
                        o = os;
                        steps_hold = true;
                    }
                };
                uint32_t o;
                if constexpr (!BEST) {
                    o = fit_from(0);
                } else {
                    // Best-fit: the feasible offsets found in ascending order are the starts of the
                    // holes that fit; a hole ends at the lowest start of a neighbour above it.  The
                    // smallest such hole wins, the first of equally small ones; an exact fit ends the
                    // search; with no neighbour above, the offset is the top of the neighbours.
                    uint32_t best_gap = NONE32, best_off = 0, from = 0;
                    for (;;) {
                        const uint32_t pp = fit_from(from);
                        __syncthreads();
                        // the sweeps stopped at the first entry above the hole: the next neighbour is
                        // the first time-overlapping entry from there on
                        uint32_t e = coop_next_overlap(m_oe[mb], m_life[mb], nm, cm, va, vf, wave, s_hq);
                        e = min(e, coop_next_overlap(r_oe[rb], r_life[rb], nr, cr, va, vf, wave, s_hq));
                        uint32_t c = NONE32;
                        if (wave == 0) {
                            for (uint32_t idx = l; idx < np; idx += WAVE) {
                                const LT lf = p_life[idx];
                                const uint32_t po = (uint32_t)(p_oe[idx] >> 32);
                                if (Life<LT>::a(lf) < vf && va < Life<LT>::f(lf) && po >= pp) c = min(c, po);
                            }
                        }
                        if (mode1) c = min(c, steps_extent_pass(L, A.lstart, l_ns, va, vf, pp, (const uint32_t *)hl));
                        c = ~wave_reduce_max32(~c);
                        if (l == 0) s_sf[0][wave] = c;
                        __syncthreads();
                        e = min(e, min(min(s_sf[0][0], s_sf[0][1]), min(s_sf[0][2], s_sf[0][3])));
                        __syncthreads();
                        if (e == NONE32) { o = best_gap == NONE32 ? pp : best_off; break; }
                        const uint32_t gap = e - pp;
                        if (gap < best_gap) { best_gap = gap; best_off = pp; }
                        if (gap == vs) { o = pp; break; }
                        from = e;
                    }
                }
                const uint32_t en = o + vs;
                fp = max(fp, en);
                if (threadIdx.x == 0) {
                    offs[r0 + p] = (uint64_t)o << sh;        // offsets are kept in rank order
                    if (multi_left > 1) {               // someone will still query ALL
                        p_oe[np] = pk(o, en);
                        p_life[np] = Life<LT>::mk(va, vf);
                    }
                }
                if (multi_left > 1) ++np_multi;
                if (mode1) {
                    // The block enters the list of every step it covers.  Where it lies in the list's
                    // top hole (nearly always) and no block is waiting there, it is taken out right
                    // away: the top hole moves up, and a hole may be left below it.  Otherwise it waits
                    // in the list's unsorted tail for the next one-step variable of that step.
                    const uint64_t x = pk(o, en);
                    for (uint32_t t = va + wave * WAVE + l; t < vf; t += PW * WAVE) {
                        const uint32_t ns = l_ns[t], nu = l_nu[t], tp = l_top[t];
                        uint64_t *Lt = L + A.lstart[t];
                        if (nu == 0 && o >= tp) {
                            uint32_t k = ns - 1;
                            if (o > tp) {
                                Lt[k] = pk(tp, o - tp);
                                ++k;
                                l_ns[t] = k + 1;
                            }
                            Lt[k] = pk(en, NONE32 - en);
                            l_top[t] = en;
                        } else {
                            Lt[ns + nu] = x;
                            l_nu[t] = nu + 1;
                        }
                    }
                }
                --multi_left;
                __syncthreads();
                // the tails of the steps it covers grew: refresh the counts of the ranks to come
                if (own && (uint32_t)l > p && a >= va && a < vf) { pns = l_ns[a]; pnu = l_nu[a]; }
                ++p;
            } else {
                // ---- a run of one-step variables: each wave takes the steps it owns --------
                const uint64_t rest = (~mm & im) >> p;
                const uint32_t run = (~rest == 0ull) ? 64u : (uint32_t)(__ffsll((unsigned long long)~rest) - 1);
                const uint32_t q = p + run;
                uint64_t mine = ballot((uint32_t)l >= p && (uint32_t)l < q && (a % PW) == wave);
                // results stay in the lane of their rank until the run ends: one store then, none
                // in flight while the next list is waited for
                const bool my_rank = (mine >> l) & 1ull;
                uint32_t res = 0;
                // the list of the NEXT variable of this wave is fetched into registers while the
                // current one is being placed
                uint64_t pf[LH / WAVE];
                uint32_t pf_t = NONE32;
                uint64_t fc = 0;                    // ... or, for the short path below, its first 64 holes only
                uint32_t fc_t = NONE32;
                uint32_t fail_t = NONE32;           // step whose last variable needed the full path
#pragma unroll
                for (int c = 0; c < (int)(LH / WAVE); ++c) pf[c] = 0;
                while (mine) {
                    int j = __ffsll((unsigned long long)mine) - 1;
                    mine &= mine - 1;
                    const uint32_t t = read_lane(a, j);
                    uint32_t vs = read_lane(s, j), o = 0;
                    // Nearly every one-step variable finds its hole among the first few of its
                    // step's list (at the benchmark's configuration 97 % among the first 16) and
                    // takes its lower end: the first 64 holes, fetched ahead while the variable
                    // before was placed, one ballot, one entry written back.  Everything else
                    // (blocks waiting in the list's tail, no fit among the first 64, a hole used up,
                    // the list already in LDS, best-fit) takes the full path below.
                    bool placed = false;
                    const bool same_next = mine != 0 && read_lane(a, __ffsll((unsigned long long)mine) - 1) == t;
                    if (!BEST && t != cur_t && read_lane(pnu, j) == 0) {
                        const uint32_t base = read_lane(plb, j), ns = read_lane(pns, j);
                        uint64_t y = fc;
                        if (fc_t != t) {
                            if (wmask & (1ull << ((t / PW) & 63))) { wave_fence(); wmask = 0; }
                            y = (uint32_t)l < ns ? L[base + l] : 0ull;
                        }
                        fc_t = NONE32;
                        const uint64_t m = ballot((uint32_t)l < ns && (uint32_t)y >= vs);
                        if (m) {
                            const int h = __ffsll((unsigned long long)m) - 1;
                            const uint64_t x = read_lane64(y, h);
                            if ((uint32_t)x != vs) {              // the hole shrinks from below
                                // the next variable's first holes are asked for only now that this
                                // one's have arrived: the wait for these must not take in that read
                                if (mine && !same_next) {
                                    const int jn = __ffsll((unsigned long long)mine) - 1;
                                    const uint32_t tn = read_lane(a, jn);
                                    if (tn != t && tn != cur_t && read_lane(pnu, jn) == 0 && !(wmask & (1ull << ((tn / PW) & 63)))) {
                                        fc = (uint32_t)l < read_lane(pns, jn) ? L[read_lane(plb, jn) + l] : 0ull;
                                        fc_t = tn;
                                    }
                                }
                                o = (uint32_t)(x >> 32);
                                const uint64_t z = pk(o + vs, (uint32_t)x - vs);
                                if (l == 0) {
                                    L[base + h] = z;
                                    if ((uint32_t)h + 1 == ns) l_top[t] = o + vs;
                                }
                                if (l == h) y = z;
                                // The wave's next variables of the same step (in orders that keep a
                                // step's variables together, all of them) are placed from these
                                // registers, nothing read: a ballot, one entry stored.
                                while (mine) {
                                    const int jn = __ffsll((unsigned long long)mine) - 1;
                                    if (read_lane(a, jn) != t) break;
                                    const uint32_t vn = read_lane(s, jn);
                                    const uint64_t mn = ballot((uint32_t)l < ns && (uint32_t)y >= vn);
                                    if (!mn) break;
                                    const int hn = __ffsll((unsigned long long)mn) - 1;
                                    const uint64_t xn = read_lane64(y, hn);
                                    if ((uint32_t)xn == vn) break;
                                    fp = max(fp, o + vs);       // the one before is done
                                    if (l == j) res = o;
                                    mine &= mine - 1;
                                    j = jn;
                                    vs = vn;
                                    o = (uint32_t)(xn >> 32);
                                    const uint64_t zn = pk(o + vn, (uint32_t)xn - vn);
                                    if (l == 0) {
                                        L[base + hn] = zn;
                                        if ((uint32_t)hn + 1 == ns) l_top[t] = o + vn;
                                    }
                                    if (l == hn) y = zn;
                                }
                                wmask |= 1ull << ((t / PW) & 63);
                                pf_t = NONE32;      // (a whole list fetched ahead by the full path is stale now, if it is this one)
                                fail_t = NONE32;
                                placed = true;
                            }
                        }
                    }
                    if (!placed) {
                        fc_t = NONE32;
                        if (t != cur_t) {
                            writeback(one_step ? a : NONE32);
                            cur_t = NONE32;
                            const uint32_t base = read_lane(plb, j);
                            const uint32_t ns = read_lane(pns, j), nu = read_lane(pnu, j), tot = ns + nu;
                            if (pf_t != t && (wmask & (1ull << ((t / PW) & 63)))) { wave_fence(); wmask = 0; }
                            if (tot + 1 <= LH) {
                                if (pf_t == t) {
                                    lds_from_regs<0>(hl, pf, tot, l);
                                } else {
                                    // not fetched ahead (the first of a run, mostly): all its chunks are
                                    // asked for before the first is waited for
                                    const uint64_t *Lt = L + base;
                                    uint32_t done = 0;
                                    if (tot <= 4 * WAVE) {
                                        uint64_t y[4];
    #pragma unroll
                                        for (int c = 0; c < 4; ++c) {
                                            const uint32_t idx = c * WAVE + l;
                                            y[c] = idx < tot ? Lt[idx] : 0ull;
                                        }
    #pragma unroll
                                        for (int c = 0; c < 4; ++c) {
                                            const uint32_t idx = c * WAVE + l;
                                            if (idx < tot) hl[idx] = y[c];
                                        }
                                        done = tot;
                                    }
                                    for (uint32_t idx = done + l; idx < tot; idx += WAVE) hl[idx] = Lt[idx];
                                }
                                lds_sync();
                                // carve the multi-step blocks that arrived since out of the holes.  The tail
                                // is taken into registers 64 entries at a time (lane i holds entry i); the
                                // holes may then grow over its place: k blocks add at most k holes, and
                                // the next 64 start 64 entries further up.
                                uint32_t nh = ns;
                                for (uint32_t tb = 0; tb < nu; tb += WAVE) {
                                    const uint32_t m = min(nu - tb, (uint32_t)WAVE);
                                    const uint64_t te = (uint32_t)l < m ? hl[ns + tb + l] : 0ull;
                                    lds_sync();
                                    for (uint32_t i = 0; i < m; ++i) {
                                        const uint64_t x = read_lane64(te, (int)i);
                                        nh = h_carve(hl, nh, (uint32_t)(x >> 32), (uint32_t)x, wb_from, wb_to);
                                    }
                                }
                                cur_t = t;
                                cur_base = base;
                                cnt = nh;
                            }
                        }
                        pf_t = NONE32;
                        if (mine) {
                            const int jn = __ffsll((unsigned long long)mine) - 1;
                            const uint32_t tn = read_lane(a, jn);
                            const uint32_t totn = read_lane(pns, jn) + read_lane(pnu, jn);
                            if (tn != t && totn + 1 <= LH && !(wmask & (1ull << ((tn / PW) & 63)))) {
                                regs_from_global<0>(pf, L + read_lane(plb, jn), totn, l);
                                pf_t = tn;
                            }
                        }
                        if (cur_t == t) {
                            const uint32_t h = BEST ? h_best_fit(hl, cnt, vs) : h_first_fit(hl, cnt, vs);
                            const uint64_t x = uniform64(hl[h]);
                            o = (uint32_t)(x >> 32);
                            lds_sync();
                            if ((uint32_t)x == vs) {         // used up: the hole leaves the list
                                h_delete(hl, cnt, h);
                                --cnt;
                                wb_from = min(wb_from, h);   // (a lone entry above h moved down: now inside)
                                wb_to = max(wb_to, cnt);
                            } else {
                                if (l == 0) hl[h] = pk(o + vs, (uint32_t)x - vs);
                                lds_sync();
                                if (h >= wb_from && h < wb_to) {
                                    // inside the range already
                                } else if (wb_one == NONE32 || wb_one == h) {
                                    wb_one = h;
                                } else {                     // a second lone entry: widen the range over both
                                    wb_from = min(wb_from, min(h, wb_one));
                                    wb_to = max(wb_to, max(h, wb_one) + 1);
                                    wb_one = NONE32;
                                }
                            }
                        } else {
                            // list too long for the LDS area: same steps directly in global memory
                            uint64_t *Lt = L + A.lstart[t];
                            uint32_t nh = l_ns[t];
                            for (uint32_t nt = l_nu[t]; nt > 0; --nt) {
                                const uint64_t xb = Lt[nh + nt - 1];
                                const uint32_t bo = (uint32_t)(xb >> 32), be = (uint32_t)xb;
                                const uint32_t h = mem_find_hole(Lt, nh, bo);
                                const uint64_t x = Lt[h];
                                const uint32_t st = (uint32_t)(x >> 32), hend = st + (uint32_t)x;
                                wave_fence();
                                if (bo == st) {
                                    if (l == 0) Lt[h] = pk(be, hend - be);
                                } else {
                                    if (l == 0) Lt[h] = pk(st, bo - st);
                                    if (be != hend) {
                                        wave_fence();
                                        insert_at32(Lt, nullptr, nh + nt - 1, h + 1, pk(be, hend - be), 0);
                                        ++nh;
                                    }
                                }
                                wave_fence();
                            }
                            const uint32_t h = BEST ? h_best_fit(Lt, nh, vs) : mem_first_fit(Lt, nh, vs);
                            const uint64_t x = Lt[h];
                            o = (uint32_t)(x >> 32);
                            wave_fence();
                            if (l == 0) { Lt[h] = pk(o + vs, (uint32_t)x - vs); l_ns[t] = nh; l_nu[t] = 0; }
                            wave_fence();
                            if (l == 0) l_top[t] = (uint32_t)(Lt[nh - 1] >> 32);
                            if (one_step && a == t) { pns = nh; pnu = 0; }
                        }
                    }
                    // A run of one step's variables goes back to the registers after the odd one that
                    // needed the full path (unless the one before needed it too).
                    if (!BEST && !placed && same_next && cur_t == t) {
                        if (fail_t != t) {
                            fail_t = t;
                            writeback(one_step ? a : NONE32);
                            cur_t = NONE32;
                        }
                    }
                    fp = max(fp, o + vs);
                    if (l == j) res = o;
                }
                if (my_rank) offs[ridx] = (uint64_t)res << sh;
                p = q;
            }
        }
        // No barrier between windows: a wave reads, for the next window, only the counts of the
        // steps it owns, which no other wave writes outside the barriers of a multi-step
        // variable; its own stores to them are complete after this fence.  The waves drift
        // apart until the next multi-step variable brings them together.
        wave_fence();
    }
    if (l == 0) s_fp[wave] = fp;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t m = s_fp[0];
        for (int w = 1; w < PW; ++w) m = max(m, s_fp[w]);
        A.fps[b] = (uint64_t)m << sh;
        A.ticks[b] = (uint64_t)(wall_clock64() - t_begin);
    }
}

hipError_t launch_plan_prep(uint32_t n, uint32_t T, uint32_t B, const uint64_t *size, const uint32_t *alloc,
                            const uint32_t *free_, uint32_t *cntd, uint32_t *lstart, PlanHeader *hdr, void *vrec,
                            uint64_t seg_pool_entries, uint64_t seg_min_vars, hipStream_t st)
{
    uint32_t blocks = (n + 255) / 256;
    blocks = blocks > 1024 ? 1024 : blocks;
    hipLaunchKernelGGL(k_plan_prep1, dim3(blocks), dim3(256), 0, st, n, T, size, alloc, free_, cntd, hdr);
    hipLaunchKernelGGL(k_plan_prep2, dim3(1), dim3(PREP_THREADS), 0, st, n, T, B, cntd, lstart, hdr, seg_pool_entries,
                       seg_min_vars);
    hipLaunchKernelGGL(k_plan_pack, dim3(blocks), dim3(256), 0, st, n, size, alloc, free_, hdr, (uint4 *)vrec);
    return hipGetLastError();
}

hipError_t launch_place_fast(uint32_t n, uint32_t T, uint32_t B, const uint64_t *size, const uint32_t *alloc,
                             const uint32_t *free_, const uint32_t *perm, const uint32_t *fits, bool any_first,
                             bool any_best, PlanHeader *hdr, const void *vrec,
                             const uint32_t *lstart, uint64_t *m_oe, uint64_t *m_life, uint64_t *m_oe2,
                             uint64_t *m_life2, uint64_t *r_oe, uint64_t *r_life, uint64_t *r_oe2,
                             uint64_t *r_life2, uint64_t *L, uint64_t capL,
                             uint32_t *l_ns, uint32_t *l_nu, uint64_t *offs, uint64_t *fps, uint64_t *ticks,
                             hipStream_t st)
{
    FastArgs A{n, T, size, alloc, free_, (const uint4 *)vrec, perm, fits, hdr, lstart, {m_oe, m_oe2}, {m_life, m_life2}, {r_oe, r_oe2}, {r_life, r_life2},
               L, l_ns,
               l_nu, capL,
               offs, fps, ticks};
    // each instantiation leaves the orderings of the other policy alone
    if (T <= 0xFFFFu) {
        if (any_first) hipLaunchKernelGGL((k_place_fast<uint32_t, false>), dim3(B), dim3(PW * WAVE), 0, st, A);
        if (any_best) hipLaunchKernelGGL((k_place_fast<uint32_t, true>), dim3(B), dim3(PW * WAVE), 0, st, A);
    } else {
        if (any_first) hipLaunchKernelGGL((k_place_fast<uint64_t, false>), dim3(B), dim3(PW * WAVE), 0, st, A);
        if (any_best) hipLaunchKernelGGL((k_place_fast<uint64_t, true>), dim3(B), dim3(PW * WAVE), 0, st, A);
    }
    return hipGetLastError();
}

}  // namespace lap
