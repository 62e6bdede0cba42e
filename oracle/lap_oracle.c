/*
 * lap_oracle.c -- plain CPU reference for the lifetime-aware pool planner.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * definition that the HIP library is checked against.  It shares no code,
 * header, table or helper with the HIP path and must never be called from the
 * product path (only tests, the smoke check and the benchmark's CPU-baseline
 * leg use it).  Everything is single-threaded, fp64/integer, host pointers.
 *
 * Conventions (all integer unless noted):
 *   variable i : size[i] bytes > 0, live during steps alloc[i] .. free[i]-1
 *                (half-open [alloc, free), 0 <= alloc < free <= T).
 *   two variables overlap in time  <=>  alloc_i < free_j && alloc_j < free_i
 *                (edge E_ij of the weighted interval graph, Section III-B).
 *   accesses gap_lo[i] <= gap_hi[i] bound the idle gap used for swapping
 *                (the two consecutive accesses t_i, t_{i+1} of Section IV-B).
 *
 * Parity status of each function (what pins it, see tests/test_oracle_*.py):
 *   lapo_load_profile : pinned (literal definition, closed-form special
 *                       cases of Section VI-A, hand-worked examples).
 *   lapo_make_perm    : kinds 0..3 pinned against numpy lexsort and the
 *                       hand-worked example; kind 4 (seeded) is pinned only as
 *                       "a permutation, deterministic, published splitmix64
 *                       test vector" -- the paper defines no seeded order:
 *                       PARITY UNPINNED by the paper for kinds 4 and 6 (6 is
 *                       checked against numpy lexsort on (class, key, index)).
 *   lapo_place        : pinned (granule brute force, validity and lower-bound
 *                       invariants of Eq. 2, exhaustive orderings on N<=8
 *                       against an independent exhaustive offset search).
 *   lapo_place_best   : pinned (granule brute force that lists the free runs of
 *                       an occupancy bitmap, hand-worked example where it
 *                       differs from first-fit, validity and Eq. 2 invariants,
 *                       equality with first-fit when at most one hole fits).
 *   lapo_score_swaps  : DOA/AOA/WDOA pinned (hand-worked example, closed
 *                       forms, sign rule of Section IV-B); the peak-cut score
 *                       is this build's reading of "how much the peak drops",
 *                       pinned against a literal re-simulation of the load
 *                       curve with the variable removed.
 *   lapo_detect_iteration : pinned (Z-function of the reversed stream, streams built
 *                       from a known iteration with warm-up prefix and partial tail,
 *                       inner repetitions against min_period).
 *   lapo_schedule_swaps : pinned (hand-worked example; the properties that define an
 *                       as-soon-as-possible and an as-late-as-possible stream schedule
 *                       uniquely; an event-queue re-simulation of the swap-out stream;
 *                       load re-derived with exact fractions).  The stalls of a tight
 *                       limit (the paper's LOAD'') are not modelled.
 *   lapo_simulate_swaps : pinned (hand-worked example with a delayed Malloc and delayed
 *                       swap-ins; a tick-by-tick re-simulation; zero overhead when the
 *                       limit is loose and nothing is late).  The event order at one instant,
 *                       the issue boundary of a swap-in and the deadlock rule are this build's
 *                       readings.
 *   lapo_evaluate_weights : a composition of the pinned pieces above; pinned as such (unit
 *                       weight vectors reproduce the four basic orders, scaling by a
 *                       power of two changes nothing, best = argmin by brute force,
 *                       hand-worked SWDOA values).
 *   lapo_select_swaps : pinned (two hand-worked examples, one where the SWDOA
 *                       order differs from the WDOA order; a dense-matrix
 *                       re-simulation in exact integers; monotone peaks and
 *                       minimal-prefix properties).  Tie rule (lower index
 *                       first) and "away on whole steps only" are this build's
 *                       readings; load_min takes "synchronously" as: away on
 *                       every idle step.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
    LAPO_OK = 0,
    LAPO_E_NULL = -1,
    LAPO_E_SIZE = -2,
    LAPO_E_ORDERING = -4,
    LAPO_E_LINK = -5,
    LAPO_E_TRACE = -6,
    LAPO_E_RANGE = -7,
    LAPO_E_NOMEM = -100
};

/* ------------------------------------------------------------------------ */
/* (a) memory load profile and its peak                                      */
/* ------------------------------------------------------------------------ */

/* Section II, Definition 2: the load at a time point is the sum of the sizes
 * of the variables resident at that point.  Definition 4 / Eq. 1: the peak
 * load is its maximum over the iteration (the weighted clique number), the
 * peak time is where it occurs; when the maximum is reached more than once
 * the earliest step is reported.  Written as the definition: every variable
 * adds its size to every step of its lifetime. */
int lapo_load_profile(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc,
                      const uint32_t *free_, uint64_t *load, uint64_t *peak, uint32_t *t_peak)
{
    if (!size || !alloc || !free_ || !load || !peak || !t_peak) return LAPO_E_NULL;
    if (n == 0 || T == 0) return LAPO_E_SIZE;
    for (uint32_t t = 0; t < T; ++t) load[t] = 0;
    for (uint32_t i = 0; i < n; ++i)
        for (uint32_t t = alloc[i]; t < free_[i]; ++t) load[t] += size[i];
    uint64_t best = load[0];
    uint32_t at = 0;
    for (uint32_t t = 1; t < T; ++t)
        if (load[t] > best) { best = load[t]; at = t; }
    *peak = best;
    *t_peak = at;
    return LAPO_OK;
}

/* Number of edges of the interval graph G (Section III-B): pairs of variables
 * whose lifetimes overlap.  Used only as a work measure. */
uint64_t lapo_count_edges(uint32_t n, const uint32_t *alloc, const uint32_t *free_)
{
    uint64_t e = 0;
    for (uint32_t i = 0; i < n; ++i)
        for (uint32_t j = i + 1; j < n; ++j)
            if (alloc[i] < free_[j] && alloc[j] < free_[i]) ++e;
    return e;
}

/* ------------------------------------------------------------------------ */
/* trace validation                                                          */
/* ------------------------------------------------------------------------ */

int lapo_validate_trace(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc,
                        const uint32_t *free_, const uint32_t *gap_lo, const uint32_t *gap_hi,
                        const uint64_t *step_ns)
{
    if (!size || !alloc || !free_) return LAPO_E_NULL;
    if ((gap_lo == NULL) != (gap_hi == NULL)) return LAPO_E_NULL;
    if (n == 0 || T == 0) return LAPO_E_SIZE;
    const uint64_t two53 = (uint64_t)1 << 53, two63 = (uint64_t)1 << 63;
    uint64_t sum = 0, maxsize = 0;
    for (uint32_t i = 0; i < n; ++i) {
        if (size[i] == 0 || alloc[i] >= free_[i] || free_[i] > T) return LAPO_E_TRACE;
        if (gap_lo && (gap_lo[i] < alloc[i] || gap_hi[i] > free_[i] - 1 || gap_lo[i] > gap_hi[i]))
            return LAPO_E_TRACE;
    }
    if (step_ns)
        for (uint32_t t = 0; t < T; ++t)
            if (step_ns[t] == 0) return LAPO_E_TRACE;
    for (uint32_t i = 0; i < n; ++i) {
        if (size[i] >= two53) return LAPO_E_RANGE;
        sum += size[i];
        if (sum >= two63) return LAPO_E_RANGE;
        if (size[i] > maxsize) maxsize = size[i];
    }
    /* max size * T must fit 64 bits (area key, load prefix sums) */
    if (maxsize > UINT64_MAX / T) return LAPO_E_RANGE;
    uint64_t total_ns = 0;
    for (uint32_t t = 0; t < T; ++t) {
        uint64_t ns = step_ns ? step_ns[t] : 1000000u;
        if (ns >= two53) return LAPO_E_RANGE;
        total_ns += ns;
        if (total_ns >= two53) return LAPO_E_RANGE;
    }
    return LAPO_OK;
}

/* ------------------------------------------------------------------------ */
/* (b) orderings                                                             */
/* ------------------------------------------------------------------------ */

/* Key of the seeded shuffle: the splitmix64 output function (Steele, Lea,
 * Flood 2014; Vigna's public-domain formulation) applied to the counter
 * seed + (i+1)*golden-gamma.  Counter based: no state is carried between
 * variables. */
static uint64_t mix64(uint64_t seed, uint32_t i)
{
    uint64_t z = seed + ((uint64_t)i + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t lapo_mix64(uint64_t seed, uint32_t i) { return mix64(seed, i); }

typedef struct { uint64_t key; uint32_t idx; } keyed;

static int cmp_key_asc(const void *a, const void *b)
{
    const keyed *x = (const keyed *)a, *y = (const keyed *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx);
}

static int cmp_key_desc(const void *a, const void *b)
{
    const keyed *x = (const keyed *)a, *y = (const keyed *)b;
    if (x->key != y->key) return x->key > y->key ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx);
}

typedef struct { uint32_t cls; uint64_t key; uint32_t idx; } classed;

static int cmp_class_desc_key_asc(const void *a, const void *b)
{
    const classed *x = (const classed *)a, *y = (const classed *)b;
    if (x->cls != y->cls) return x->cls > y->cls ? -1 : 1;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx);
}

/* Section III-C sorts the variables by size, largest first (kind 0).  The
 * other kinds are the extra heuristic orders evaluated in parallel:
 *   1 lifetime descending, 2 size x lifetime descending, 3 alloc step
 *   ascending (arrival order, what an online pool would see), 4 seeded
 *   shuffle (ascending mix64 key), 5 caller-supplied permutation, 6 seeded
 *   shuffle inside size classes: class = floor(log2 size), larger classes
 *   first, ascending mix64 key within a class (a randomised relative of the
 *   paper's order that keeps big blocks early).
 * Equal keys keep ascending variable index (a stable sort). */
int lapo_make_perm(uint32_t n, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                   uint32_t kind, uint64_t seed, const uint32_t *explicit_perm, uint32_t *perm)
{
    if (!size || !alloc || !free_ || !perm) return LAPO_E_NULL;
    if (n == 0) return LAPO_E_SIZE;
    if (kind > 6) return LAPO_E_ORDERING;
    if (kind == 6) {
        classed *c = (classed *)malloc((size_t)n * sizeof(classed));
        if (!c) return LAPO_E_NOMEM;
        for (uint32_t i = 0; i < n; ++i) {
            uint32_t lg = 0;
            while ((size[i] >> lg) > 1) ++lg;          /* floor(log2 size), size > 0 */
            c[i].cls = lg; c[i].key = mix64(seed, i); c[i].idx = i;
        }
        qsort(c, n, sizeof(classed), cmp_class_desc_key_asc);
        for (uint32_t r = 0; r < n; ++r) perm[r] = c[r].idx;
        free(c);
        return LAPO_OK;
    }
    if (kind == 5) {
        if (!explicit_perm) return LAPO_E_NULL;
        unsigned char *seen = (unsigned char *)calloc(n, 1);
        if (!seen) return LAPO_E_NOMEM;
        for (uint32_t r = 0; r < n; ++r) {
            uint32_t v = explicit_perm[r];
            if (v >= n || seen[v]) { free(seen); return LAPO_E_ORDERING; }
            seen[v] = 1;
            perm[r] = v;
        }
        free(seen);
        return LAPO_OK;
    }
    keyed *k = (keyed *)malloc((size_t)n * sizeof(keyed));
    if (!k) return LAPO_E_NOMEM;
    for (uint32_t i = 0; i < n; ++i) {
        uint64_t life = (uint64_t)(free_[i] - alloc[i]);
        k[i].idx = i;
        switch (kind) {
        case 0: k[i].key = size[i]; break;
        case 1: k[i].key = life; break;
        case 2: k[i].key = size[i] * life; break;
        case 3: k[i].key = alloc[i]; break;
        default: k[i].key = mix64(seed, i); break;
        }
    }
    qsort(k, n, sizeof(keyed), kind <= 2 ? cmp_key_desc : cmp_key_asc);
    for (uint32_t r = 0; r < n; ++r) perm[r] = k[r].idx;
    free(k);
    return LAPO_OK;
}

/* ------------------------------------------------------------------------ */
/* (b) first-fit placement                                                   */
/* ------------------------------------------------------------------------ */

typedef struct { uint64_t off, end; } span;

static int cmp_span(const void *a, const void *b)
{
    const span *x = (const span *)a, *y = (const span *)b;
    if (x->off != y->off) return x->off < y->off ? -1 : 1;
    return x->end < y->end ? -1 : (x->end > y->end);
}

/* Section III-C: take the variables in the given order; each one gets an
 * address range that none of its already-placed, time-overlapping neighbours
 * uses.  First-fit: the first (lowest) hole between the neighbours' blocks
 * that is large enough -- a hole of exactly the variable's size fits -- and
 * when no hole fits the block goes above the topmost neighbour (the pool is
 * extended).  Blocks of variables that do not overlap in time are invisible
 * to each other.  footprint = highest end address over all variables. */
int lapo_place(uint32_t n, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
               const uint32_t *perm, uint64_t *off, uint64_t *footprint)
{
    if (!size || !alloc || !free_ || !perm || !off || !footprint) return LAPO_E_NULL;
    if (n == 0) return LAPO_E_SIZE;
    /* placed variables in placement order */
    uint32_t *pa = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    uint32_t *pf = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    span *ps = (span *)malloc((size_t)n * sizeof(span));
    span *nb = (span *)malloc((size_t)n * sizeof(span));
    if (!pa || !pf || !ps || !nb) { free(pa); free(pf); free(ps); free(nb); return LAPO_E_NOMEM; }
    uint64_t fp = 0;
    for (uint32_t r = 0; r < n; ++r) {
        const uint32_t v = perm[r];
        const uint32_t a = alloc[v], f = free_[v];
        const uint64_t s = size[v];
        /* neighbours: placed earlier and overlapping in lifetime */
        uint32_t m = 0;
        for (uint32_t j = 0; j < r; ++j)
            if (pa[j] < f && a < pf[j]) nb[m++] = ps[j];
        qsort(nb, m, sizeof(span), cmp_span);
        /* walk the neighbours' blocks upward from address 0 */
        uint64_t o = 0;
        for (uint32_t j = 0; j < m; ++j) {
            if (nb[j].off >= o && nb[j].off - o >= s) break;   /* hole [o, nb.off) fits */
            if (nb[j].end > o) o = nb[j].end;
        }
        off[v] = o;
        pa[r] = a; pf[r] = f; ps[r].off = o; ps[r].end = o + s;
        if (o + s > fp) fp = o + s;
    }
    *footprint = fp;
    free(pa); free(pf); free(ps); free(nb);
    return LAPO_OK;
}

/* Section III-C, the other policy: best-fit.  Same walk over the neighbours' blocks, but
 * every hole is looked at -- the free range below the lowest block and the free ranges between
 * blocks -- and the SMALLEST one that is large enough is taken (the lowest of several equally
 * small ones); the block goes to that hole's start.  When no hole fits the block goes above
 * the topmost neighbour, as with first-fit. */
int lapo_place_best(uint32_t n, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                    const uint32_t *perm, uint64_t *off, uint64_t *footprint)
{
    if (!size || !alloc || !free_ || !perm || !off || !footprint) return LAPO_E_NULL;
    if (n == 0) return LAPO_E_SIZE;
    uint32_t *pa = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    uint32_t *pf = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    span *ps = (span *)malloc((size_t)n * sizeof(span));
    span *nb = (span *)malloc((size_t)n * sizeof(span));
    if (!pa || !pf || !ps || !nb) { free(pa); free(pf); free(ps); free(nb); return LAPO_E_NOMEM; }
    uint64_t fp = 0;
    for (uint32_t r = 0; r < n; ++r) {
        const uint32_t v = perm[r];
        const uint32_t a = alloc[v], f = free_[v];
        const uint64_t s = size[v];
        uint32_t m = 0;
        for (uint32_t j = 0; j < r; ++j)
            if (pa[j] < f && a < pf[j]) nb[m++] = ps[j];
        qsort(nb, m, sizeof(span), cmp_span);
        uint64_t top = 0, best_gap = UINT64_MAX, best_at = 0;
        for (uint32_t j = 0; j < m; ++j) {
            if (nb[j].off > top) {                               /* hole [top, nb.off) */
                const uint64_t gap = nb[j].off - top;
                if (gap >= s && gap < best_gap) { best_gap = gap; best_at = top; }
            }
            if (nb[j].end > top) top = nb[j].end;
        }
        const uint64_t o = best_gap != UINT64_MAX ? best_at : top;
        off[v] = o;
        pa[r] = a; pf[r] = f; ps[r].off = o; ps[r].end = o + s;
        if (o + s > fp) fp = o + s;
    }
    *footprint = fp;
    free(pa); free(pf); free(ps); free(nb);
    return LAPO_OK;
}

/* Evaluate B orderings and keep the smallest footprint (lowest ordering index
 * on ties).  kinds/seeds are host arrays; for kind 5 the seed field is the
 * host address of a u32[n] permutation.  footprints / all_off may be NULL. */
int lapo_plan_pool(uint32_t n, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                   uint32_t B, const uint32_t *kinds, const uint64_t *seeds,
                   uint64_t *best_off, uint64_t *best_fp, uint32_t *best_idx,
                   uint64_t *footprints, uint64_t *all_off)
{
    if (!kinds || !seeds || !best_off || !best_fp || !best_idx) return LAPO_E_NULL;
    if (n == 0 || B == 0) return LAPO_E_SIZE;
    uint32_t *perm = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    uint64_t *off = (uint64_t *)malloc((size_t)n * sizeof(uint64_t));
    if (!perm || !off) { free(perm); free(off); return LAPO_E_NOMEM; }
    int rc = LAPO_OK;
    uint64_t bfp = 0;
    uint32_t bidx = 0;
    for (uint32_t b = 0; b < B; ++b) {
        const uint32_t *ex = kinds[b] == 5 ? (const uint32_t *)(uintptr_t)seeds[b] : NULL;
        rc = lapo_make_perm(n, size, alloc, free_, kinds[b], seeds[b], ex, perm);
        if (rc) break;
        uint64_t fp;
        rc = lapo_place(n, size, alloc, free_, perm, off, &fp);
        if (rc) break;
        if (footprints) footprints[b] = fp;
        if (all_off) memcpy(all_off + (size_t)b * n, off, (size_t)n * sizeof(uint64_t));
        if (b == 0 || fp < bfp) {
            bfp = fp; bidx = b;
            memcpy(best_off, off, (size_t)n * sizeof(uint64_t));
        }
    }
    if (!rc) { *best_fp = bfp; *best_idx = bidx; }
    free(perm); free(off);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* (c) swap-candidate scores                                                 */
/* ------------------------------------------------------------------------ */

/* Section IV.  Per variable, with t_lo = gap_lo, t_hi = gap_hi its two
 * consecutive accesses (defaults: alloc and free-1) and step t occupying wall
 * clock [C[t], C[t+1]) where C is the prefix sum of step_ns:
 *   candidate (IV-A): size >= min_bytes, lifetime spans the peak time
 *                     (alloc <= t_peak < free), and the gap is not empty.
 *   transfer time   : delta = ceil(size*1000 / bpus) ns each way, with
 *                     bpus = llround(link_GBps*1000) bytes per microsecond.
 *   DOA (IV-B i)    : time between the accesses minus swap-out and swap-in:
 *                     C[t_hi] - C[t_lo+1] - 2*delta (may be negative).
 *   AOA (IV-B ii)   : DOA*size when DOA >= 0, DOA/size otherwise (binary64,
 *                     one operation).
 *   WDOA (IV-B iii) : area under the ORIGINAL load curve between the two
 *                     accesses: sum of load over steps t_lo+1 .. t_hi-1.
 *   peak cut        : the variable is absent for the whole steps that lie
 *                     inside [C[t_lo+1]+delta, C[t_hi]-delta); cut = peak -
 *                     peak of the load curve with size removed on those steps
 *                     (0 when DOA < 0 or no whole step fits).
 * Variables with gap_hi == gap_lo get 0 in every output. */
int lapo_score_swaps(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc,
                     const uint32_t *free_, const uint32_t *gap_lo, const uint32_t *gap_hi,
                     const uint64_t *step_ns, double link_GBps, uint64_t min_bytes,
                     uint8_t *cand, int64_t *doa, double *aoa, uint64_t *wdoa, uint64_t *cut)
{
    if (!size || !alloc || !free_ || !cand || !doa || !aoa || !wdoa || !cut) return LAPO_E_NULL;
    if ((gap_lo == NULL) != (gap_hi == NULL)) return LAPO_E_NULL;
    if (n == 0 || T == 0) return LAPO_E_SIZE;
    if (!(link_GBps > 0.0) || !isfinite(link_GBps) || link_GBps * 1000.0 >= 9.0e18) return LAPO_E_LINK;
    const long long bpus_ll = llround(link_GBps * 1000.0);
    if (bpus_ll <= 0) return LAPO_E_LINK;
    const uint64_t bpus = (uint64_t)bpus_ll;

    uint64_t *load = (uint64_t *)malloc((size_t)T * sizeof(uint64_t));
    uint64_t *C = (uint64_t *)malloc(((size_t)T + 1) * sizeof(uint64_t));
    if (!load || !C) { free(load); free(C); return LAPO_E_NOMEM; }
    uint64_t peak; uint32_t t_peak;
    int rc = lapo_load_profile(n, T, size, alloc, free_, load, &peak, &t_peak);
    if (rc) { free(load); free(C); return rc; }
    C[0] = 0;
    for (uint32_t t = 0; t < T; ++t) C[t + 1] = C[t] + (step_ns ? step_ns[t] : 1000000u);

    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t tl = gap_lo ? gap_lo[i] : alloc[i];
        const uint32_t th = gap_hi ? gap_hi[i] : free_[i] - 1;
        cand[i] = 0; doa[i] = 0; aoa[i] = 0.0; wdoa[i] = 0; cut[i] = 0;
        if (th <= tl) continue;
        const uint64_t s = size[i];
        cand[i] = (s >= min_bytes && alloc[i] <= t_peak && t_peak < free_[i]) ? 1 : 0;
        const uint64_t delta = (s * 1000u + bpus - 1) / bpus;
        const int64_t d = (int64_t)(C[th] - C[tl + 1]) - 2 * (int64_t)delta;
        doa[i] = d;
        aoa[i] = d >= 0 ? (double)d * (double)s : (double)d / (double)s;
        uint64_t area = 0;
        for (uint32_t t = tl + 1; t < th; ++t) area += load[t];
        wdoa[i] = area;
        if (d < 0) continue;
        /* whole steps inside [out_done, in_start) */
        const uint64_t out_done = C[tl + 1] + delta, in_start = C[th] - delta;
        uint32_t lo = 0, hi = 0;
        while (C[lo] < out_done) ++lo;                 /* first step starting at/after out_done */
        for (uint32_t t = 0; t <= T; ++t) if (C[t] <= in_start) hi = t;   /* last boundary <= in_start */
        if (hi <= lo) continue;
        uint64_t np = 0;
        for (uint32_t t = 0; t < T; ++t) {
            uint64_t l = (t >= lo && t < hi) ? load[t] - s : load[t];
            if (l > np) np = l;
        }
        cut[i] = peak - np;
    }
    free(load); free(C);
    return LAPO_OK;
}

/* ------------------------------------------------------------------------ */
/* selection of swap variables down to a memory-load limit (Section IV-D),  */
/* with the submodular WDOA order of Section IV-B (iv) and load_min (VI-B)   */
/* ------------------------------------------------------------------------ */

enum { LAPO_PS_DOA = 0, LAPO_PS_AOA = 1, LAPO_PS_WDOA = 2, LAPO_PS_SWDOA = 3, LAPO_PS_PEAK_CUT = 4 };

/* Whole steps [lo, hi) during which variable i is away when swapped: those inside
 * [C[t_lo+1]+delta, C[t_hi]-delta); lo = hi = 0 when DOA < 0 or no whole step fits. */
static void absent_window(uint32_t T, const uint64_t *C, uint32_t tl, uint32_t th, uint64_t delta,
                          uint32_t *lo_out, uint32_t *hi_out)
{
    *lo_out = 0; *hi_out = 0;
    if (th <= tl) return;
    const int64_t d = (int64_t)(C[th] - C[tl + 1]) - 2 * (int64_t)delta;
    if (d < 0) return;
    const uint64_t out_done = C[tl + 1] + delta, in_start = C[th] - delta;
    uint32_t lo = 0, hi = 0;
    while (C[lo] < out_done) ++lo;
    for (uint32_t t = 0; t <= T; ++t) if (C[t] <= in_start) hi = t;
    if (hi > lo) { *lo_out = lo; *hi_out = hi; }
}

/* Section IV-D: the candidates (Section IV-A) are ordered by a priority score, highest first
 * (equal scores: lower variable index first), and added to the swap list one by one; every
 * addition removes the variable's size from the load on its absent steps; the walk stops as
 * soon as the peak load is no larger than the limit.
 *   score_kind 0..2, 4: order by DOA / AOA / WDOA / peak cut as lapo_score_swaps gives them.
 *   score_kind 3 (SWDOA, Section IV-B iv): repeatedly take the candidate with the largest
 *     WDOA measured on the CURRENT (already reduced) load curve, then reduce the curve.
 * Outputs: order[k] = k-th variable of the priority order (k < *n_cand), rank[i] = its
 * position or 0xFFFFFFFF for non-candidates, peaks[k] = peak load after the first k
 * additions (k = 0 .. *n_cand), and for every limit the number of variables selected and
 * the peak reached (all candidates when the limit is out of reach).
 * load_min (Section VI-B1): the peak of the curve with every candidate away on ALL its idle
 * steps gap_lo+1 .. gap_hi-1 (swapped out and in synchronously, transfers not hidden). */
enum { LAPO_PS_CUSTOM = 5 };

/* score_kind 5 walks by a caller-supplied binary64 score per variable (`custom`); pick_wdoa, if
 * given, receives for every candidate the WDOA it had on the current curve when it was picked
 * (for the SWDOA walk that is the value the pick was decided on). */
static int select_core(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc,
                       const uint32_t *free_, const uint32_t *gap_lo, const uint32_t *gap_hi,
                       const uint64_t *step_ns, double link_GBps, uint64_t min_bytes, uint32_t score_kind,
                       const double *custom, const uint64_t *limits, uint32_t n_limits,
                       uint32_t *order, uint32_t *rank, uint32_t *n_cand, uint64_t *peaks,
                       uint32_t *n_selected, uint64_t *peak_after, uint64_t *load_min, uint64_t *pick_wdoa)
{
    if (!order || !rank || !n_cand || !peaks || !load_min) return LAPO_E_NULL;
    if (n_limits && (!limits || !n_selected || !peak_after)) return LAPO_E_NULL;
    if (score_kind > 5 || (score_kind == 5 && !custom)) return LAPO_E_ORDERING;
    uint8_t *cand = (uint8_t *)malloc(n);
    int64_t *doa = (int64_t *)malloc((size_t)n * 8);
    double *aoa = (double *)malloc((size_t)n * 8);
    uint64_t *wdoa = (uint64_t *)malloc((size_t)n * 8);
    uint64_t *cut = (uint64_t *)malloc((size_t)n * 8);
    uint64_t *load = (uint64_t *)malloc((size_t)T * 8);
    uint64_t *C = (uint64_t *)malloc(((size_t)T + 1) * 8);
    uint32_t *wlo = (uint32_t *)malloc((size_t)n * 4), *whi = (uint32_t *)malloc((size_t)n * 4);
    uint8_t *taken = (uint8_t *)calloc(n, 1);
    int rc = LAPO_E_NOMEM;
    if (!cand || !doa || !aoa || !wdoa || !cut || !load || !C || !wlo || !whi || !taken) goto done;
    rc = lapo_score_swaps(n, T, size, alloc, free_, gap_lo, gap_hi, step_ns, link_GBps, min_bytes, cand, doa, aoa,
                          wdoa, cut);
    if (rc) goto done;
    {
        uint64_t peak; uint32_t t_peak;
        rc = lapo_load_profile(n, T, size, alloc, free_, load, &peak, &t_peak);
        if (rc) goto done;
    }
    const uint64_t bpus = (uint64_t)llround(link_GBps * 1000.0);
    C[0] = 0;
    for (uint32_t t = 0; t < T; ++t) C[t + 1] = C[t] + (step_ns ? step_ns[t] : 1000000u);
    uint32_t nc = 0;
    for (uint32_t i = 0; i < n; ++i) {
        rank[i] = 0xFFFFFFFFu;
        const uint32_t tl = gap_lo ? gap_lo[i] : alloc[i], th = gap_hi ? gap_hi[i] : free_[i] - 1;
        absent_window(T, C, tl, th, (size[i] * 1000u + bpus - 1) / bpus, &wlo[i], &whi[i]);
        if (cand[i]) ++nc;
    }
    *n_cand = nc;
    /* load_min: every candidate away on all its idle steps */
    {
        uint64_t m = 0;
        for (uint32_t t = 0; t < T; ++t) {
            uint64_t l = load[t];
            for (uint32_t i = 0; i < n; ++i) {
                if (!cand[i]) continue;
                const uint32_t tl = gap_lo ? gap_lo[i] : alloc[i], th = gap_hi ? gap_hi[i] : free_[i] - 1;
                if (t > tl && t < th) l -= size[i];
            }
            if (l > m) m = l;
        }
        *load_min = m;
    }
    /* the walk */
    {
        uint64_t pk = 0;
        for (uint32_t t = 0; t < T; ++t) if (load[t] > pk) pk = load[t];
        peaks[0] = pk;
    }
    for (uint32_t k = 0; k < nc; ++k) {
        /* next variable of the priority order: best score among the candidates not taken yet */
        uint32_t best = 0xFFFFFFFFu;
        for (uint32_t i = 0; i < n; ++i) {
            if (!cand[i] || taken[i]) continue;
            if (score_kind == LAPO_PS_SWDOA) {           /* WDOA on the current curve */
                const uint32_t tl = gap_lo ? gap_lo[i] : alloc[i], th = gap_hi ? gap_hi[i] : free_[i] - 1;
                uint64_t area = 0;
                for (uint32_t t = tl + 1; t < th; ++t) area += load[t];
                wdoa[i] = area;
            }
            int better;
            if (best == 0xFFFFFFFFu) better = 1;
            else switch (score_kind) {
                case LAPO_PS_DOA: better = doa[i] > doa[best]; break;
                case LAPO_PS_AOA: better = aoa[i] > aoa[best]; break;
                case LAPO_PS_PEAK_CUT: better = cut[i] > cut[best]; break;
                case LAPO_PS_CUSTOM: better = custom[i] > custom[best]; break;
                default: better = wdoa[i] > wdoa[best]; break;
            }
            if (better) best = i;
        }
        if (pick_wdoa) {
            const uint32_t tl = gap_lo ? gap_lo[best] : alloc[best], th = gap_hi ? gap_hi[best] : free_[best] - 1;
            uint64_t area = 0;
            for (uint32_t t = tl + 1; t < th; ++t) area += load[t];
            pick_wdoa[best] = area;
        }
        taken[best] = 1;
        order[k] = best;
        rank[best] = k;
        for (uint32_t t = wlo[best]; t < whi[best]; ++t) load[t] -= size[best];
        uint64_t pk = 0;
        for (uint32_t t = 0; t < T; ++t) if (load[t] > pk) pk = load[t];
        peaks[k + 1] = pk;
    }
    for (uint32_t q = 0; q < n_limits; ++q) {
        uint32_t k = 0;
        while (k < nc && peaks[k] > limits[q]) ++k;
        n_selected[q] = k;
        peak_after[q] = peaks[k];
    }
    rc = LAPO_OK;
done:
    free(cand); free(doa); free(aoa); free(wdoa); free(cut); free(load); free(C); free(wlo); free(whi); free(taken);
    return rc;
}

int lapo_select_swaps(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc,
                      const uint32_t *free_, const uint32_t *gap_lo, const uint32_t *gap_hi,
                      const uint64_t *step_ns, double link_GBps, uint64_t min_bytes, uint32_t score_kind,
                      const uint64_t *limits, uint32_t n_limits,
                      uint32_t *order, uint32_t *rank, uint32_t *n_cand, uint64_t *peaks,
                      uint32_t *n_selected, uint64_t *peak_after, uint64_t *load_min)
{
    if (score_kind > 4) return LAPO_E_ORDERING;
    return select_core(n, T, size, alloc, free_, gap_lo, gap_hi, step_ns, link_GBps, min_bytes, score_kind, NULL,
                       limits, n_limits, order, rank, n_cand, peaks, n_selected, peak_after, load_min, NULL);
}

/* ------------------------------------------------------------------------ */
/* iteration detection on a recorded request stream (Section V)              */
/* ------------------------------------------------------------------------ */

/* The requests of the first iterations are recorded in a list; an iteration has been seen as
 * soon as the list ends with two consecutive equal subsequences, and that subsequence is one
 * iteration's operations.  tokens[i] stands for request i (operation kind and size, whatever the
 * caller folds into 64 bits; addresses are not part of it, they differ between iterations).
 * *period = the smallest p >= min_period (min_period >= 1) with
 *     tokens[M-2p+i] == tokens[M-p+i]  for all 0 <= i < p,
 * or 0 when there is none (in particular when 2*min_period > M).  The iteration is then
 * tokens[M-p .. M). */
int lapo_detect_iteration(const uint64_t *tokens, uint32_t M, uint32_t min_period, uint32_t *period)
{
    if (!tokens || !period) return LAPO_E_NULL;
    if (M == 0 || min_period == 0) return LAPO_E_SIZE;
    *period = 0;
    for (uint32_t p = min_period; 2 * (uint64_t)p <= M; ++p) {
        uint32_t i = 0;
        while (i < p && tokens[M - 2 * p + i] == tokens[M - p + i]) ++i;
        if (i == p) { *period = p; break; }
    }
    return LAPO_OK;
}

/* ------------------------------------------------------------------------ */
/* swap schedule (Section IV-E), without the stalls a tight limit may force  */
/* ------------------------------------------------------------------------ */

typedef struct { uint32_t step, var, pos; } sched_key;

static int cmp_sched(const void *a, const void *b)
{
    const sched_key *x = (const sched_key *)a, *y = (const sched_key *)b;
    if (x->step != y->step) return x->step < y->step ? -1 : 1;
    return x->var < y->var ? -1 : (x->var > y->var);
}

/* Section IV-E: the selected variables are swapped out when not in use and prefetched before
 * their next access.  Swap-outs run one after the other on one stream in ascending order of
 * their access (ties: variable index); each starts as soon as its access has completed (the end
 * of step gap_lo) and the previous swap-out has finished.  Swap-ins run one after the other on a
 * second stream in the order of the next accesses; each starts as late as it can so that it has
 * finished when its access begins (the start of step gap_hi) and the swap-in after it can still
 * start on time.  All times in ns from the start of the iteration (swap-in times may be negative
 * when the stream is overbooked).  A transfer of a variable takes ceil(size*1000/bytes_per_us).
 *   swap_list[k]            the selected variables (distinct)
 *   out_start/out_end/in_start/in_end [k]   per list position
 *   load_sched[T]           load with every selected variable away on the whole steps that lie
 *                           between the end of its swap-out and the start of its swap-in
 *   peak_sched              its maximum
 *   late_ns                 sum over the list of max(0, out_end - in_start): transfer time the
 *                           plan cannot hide (the swap-in would have to start before the
 *                           swap-out is done) */
int lapo_schedule_swaps(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc,
                        const uint32_t *free_, const uint32_t *gap_lo, const uint32_t *gap_hi,
                        const uint64_t *step_ns, double link_GBps, const uint32_t *swap_list, uint32_t k,
                        int64_t *out_start, int64_t *out_end, int64_t *in_start, int64_t *in_end,
                        uint64_t *load_sched, uint64_t *peak_sched, uint64_t *late_ns)
{
    if (!size || !alloc || !free_ || !load_sched || !peak_sched || !late_ns) return LAPO_E_NULL;
    if (k && (!swap_list || !out_start || !out_end || !in_start || !in_end)) return LAPO_E_NULL;
    if (n == 0 || T == 0) return LAPO_E_SIZE;
    if (!(link_GBps > 0.0) || !isfinite(link_GBps)) return LAPO_E_LINK;
    const uint64_t bpus = (uint64_t)llround(link_GBps * 1000.0);
    if (bpus == 0) return LAPO_E_LINK;
    uint64_t *C = (uint64_t *)malloc(((size_t)T + 1) * 8);
    sched_key *q = (sched_key *)malloc(((size_t)k + 1) * sizeof(sched_key));
    if (!C || !q) { free(C); free(q); return LAPO_E_NOMEM; }
    C[0] = 0;
    for (uint32_t t = 0; t < T; ++t) C[t + 1] = C[t] + (step_ns ? step_ns[t] : 1000000u);
    for (uint32_t t = 0; t < T; ++t) load_sched[t] = 0;
    for (uint32_t i = 0; i < n; ++i)
        for (uint32_t t = alloc[i]; t < free_[i]; ++t) load_sched[t] += size[i];
    /* swap-outs: as soon as possible, in access order */
    for (uint32_t j = 0; j < k; ++j) {
        const uint32_t v = swap_list[j];
        q[j].step = gap_lo ? gap_lo[v] : alloc[v]; q[j].var = v; q[j].pos = j;
    }
    qsort(q, k, sizeof(sched_key), cmp_sched);
    int64_t stream_free = 0;
    for (uint32_t j = 0; j < k; ++j) {
        const uint32_t v = q[j].var;
        const int64_t delta = (int64_t)((size[v] * 1000u + bpus - 1) / bpus);
        const int64_t ready = (int64_t)C[q[j].step + 1];
        const int64_t st = ready > stream_free ? ready : stream_free;
        out_start[q[j].pos] = st;
        out_end[q[j].pos] = st + delta;
        stream_free = st + delta;
    }
    /* swap-ins: as late as possible, in next-access order, planned from the last one back */
    for (uint32_t j = 0; j < k; ++j) {
        const uint32_t v = swap_list[j];
        q[j].step = gap_hi ? gap_hi[v] : free_[v] - 1; q[j].var = v; q[j].pos = j;
    }
    qsort(q, k, sizeof(sched_key), cmp_sched);
    int64_t next_start = INT64_MAX;
    for (uint32_t j = k; j-- > 0;) {
        const uint32_t v = q[j].var;
        const int64_t delta = (int64_t)((size[v] * 1000u + bpus - 1) / bpus);
        const int64_t due = (int64_t)C[q[j].step];
        const int64_t en = due < next_start ? due : next_start;
        in_end[q[j].pos] = en;
        in_start[q[j].pos] = en - delta;
        next_start = en - delta;
    }
    /* the load under this plan, and what it cannot hide */
    uint64_t late = 0;
    for (uint32_t j = 0; j < k; ++j) {
        const uint32_t v = swap_list[j];
        if (out_end[j] > in_start[j]) { late += (uint64_t)(out_end[j] - in_start[j]); continue; }
        for (uint32_t t = 0; t < T; ++t)
            if ((int64_t)C[t] >= out_end[j] && (int64_t)C[t + 1] <= in_start[j]) load_sched[t] -= size[v];
    }
    uint64_t pk = 0;
    for (uint32_t t = 0; t < T; ++t) if (load_sched[t] > pk) pk = load_sched[t];
    *peak_sched = pk;
    *late_ns = late;
    free(C); free(q);
    return LAPO_OK;
}

/* ------------------------------------------------------------------------ */
/* the schedule under a memory-load limit (Section IV-E, second half)        */
/* ------------------------------------------------------------------------ */

/* Section IV-E: with a stringent limit the load would exceed it because variables cannot be
 * swapped out quickly enough; then the next Malloc is delayed until enough has been swapped out,
 * and a swap-in can start only after something has been freed.  That is where overhead that
 * cannot be hidden comes from.  This is a discrete-event simulation of one iteration:
 *
 *   compute   runs the steps in order.  Step t may start when the step before it has ended, every
 *             listed variable with gap_hi == t is back (its swap-in has ended), and -- if the step
 *             allocates anything -- the resident bytes plus the sizes allocated at step t stay
 *             within the limit (it is the Malloc that is delayed).
 *   resident  grows at a step's start by the sizes allocated there and at a swap-in's start;
 *             shrinks at a step's end by the sizes freed there and at a swap-out's end.
 *   swap-outs one stream, ascending (gap_lo, index); a job is issued when step gap_lo ends and
 *             starts when it is issued and the stream is free.
 *   swap-ins  a second stream, ascending (gap_hi, index); a job is issued when compute reaches the
 *             step boundary at or before its planned start (lapo_schedule_swaps), not before
 *             boundary gap_lo+1; it starts when it is issued, the stream is free, its own swap-out
 *             has ended and resident + size <= limit.
 *   at one instant: ends first (step, swap-out, swap-in), then starts in the order swap-out,
 *             step, swap-in.
 *   deadlock  if nothing runs and the next step cannot start, the limit is overridden once
 *             (counted in *forced): for the step's allocations if only they are in the way,
 *             else for the swap-in at the head of its stream.
 * Listed variables with gap_hi == gap_lo are never swapped.
 * Outputs: *total_ns end of the last step, *overhead_ns = total - sum of step_ns,
 * *peak_resident the largest resident value, *forced as above. */
int lapo_simulate_swaps(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc,
                        const uint32_t *free_, const uint32_t *gap_lo, const uint32_t *gap_hi,
                        const uint64_t *step_ns, double link_GBps, const uint32_t *swap_list, uint32_t k,
                        uint64_t limit, uint64_t *total_ns, uint64_t *overhead_ns, uint64_t *peak_resident,
                        uint32_t *forced)
{
    if (!size || !alloc || !free_ || !total_ns || !overhead_ns || !peak_resident || !forced) return LAPO_E_NULL;
    if (k && !swap_list) return LAPO_E_NULL;
    if (n == 0 || T == 0) return LAPO_E_SIZE;
    if (!(link_GBps > 0.0) || !isfinite(link_GBps)) return LAPO_E_LINK;
    const uint64_t bpus = (uint64_t)llround(link_GBps * 1000.0);
    if (bpus == 0) return LAPO_E_LINK;
    int rc = LAPO_E_NOMEM;
    int64_t *os = (int64_t *)malloc(((size_t)k + 1) * 8), *oe = (int64_t *)malloc(((size_t)k + 1) * 8);
    int64_t *is = (int64_t *)malloc(((size_t)k + 1) * 8), *ie = (int64_t *)malloc(((size_t)k + 1) * 8);
    uint64_t *ld = (uint64_t *)malloc((size_t)T * 8), *C = (uint64_t *)malloc(((size_t)T + 1) * 8);
    uint64_t *need = (uint64_t *)calloc(T, 8), *rel = (uint64_t *)calloc(T, 8);
    sched_key *qo = (sched_key *)malloc(((size_t)k + 1) * sizeof(sched_key));
    sched_key *qi = (sched_key *)malloc(((size_t)k + 1) * sizeof(sched_key));
    uint32_t *kb = (uint32_t *)calloc((size_t)k + 1, 4);          /* issue boundary of each swap-in, by list position */
    uint8_t *out_done = (uint8_t *)calloc((size_t)k + 1, 1), *back = (uint8_t *)calloc((size_t)k + 1, 1);
    uint32_t *waiting = (uint32_t *)calloc(T, 4);                 /* listed variables still away that step t needs */
    if (!os || !oe || !is || !ie || !ld || !C || !need || !rel || !qo || !qi || !kb || !out_done || !back || !waiting)
        goto done;
    C[0] = 0;
    for (uint32_t t = 0; t < T; ++t) C[t + 1] = C[t] + (step_ns ? step_ns[t] : 1000000u);
    for (uint32_t i = 0; i < n; ++i) { need[alloc[i]] += size[i]; rel[free_[i] - 1] += size[i]; }
    uint32_t m = 0;                                               /* jobs: listed variables with an idle gap */
    for (uint32_t j = 0; j < k; ++j) {
        const uint32_t v = swap_list[j];
        const uint32_t tl = gap_lo ? gap_lo[v] : alloc[v], th = gap_hi ? gap_hi[v] : free_[v] - 1;
        if (th <= tl) continue;
        qo[m].step = tl; qo[m].var = v; qo[m].pos = m;
        qi[m].step = th; qi[m].var = v; qi[m].pos = m;
        kb[m] = v;                                                /* for now: the m-th job's variable */
        ++m;
    }
    {
        /* the plan for exactly these jobs gives the swap-in starts */
        uint64_t pk, late;
        rc = lapo_schedule_swaps(n, T, size, alloc, free_, gap_lo, gap_hi, step_ns, link_GBps, kb, m, os, oe,
                                 is, ie, ld, &pk, &late);
        if (rc) goto done;
        rc = LAPO_E_NOMEM;
    }
    for (uint32_t j = 0; j < m; ++j) {
        const uint32_t v = kb[j];
        const uint32_t tl = gap_lo ? gap_lo[v] : alloc[v], th = gap_hi ? gap_hi[v] : free_[v] - 1;
        uint32_t b = 0;
        for (uint32_t t = 0; t <= th; ++t) if ((int64_t)C[t] <= is[j]) b = t;
        if (b < tl + 1) b = tl + 1;
        kb[j] = b;
        waiting[th] += 1;
    }
    qsort(qo, m, sizeof(sched_key), cmp_sched);
    qsort(qi, m, sizeof(sched_key), cmp_sched);
    {
        uint64_t now = 0, R = 0, peak = 0;
        uint32_t t = 0, nforced = 0;                 /* next step to start */
        int step_running = 0, out_running = 0, in_running = 0;
        uint64_t step_end = 0, out_end_t = 0, in_end_t = 0;
        uint32_t o_issued = 0, o_next = 0;           /* swap-outs issued / started so far (in queue order) */
        uint32_t i_issued = 0, i_next = 0;
        uint32_t boundary = 0;                       /* step boundaries compute has reached */
        while (i_issued < m && kb[qi[i_issued].pos] <= boundary) ++i_issued;
        for (;;) {
            /* ends at this instant */
            if (step_running && step_end == now) {
                step_running = 0;
                R -= rel[t];
                while (o_issued < m && qo[o_issued].step == t) ++o_issued;
                ++t;
                boundary = t;
                while (i_issued < m && kb[qi[i_issued].pos] <= boundary) ++i_issued;
            }
            if (out_running && out_end_t == now) {
                out_running = 0;
                R -= size[qo[o_next].var];
                out_done[qo[o_next].pos] = 1;
                ++o_next;
            }
            if (in_running && in_end_t == now) {
                in_running = 0;
                back[qi[i_next].pos] = 1;
                waiting[qi[i_next].step] -= 1;
                ++i_next;
            }
            if (t == T && !step_running) break;
            /* starts: swap-out, step, swap-in */
            if (!out_running && o_next < o_issued) {
                const uint32_t v = qo[o_next].var;
                out_running = 1;
                out_end_t = now + (size[v] * 1000u + bpus - 1) / bpus;
            }
            int step_mem_blocked = 0;
            if (!step_running && t < T && waiting[t] == 0) {
                if (need[t] == 0 || R + need[t] <= limit) {
                    step_running = 1; R += need[t]; step_end = now + (C[t + 1] - C[t]);
                    if (R > peak) peak = R;
                } else step_mem_blocked = 1;
            }
            int in_mem_blocked = 0;
            if (!in_running && i_next < i_issued && out_done[qi[i_next].pos]) {
                const uint32_t v = qi[i_next].var;
                if (R + size[v] <= limit) {
                    in_running = 1; R += size[v]; in_end_t = now + (size[v] * 1000u + bpus - 1) / bpus;
                    if (R > peak) peak = R;
                } else in_mem_blocked = 1;
            }
            if (!step_running && !out_running && !in_running) {
                /* nothing will ever change by itself: override the limit once */
                ++nforced;
                if (step_mem_blocked) {
                    step_running = 1; R += need[t]; step_end = now + (C[t + 1] - C[t]);
                } else if (in_mem_blocked) {
                    const uint32_t v = qi[i_next].var;
                    in_running = 1; R += size[v]; in_end_t = now + (size[v] * 1000u + bpus - 1) / bpus;
                } else { rc = LAPO_E_TRACE; goto done; }            /* cannot happen on a valid trace */
                if (R > peak) peak = R;
            }
            /* next instant */
            uint64_t nx = UINT64_MAX;
            if (step_running && step_end < nx) nx = step_end;
            if (out_running && out_end_t < nx) nx = out_end_t;
            if (in_running && in_end_t < nx) nx = in_end_t;
            now = nx;
        }
        *total_ns = now;
        *overhead_ns = now - C[T];
        *peak_resident = peak;
        *forced = nforced;
    }
    rc = LAPO_OK;
done:
    free(os); free(oe); free(is); free(ie); free(ld); free(C); free(need); free(rel); free(qo); free(qi); free(kb);
    free(out_done); free(back); free(waiting);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* aggregated priority score (Section IV-C) evaluated for many weight vectors */
/* ------------------------------------------------------------------------ */

/* Section IV-C (Eq. 3): the aggregated score is a linear combination of the four basic scores,
 *     BO = a*AOA + b*DOA + c*WDOA + d*SWDOA,
 * and its weights are tuned against the communication overhead the resulting schedule causes.
 * Here the weights apply to the RAW scores (standardising a score is an affine map, so for the
 * order it induces it only rescales that score's weight; the caller folds 1/sigma in), SWDOA_i
 * is the WDOA variable i had on the reduced curve when the SWDOA walk picked it, the overhead is
 * the one lapo_simulate_swaps reports, and the optimiser is whoever calls this with weight
 * vectors: for each of W vectors (a, b, c, d) the candidates are walked by BO (one binary64
 * expression, evaluated ((a*AOA + b*DOA) + c*WDOA) + d*SWDOA without contraction; ties: lower
 * index) down to `limit`, and that selection is replayed under the limit.
 * Outputs per vector: order (row of n, first *n_cand valid), n_selected, peak_after,
 * overhead_ns, forced; *best = the vector with the least overhead (lowest index on ties);
 * swdoa[n] = the SWDOA values used (0 for non-candidates). */
int lapo_evaluate_weights(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc,
                          const uint32_t *free_, const uint32_t *gap_lo, const uint32_t *gap_hi,
                          const uint64_t *step_ns, double link_GBps, uint64_t min_bytes,
                          const double *weights, uint32_t W, uint64_t limit,
                          uint32_t *order, uint32_t *n_cand, uint32_t *n_selected, uint64_t *peak_after,
                          uint64_t *overhead_ns, uint32_t *forced, uint32_t *best, uint64_t *swdoa)
{
    if (!weights || !order || !n_cand || !n_selected || !peak_after || !overhead_ns || !forced || !best || !swdoa)
        return LAPO_E_NULL;
    if (W == 0) return LAPO_E_SIZE;
    uint8_t *cand = (uint8_t *)malloc(n);
    int64_t *doa = (int64_t *)malloc((size_t)n * 8);
    double *aoa = (double *)malloc((size_t)n * 8), *bo = (double *)malloc((size_t)n * 8);
    uint64_t *wdoa = (uint64_t *)malloc((size_t)n * 8), *cut = (uint64_t *)malloc((size_t)n * 8);
    uint32_t *rank = (uint32_t *)malloc((size_t)n * 4), *ord = (uint32_t *)malloc((size_t)n * 4);
    uint64_t *peaks = (uint64_t *)malloc(((size_t)n + 1) * 8);
    int rc = LAPO_E_NOMEM;
    if (!cand || !doa || !aoa || !bo || !wdoa || !cut || !rank || !ord || !peaks) goto done;
    rc = lapo_score_swaps(n, T, size, alloc, free_, gap_lo, gap_hi, step_ns, link_GBps, min_bytes, cand, doa, aoa,
                          wdoa, cut);
    if (rc) goto done;
    {
        uint64_t lm;
        for (uint32_t i = 0; i < n; ++i) swdoa[i] = 0;
        rc = select_core(n, T, size, alloc, free_, gap_lo, gap_hi, step_ns, link_GBps, min_bytes, LAPO_PS_SWDOA,
                         NULL, NULL, 0, ord, rank, n_cand, peaks, NULL, NULL, &lm, swdoa);
        if (rc) goto done;
    }
    for (uint32_t w = 0; w < W; ++w) {
        const double a = weights[4 * w], b = weights[4 * w + 1], c = weights[4 * w + 2], d = weights[4 * w + 3];
        for (uint32_t i = 0; i < n; ++i) {
            const double t1 = a * aoa[i], t2 = b * (double)doa[i];
            const double t3 = t1 + t2, t4 = c * (double)wdoa[i];
            const double t5 = t3 + t4, t6 = d * (double)swdoa[i];
            bo[i] = t5 + t6;
        }
        uint32_t nc;
        uint64_t lm;
        rc = select_core(n, T, size, alloc, free_, gap_lo, gap_hi, step_ns, link_GBps, min_bytes, LAPO_PS_CUSTOM, bo,
                         &limit, 1, order + (size_t)w * n, rank, &nc, peaks, &n_selected[w], &peak_after[w], &lm,
                         NULL);
        if (rc) goto done;
        uint64_t total, pk;
        rc = lapo_simulate_swaps(n, T, size, alloc, free_, gap_lo, gap_hi, step_ns, link_GBps,
                                 order + (size_t)w * n, n_selected[w], limit, &total, &overhead_ns[w], &pk,
                                 &forced[w]);
        if (rc) goto done;
    }
    *best = 0;
    for (uint32_t w = 1; w < W; ++w)
        if (overhead_ns[w] < overhead_ns[*best]) *best = w;
    rc = LAPO_OK;
done:
    free(cand); free(doa); free(aoa); free(bo); free(wdoa); free(cut); free(rank); free(ord); free(peaks);
    return rc;
}
