// Free-range ("hole") lists over time segments: the per-thread primitives and the geometry of
// the segment placement kernel (place_seg.hip).  Plain functions on memory, written so that a
// host compiler accepts them too (LAP_HD is plain `inline` there): the same code can be run under a
// host-side bounds checker.
//
// A list holds the free address ranges with respect to some set of placed blocks, sorted by
// address, one 64-bit word each: start << 32 | end, in granules.  Starts and ends ascend strictly
// (start_i < end_i < start_{i+1}), so a list can be binary searched by end.  The last of a list's
// `len` >= 1 ranges is the one above the highest block, with end = SEG_INF; of that one only
// the start is kept, apart from the others (`top`, in an array of its own with one word per list):
// long-lived blocks go there nearly always, and then neither the question nor the change touches
// the list's memory.  L holds the len - 1 ranges below.
#pragma once
#include <stdint.h>

#ifndef LAP_HD
#define LAP_HD inline
#endif
#ifndef SEG_LD
#define SEG_LD(list, i) (list)[i]       // a host harness may count the reads
#endif

namespace lap {

constexpr uint32_t SEG_INF = 0xFFFFFFFFu;
constexpr uint32_t SEG_NOHINT = 0xFFFFFFFFu;     // seg_lower_end / seg_fit / seg_carve: no idea where to look

LAP_HD uint64_t seg_pack(uint32_t start, uint32_t end) { return ((uint64_t)start << 32) | end; }
LAP_HD uint32_t seg_start(uint64_t x) { return (uint32_t)(x >> 32); }
LAP_HD uint32_t seg_end(uint64_t x) { return (uint32_t)x; }

// entry i < len of a list
LAP_HD uint64_t seg_entry(const uint64_t *L, uint32_t len, uint32_t top, uint32_t i)
{
    return i + 1 < len ? SEG_LD(L, i) : seg_pack(top, SEG_INF);
}

// Index of the first of the `len` >= 1 entries whose end is >= key (key < SEG_INF or the answer is
// the last entry: its end is SEG_INF).  The search runs outward from `hint` in doubling steps and
// finishes with a binary search, so an answer near the hint costs two or three probes.  (Probing
// eight ways at a time shortens the chain of dependent reads but reads more: measured slower,
// the lists' scattered reads are bound by their number, not by their latency.)
LAP_HD uint32_t seg_lower_end(const uint64_t *L, uint32_t len, uint32_t top, uint32_t key, uint32_t hint)
{
    uint32_t lo, hi;                         // the answer lies in [lo, hi]
    if (hint == SEG_NOHINT) {                // nothing known: plain binary search
        lo = 0;
        hi = len - 1;
    } else if (hint >= len) {
        hint = len - 1;
    }
    if (hint == SEG_NOHINT) {
    } else if (seg_end(seg_entry(L, len, top, hint)) >= key) {
        lo = 0;
        hi = hint;
        uint32_t step = 1;
        while (hi > 0) {
            const uint32_t p = hi > step ? hi - step : 0;
            if (seg_end(SEG_LD(L, p)) >= key) {          // p < hint <= len - 1: in memory
                hi = p;
                step <<= 1;
            } else {
                lo = p + 1;
                break;
            }
        }
    } else {
        lo = hint + 1;                       // hint < len - 1 here: the last end is SEG_INF >= key
        hi = len - 1;
        uint32_t step = 1;
        while (lo < hi) {
            const uint32_t p = (hi - lo > step - 1) ? lo + step - 1 : hi;
            if (seg_end(seg_entry(L, len, top, p)) >= key) {
                hi = p;
                break;
            }
            lo = p + 1;
            step <<= 1;
        }
    }
    while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo) >> 1);      // mid < hi <= len - 1: in memory
        if (seg_end(SEG_LD(L, mid)) >= key) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// Lowest address >= o at which s granules are free (o + s < SEG_INF).  idx: in, where to start
// looking; out, the entry that holds the answer.  hole_end receives that entry's end (where the
// free range around the answer stops).
LAP_HD uint32_t seg_fit(const uint64_t *L, uint32_t len, uint32_t top, uint32_t o, uint32_t s, uint32_t &idx,
                        uint32_t &hole_end)
{
    if (o >= top) {                          // inside the topmost range: nothing to read
        idx = len - 1;
        hole_end = SEG_INF;
        return o;
    }
    uint32_t i = seg_lower_end(L, len, top, o + s, idx);
    for (;;) {
        // four entries per step: their reads do not wait for one another (past the end, the last
        // entry again, which always fits: the loop ends inside the list)
        uint64_t x[4];
        for (uint32_t k = 0; k < 4; ++k) x[k] = seg_entry(L, len, top, i + k < len ? i + k : len - 1);
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t st = seg_start(x[k]), en = seg_end(x[k]);
            const uint32_t from = st > o ? st : o;
            if (en - from >= s) {            // en >= o + s and en > st, so en >= from
                idx = i + k < len ? i + k : len - 1;
                hole_end = en;
                return from;
            }
        }
        i += 4;
    }
}

// Taking [o, e) out of the free ranges (the range may be free, partly free or not free at all), in
// three steps so that a caller can do the middle one its own way: what changes (seg_carve_plan),
// the move of the list's tail (seg_carve_shift), the one or two ranges written (seg_carve_finish).
struct SegCarve {
    uint32_t i, j;           // ranges i .. j-1 meet [o, e); j == i: nothing free inside, nothing to do
    uint32_t hs, last_end;   // start of range i, end of range j-1
    int32_t delta;           // what the length changes by: +1 (one range becomes two), 0, or -(ranges that go)
};

LAP_HD SegCarve seg_carve_plan(const uint64_t *L, uint32_t len, uint32_t top, uint32_t o, uint32_t e, uint32_t hint)
{
    SegCarve c;
    if (o >= top) {                                              // inside the topmost range: nothing to read
        c.i = len - 1;
        c.j = len;
        c.hs = top;
        c.last_end = SEG_INF;
        c.delta = top < o ? 1 : 0;
        return c;
    }
    c.i = seg_lower_end(L, len, top, o + 1, hint);               // first range that ends above o
    const uint64_t x = seg_entry(L, len, top, c.i);
    c.hs = seg_start(x);
    c.last_end = seg_end(x);
    c.j = c.i;
    c.delta = 0;
    if (c.hs >= e) return c;                                     // nothing free inside [o, e)
    uint32_t j = c.i + 1;
    for (bool more = j < len; more;) {                           // four entries per step, as in seg_fit
        uint64_t y[4];
        for (uint32_t k = 0; k < 4; ++k) y[k] = seg_entry(L, len, top, j + k < len ? j + k : len - 1);
        for (uint32_t k = 0; k < 4 && more; ++k) {
            if (seg_start(y[k]) >= e) {
                more = false;
            } else {
                c.last_end = seg_end(y[k]);
                ++j;
                more = j < len;
            }
        }
    }
    c.j = j;
    const uint32_t keep = (c.hs < o ? 1u : 0u) + (c.last_end > e ? 1u : 0u);
    c.delta = (int32_t)keep - (int32_t)(j - c.i);
    return c;
}

// The entries j .. len-1 move by delta (+1, or down by -delta <= j); those in memory (all but the
// last) four per step: all reads of a step come before its writes, and no later step reads
// what an earlier one wrote.
LAP_HD void seg_carve_shift(uint64_t *L, uint32_t len, uint32_t j, int32_t delta)
{
    const uint32_t mem = len - 1;                                // entries 0 .. mem-1 are in memory
    if (delta > 0) {
        for (uint32_t q = mem; q > j;) {
            const uint32_t m = q - j < 4 ? q - j : 4;
            uint64_t v[4];
            for (uint32_t k = 0; k < 4; ++k)
                if (k < m) v[k] = SEG_LD(L, q - 1 - k);
            for (uint32_t k = 0; k < 4; ++k)
                if (k < m) L[q - k] = v[k];
            q -= m;
        }
    } else if (delta < 0) {
        const uint32_t d = (uint32_t)-delta;
        for (uint32_t q = j; q < mem;) {
            const uint32_t m = mem - q < 4 ? mem - q : 4;
            uint64_t v[4];
            for (uint32_t k = 0; k < 4; ++k)
                if (k < m) v[k] = SEG_LD(L, q + k);
            for (uint32_t k = 0; k < 4; ++k)
                if (k < m) L[q + k - d] = v[k];
            q += m;
        }
    }
}

// new_len = the length after the change; the last entry's start goes to `top`, the others to memory
LAP_HD void seg_carve_finish(uint64_t *L, uint32_t new_len, uint32_t &top, const SegCarve &c, uint32_t o, uint32_t e)
{
    uint32_t w = c.i;
    if (c.hs < o) {                                              // (never the last entry: one that ends above e follows,
        L[w] = seg_pack(c.hs, o);                                //  written below or already there)
        ++w;
    }
    if (c.last_end > e) {
        if (w + 1 < new_len) L[w] = seg_pack(e, c.last_end); else top = e;
    }
}

// All three.  A list grows by at most one entry per call; `cap` is the room it has (entries in
// memory + 1).  Returns false, and leaves the list alone, if it would outgrow cap.
LAP_HD bool seg_carve(uint64_t *L, uint32_t &len, uint32_t &top, uint32_t cap, uint32_t o, uint32_t e, uint32_t hint)
{
    const SegCarve c = seg_carve_plan(L, len, top, o, e, hint);
    if (c.j == c.i) return true;
    if (c.delta > 0 && len + 1 > cap) return false;
    seg_carve_shift(L, len, c.j, c.delta);
    const uint32_t new_len = (uint32_t)((int32_t)len + c.delta);
    seg_carve_finish(L, new_len, top, c, o, e);
    len = new_len;
    return true;
}

// ---------------------------------------------------------------------------
// geometry: the time line in segments of 2^shift steps
// ---------------------------------------------------------------------------
//
// Three families of lists, numbered in one directory:
//   all[k]    id k            free w.r.t. every block whose lifetime meets segment k
//   cover[k]  id K + k        free w.r.t. the blocks that live through all of segment k
//   step[t]   id 2K + t       free w.r.t. the blocks alive at step t that do not live through
//                             all of t's segment
//   every     id 2K + T       free w.r.t. every block: all a variable that lives through the whole
//                             time line has to ask
// A variable that lives through all of segment k meets, in time, exactly the blocks of all[k];
// one that lives through a part of it meets, at each of its steps t there, the blocks of
// cover[k] and of step[t].  Its lifetime [a, f) therefore decomposes into full segments
// [kf0, kf0 + nf) and at most two partial ones (the first and the last it touches).
struct SegGeom {
    uint32_t shift, K, T;
    LAP_HD uint32_t w() const { return 1u << shift; }
    LAP_HD uint32_t n_lists() const { return 2 * K + T + 1; }
};

struct SegSpan {
    uint32_t k0, nseg;       // segments the lifetime touches: [k0, k0 + nseg)
    uint32_t kf0, nf;        // of which it lives through entirely: [kf0, kf0 + nf)
    uint32_t p0, p0a, p0n;   // first partial segment, its first step there, number of steps (0: none)
    uint32_t p1, p1a, p1n;   // second partial segment
    bool whole;              // lives through every segment
    LAP_HD uint32_t n_query() const { return whole ? 1 : nf + (p0n ? 1 + p0n : 0) + (p1n ? 1 + p1n : 0); }
    LAP_HD uint32_t n_update() const { return 1 + nseg + nf + p0n + p1n; }
};

LAP_HD SegSpan seg_span(const SegGeom &g, uint32_t a, uint32_t f)
{
    SegSpan sp;
    const uint32_t sh = g.shift, w = 1u << sh;
    sp.k0 = a >> sh;
    const uint32_t k1 = (f - 1) >> sh;
    sp.nseg = k1 - sp.k0 + 1;
    sp.kf0 = (a + w - 1) >> sh;                          // first segment that starts at or after a
    const uint32_t kf1 = f == g.T ? g.K : f >> sh;       // first segment that does not end by f
    sp.nf = kf1 > sp.kf0 ? kf1 - sp.kf0 : 0;
    sp.p0 = sp.p1 = 0;
    sp.p0a = sp.p1a = 0;
    sp.p0n = sp.p1n = 0;
    const bool first_partial = sp.nf == 0 || sp.k0 < sp.kf0;
    const bool last_partial = sp.nf == 0 ? k1 != sp.k0 : k1 >= kf1;
    if (first_partial) {
        sp.p0 = sp.k0;
        sp.p0a = a;
        const uint32_t seg_end_step = (sp.k0 + 1) << sh;
        sp.p0n = (f < seg_end_step ? f : seg_end_step) - a;
    }
    if (last_partial) {
        sp.p1 = k1;
        sp.p1a = k1 << sh;
        sp.p1n = f - sp.p1a;
    }
    sp.whole = sp.nf == g.K;
    return sp;
}

// i-th list a variable asks (i < n_query): the all-lists of its full segments (the one list of
// everything if those are all segments), then for each partial segment the cover-list and the
// step-lists of its steps there
LAP_HD uint32_t seg_query_list(const SegGeom &g, const SegSpan &sp, uint32_t i)
{
    if (sp.whole) return 2 * g.K + g.T;
    if (i < sp.nf) return sp.kf0 + i;
    i -= sp.nf;
    if (sp.p0n) {
        if (i == 0) return g.K + sp.p0;
        if (i <= sp.p0n) return 2 * g.K + sp.p0a + (i - 1);
        i -= 1 + sp.p0n;
    }
    if (i == 0) return g.K + sp.p1;
    return 2 * g.K + sp.p1a + (i - 1);
}

// i-th list a placed block is taken out of (i < n_update): the list of everything, all[k] of every segment it touches,
// cover[k] of its full segments, step[t] of its steps in the partial segments
LAP_HD uint32_t seg_update_list(const SegGeom &g, const SegSpan &sp, uint32_t i)
{
    if (i == 0) return 2 * g.K + g.T;
    i -= 1;
    if (i < sp.nseg) return sp.k0 + i;
    i -= sp.nseg;
    if (i < sp.nf) return g.K + sp.kf0 + i;
    i -= sp.nf;
    if (i < sp.p0n) return 2 * g.K + sp.p0a + i;
    i -= sp.p0n;
    return 2 * g.K + sp.p1a + i;
}

// which of the lists a variable asks (index as in seg_query_list) the i-th list it is taken out
// of is; SEG_NOHINT if it does not ask that list
LAP_HD uint32_t seg_update_query(const SegSpan &sp, uint32_t i)
{
    if (sp.whole) return i == 0 ? 0u : SEG_NOHINT;       // asks the list of everything alone
    if (i == 0) return SEG_NOHINT;
    i -= 1;
    if (i < sp.nseg) {                                    // all[k0 + i]: asked if the segment is lived through entirely
        const uint32_t k = sp.k0 + i;
        return k >= sp.kf0 && k - sp.kf0 < sp.nf ? k - sp.kf0 : SEG_NOHINT;
    }
    i -= sp.nseg;
    if (i < sp.nf) return SEG_NOHINT;                     // cover[k] of a full segment
    i -= sp.nf;
    if (i < sp.p0n) return sp.nf + 1 + i;                 // step lists of the first partial segment ...
    i -= sp.p0n;
    return sp.nf + (sp.p0n ? 1 + sp.p0n : 0) + 1 + i;     // ... and of the second
}

}  // namespace lap
