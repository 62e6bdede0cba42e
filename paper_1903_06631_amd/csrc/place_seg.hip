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
// A variable with few lists (two thirds of them: one- and two-step variables) is worked on by one
// wave instead, 64 entries per read, up to three such variables side by side (further down).  The
// topmost range of every list is kept apart, one word per list (seg_core.h): long-lived blocks go
// there nearly always, and then the list's memory is not touched.
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
#define LAP_HD __device__ __forceinline__
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
        uint64_t slots = pool_entries / carry;
        lst[nl] = (uint32_t)carry;
        hdr->seg_need = carry;
        if (slots == 0 || carry >= 0xFFFFFFFFull) {
            hdr->mode2 = 0;
            slots = 1;
        }
        if (slots > B) slots = B;
        // No more slots than make every slot's share of the orderings the same number: the
        // launch ends when the slots with the largest share do, and fewer slots slow one
        // another down less.
        const uint64_t share = (B + slots - 1) / slots;
        hdr->seg_slots = (uint32_t)((B + share - 1) / share);
    }
}

// ---------------------------------------------------------------------------
// one wave on one list: its 64 lanes read 64 neighbouring entries at once
// ---------------------------------------------------------------------------
//
// A variable that lives one or two steps asks two to four lists and is taken out of three to
// five: with one list per thread nearly all of the workgroup idles while one thread follows a
// chain of dependent 8-byte reads (a search, a walk over ranges too small, a shift of the list's
// tail entry by entry).  Such a variable is handled by one wave instead, all lanes on the same
// list: a read fetches 64 neighbouring entries, a ballot finds the first that qualifies, the tail
// is shifted 256 entries per step, and the wave needs no workgroup barrier between one such
// variable and the next.  All arguments of these functions are the same in every lane.
constexpr uint32_t SEG_SHORT_Q = 4;      // most lists such a variable may ask ...
constexpr uint32_t SEG_SHORT_U = 5;      // ... and be taken out of
constexpr uint32_t SEG_GROUP = 3;        // such variables placed side by side, one wave each
constexpr uint32_t SEG_TAIL_SELF = 16;   // a thread moves a list's tail itself up to this many entries

// (a variable that lives through the whole time line asks the list of everything, which the
// waves do not keep up to date among themselves: it is placed by all threads)
__device__ __forceinline__ bool seg_is_short(const SegSpan &sp)
{
    return !sp.whole && sp.n_query() <= SEG_SHORT_Q && sp.n_update() <= SEG_SHORT_U;
}

// entries at .. at + 63 (at < len), one per lane; lanes past the end repeat the last entry (which
// is not in memory: seg_core.h)
__device__ __forceinline__ uint64_t wv_chunk(const uint64_t *L, uint32_t len, uint32_t top, uint32_t at, uint32_t l)
{
    const uint32_t i = at + l;
    return i + 1 < len ? L[i] : seg_pack(top, SEG_INF);
}

// Index of the first entry whose end is >= key.  In: x = wv_chunk(at); floor_known says that no
// entry before `at` qualifies.  Out: (at, x) is a chunk that holds the answer.
__device__ __forceinline__ uint32_t wv_lower_end(const uint64_t *L, uint32_t len, uint32_t top, uint32_t key,
                                                 bool floor_known, uint32_t l, uint32_t &at, uint64_t &x)
{
    uint32_t lo = 0, hi = len - 1;           // the answer lies in [lo, hi]; entry hi qualifies (end = SEG_INF at the top)
    {
        const uint64_t m = ballot(seg_end(x) >= key);
        if (m != 0) {
            const uint32_t f = (uint32_t)__ffsll((unsigned long long)m) - 1;
            if (f > 0 || at == 0 || floor_known) return at + f;
            hi = at;                          // the chunk starts at or above the answer
        } else {
            lo = at + WAVE;                   // (then at + 63 < len - 1: the last entry always qualifies)
        }
    }
    for (int level = 0; level < 8; ++level) { // 64-way: a range of 2^32 is down to four chunks after four levels
        const uint32_t m = hi - lo + 1;
        if (m <= 4u * WAVE) break;
        const uint32_t pos = lo + (uint32_t)(((uint64_t)(l + 1) * m) >> 6) - 1;    // ascending; lane 63 reads entry hi
        const uint64_t y = pos + 1 < len ? L[pos] : seg_pack(top, SEG_INF);
        const uint64_t q = ballot(seg_end(y) >= key) | (1ull << 63);
        const uint32_t f = (uint32_t)__ffsll((unsigned long long)q) - 1;
        hi = read_lane(pos, (int)f);
        if (f > 0) lo = read_lane(pos, (int)f - 1) + 1;
    }
    // what is left, up to four chunks, in one go
    const uint32_t m = hi - lo + 1;
    uint64_t c[4];
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k)
        if (m > WAVE * k) c[k] = wv_chunk(L, len, top, lo + WAVE * k, l);     // lo + 64 k <= hi < len
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k)
        if (m > WAVE * k) {
            const uint64_t q = ballot(seg_end(c[k]) >= key);
            if (q != 0) {
                at = lo + WAVE * k;
                x = c[k];
                return at + (uint32_t)__ffsll((unsigned long long)q) - 1;
            }
        }
    at = lo;                                  // not reached: entry hi qualifies
    x = c[0];
    return lo;
}

// Lowest address >= o at which s granules are free (as seg_fit).  In: x = wv_chunk(at), no entry
// before `at` ends at or above o + s.  Out: idx = the entry that holds the answer, (at, x) a chunk
// that holds that entry.
__device__ __forceinline__ uint32_t wv_fit(const uint64_t *L, uint32_t len, uint32_t top, uint32_t o, uint32_t s,
                                           uint32_t l, uint32_t &at, uint64_t &x, uint32_t &idx)
{
    if (o >= top) {                           // inside the topmost range: nothing to read
        idx = at = len - 1;
        x = seg_pack(top, SEG_INF);
        return o;
    }
    const uint32_t i = wv_lower_end(L, len, top, o + s, true, l, at, x);
    for (;;) {
        const uint32_t st = seg_start(x), en = seg_end(x), e = at + l;
        const uint32_t from = st > o ? st : o;
        // entries from i on end at or above o + s, so en >= from there
        const uint64_t q = ballot(e >= i && e < len && en - from >= s);
        if (q != 0) {
            const uint32_t f = (uint32_t)__ffsll((unsigned long long)q) - 1;
            idx = at + f;
            return read_lane(from, (int)f);
        }
        if (at + WAVE >= len) break;          // not reached: the last entry always fits
        at += WAVE;
        x = wv_chunk(L, len, top, at, l);
    }
    idx = at = len - 1;
    x = seg_pack(top, SEG_INF);
    return top > o ? top : o;
}

// entries j .. len-1 of those in memory move by delta (as seg_carve_shift), 256 per step: all reads
// of a step come before its writes, and no later step reads what an earlier one wrote
__device__ __forceinline__ void wv_shift(uint64_t *L, uint32_t len, uint32_t j, int32_t delta, uint32_t l)
{
    if (delta > 0) {
        for (uint32_t top = len; top > j;) {
            const uint32_t span = top - j;
            uint64_t v[4];
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k)
                if (l + WAVE * k < span) v[k] = L[top - 1 - l - WAVE * k];
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k)
                if (l + WAVE * k < span) L[top - l - WAVE * k] = v[k];
            top = span > 4 * WAVE ? top - 4 * WAVE : j;
        }
    } else if (delta < 0) {
        const uint32_t dn = (uint32_t)-delta;
        for (uint32_t base = j; base < len; base += 4 * WAVE) {
            uint64_t v[4];
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k)
                if (base + l + WAVE * k < len) v[k] = L[base + l + WAVE * k];
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k)
                if (base + l + WAVE * k < len) L[base + l + WAVE * k - dn] = v[k];
        }
    }
}

// The same for lists of several lanes at once: lane i's list starts at pool + base, `rem` of its
// entries (0: none) move by delta, the next of them at `cur` (delta > 0: the entries below cur, from
// the top down; delta < 0: the entries from cur on, upwards).  The wave moves four chunks of 64
// entries per step, of one list or of several, so that tails of a few dozen entries in many lists
// cost no more steps than one long tail.
__device__ __forceinline__ void wv_shift_lanes(uint64_t *pool, uint32_t base, uint32_t rem, uint32_t cur, int32_t delta,
                                               uint32_t l)
{
    for (;;) {
        uint64_t need = ballot(rem > 0);
        if (need == 0) break;
        uint64_t v[4];
        uint32_t s_base[4], s_cur[4], s_n[4];
        int32_t s_delta[4];
        int s_src[4];
        int src = 0;
        uint32_t srem = 0, scur = 0, sbase = 0;
        int32_t sdelta = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            s_n[k] = 0;
            if (srem == 0) {
                if (need == 0) continue;
                src = __ffsll((unsigned long long)need) - 1;
                need &= need - 1;
                srem = read_lane(rem, src);
                scur = read_lane(cur, src);
                sbase = read_lane(base, src);
                sdelta = (int32_t)read_lane((uint32_t)delta, src);
            }
            const uint32_t nk = srem < (uint32_t)WAVE ? srem : (uint32_t)WAVE;
            s_n[k] = nk;
            s_base[k] = sbase;
            s_cur[k] = scur;
            s_delta[k] = sdelta;
            s_src[k] = src;
            srem -= nk;
            scur = sdelta > 0 ? scur - nk : scur + nk;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (l < s_n[k]) v[k] = pool[s_base[k] + (s_delta[k] > 0 ? s_cur[k] - 1 - l : s_cur[k] + l)];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (l < s_n[k]) pool[s_base[k] + (uint32_t)((int32_t)(s_delta[k] > 0 ? s_cur[k] - 1 - l : s_cur[k] + l) + s_delta[k])] = v[k];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (s_n[k] != 0 && (int)l == s_src[k]) {
                rem -= s_n[k];
                cur = s_delta[k] > 0 ? cur - s_n[k] : cur + s_n[k];
            }
    }
}

// Takes [o, e) out of the free ranges (as seg_carve).  In: x = wv_chunk(at); either pos_known and
// `pos` is the first entry that ends above o, inside the chunk, or the chunk is where to start
// looking (floor_known as in wv_lower_end).  len and top receive the new length and topmost range
// (unchanged if the list has no room: not reached, see k_seg_count).
__device__ __forceinline__ void wv_carve(uint64_t *L, uint32_t &len, uint32_t &top, uint32_t cap, uint32_t o, uint32_t e,
                                         bool pos_known, uint32_t pos, bool floor_known, uint32_t l, uint32_t at,
                                         uint64_t x)
{
    if (o >= top) {                                              // inside the topmost range: nothing to read
        if (top < o) {
            if (len + 1 > cap) return;
            if (l == 0) L[len - 1] = seg_pack(top, o);
            len += 1;
        }
        top = e;
        return;
    }
    const uint32_t i = pos_known ? pos : wv_lower_end(L, len, top, o + 1, floor_known, l, at, x);
    const uint32_t d = i - at;                                   // < 64
    const uint64_t y = shfl64(x, (int)((l + d) & (WAVE - 1)));   // lane 0 holds entry i
    const uint32_t avail = min((uint32_t)WAVE - d, len - i);     // entries i .. i + avail - 1 are in lanes 0 .. avail - 1
    const uint64_t q = ballot(l < avail && seg_start(y) < e);    // a prefix: starts ascend
    const uint32_t gone = (uint32_t)__popcll((unsigned long long)q);
    if (gone == 0) return;                                       // nothing free inside [o, e)
    if (gone == avail && i + avail < len) {                      // more ranges than the chunk shows: one lane, entry by entry
        uint32_t nlen = len, ntop = top;
        if (l == 0) seg_carve(L, nlen, ntop, cap, o, e, i);
        len = read_lane(nlen, 0);
        top = read_lane(ntop, 0);
        return;
    }
    const uint32_t hs = read_lane(seg_start(y), 0), last_end = read_lane(seg_end(y), (int)gone - 1);
    const bool left = hs < o, right = last_end > e;
    const uint32_t keep = (left ? 1u : 0u) + (right ? 1u : 0u), j = i + gone;
    const int32_t delta = (int32_t)keep - (int32_t)gone;
    if (delta > 0 && len + 1 > cap) return;
    wv_shift(L, len - 1, j, delta, l);                           // the entries in memory: all but the last
    const uint32_t nlen = (uint32_t)((int32_t)len + delta);
    const uint32_t w = i + (left ? 1u : 0u);                     // where the rest above e goes, if any
    if (l == 0) {
        if (left) L[i] = seg_pack(hs, o);                        // (never the last entry: one that ends above e follows)
        if (right && w + 1 < nlen) L[w] = seg_pack(e, last_end);
    }
    if (right && w + 1 >= nlen) top = e;                         // the last entry: not in memory
    len = nlen;
}

// One variable with few lists, placed by one wave: the fixed point of k_place_seg with every list
// read 64 entries at a time.  Lane i holds what concerns the i-th list the variable asks and
// the i-th list it is taken out of.  The chunks of the lists it will be taken out of but does
// not ask (whose place to look first does not depend on the answer) are fetched together with
// the first round's, the others are those the last round left.  The list of everything (the first
// of the lists it is taken out of) is left to the caller.  Returns the offset in granules.
__device__ __forceinline__ uint32_t place_short(const SegGeom &g, const SegSpan &sp, uint32_t nq, uint32_t nu,
                                                uint32_t s, bool longv, uint32_t l,
                                                const uint32_t *__restrict__ lst, uint64_t *pool, uint32_t *lens,
                                                uint32_t *tops, uint32_t &trial_rounds)
{
    const uint32_t qid = l < nq ? seg_query_list(g, sp, l) : 0u;
    const uint32_t uid = l < nu ? seg_update_list(g, sp, l) : 0u;
    const uint32_t qbase = lst[qid], ubase = lst[uid], ucap = lst[uid + 1] - ubase;
    const uint32_t qlen = lens[qid], qtop = tops[qid];
    const uint32_t ulen0 = lens[uid], utop0 = tops[uid];
    uint32_t ulen = ulen0, utop = utop0;
    // which asked list an update list is, if any
    uint32_t uq = SEG_SHORT_Q;
    for (uint32_t i = 0; i < nq; ++i)
        if (read_lane(qid, (int)i) == uid) uq = i;

    uint64_t xq[SEG_SHORT_Q], xu[SEG_SHORT_U];
    uint32_t qat = 0, qidx = 0;                   // lane i: where list i's chunk starts, the entry that answered
    // where to look first in an update list that is not asked: long-lived blocks end up high
    uint32_t uat = (longv && ulen > (uint32_t)WAVE) ? ulen - WAVE : 0u;
#pragma unroll
    for (uint32_t i = 0; i < SEG_SHORT_Q; ++i)
        if (i < nq) xq[i] = wv_chunk(pool + read_lane(qbase, (int)i), read_lane(qlen, (int)i), read_lane(qtop, (int)i), 0u, l);
#pragma unroll
    for (uint32_t u = 1; u < SEG_SHORT_U; ++u)
        if (u < nu && read_lane(uq, (int)u) == SEG_SHORT_Q)
            xu[u] = wv_chunk(pool + read_lane(ubase, (int)u), read_lane(ulen, (int)u), read_lane(utop, (int)u),
                             read_lane(uat, (int)u), l);

    uint32_t o = 0;
    for (;;) {
        // a list's next answer is at or after its last one, often in the chunk the last round left
        uint32_t best = o;
        for (uint32_t i = 0; i < nq; ++i) {
            uint64_t x = xq[0];
#pragma unroll
            for (uint32_t k = 1; k < SEG_SHORT_Q; ++k)
                if (i == k) x = xq[k];
            uint32_t at = read_lane(qat, (int)i), idx;
            const uint32_t a = wv_fit(pool + read_lane(qbase, (int)i), read_lane(qlen, (int)i), read_lane(qtop, (int)i), o, s,
                                      l, at, x, idx);
#pragma unroll
            for (uint32_t k = 0; k < SEG_SHORT_Q; ++k)
                if (i == k) xq[k] = x;
            if (l == i) {
                qat = at;
                qidx = idx;
            }
            best = max(best, a);
        }
        if (longv) ++trial_rounds;
        if (best == o) break;                     // every list accepts o
        o = best;
    }
    const uint32_t en = o + s;
    for (uint32_t u = 1; u < nu; ++u) {
        // an asked list: the range that holds [o, en) is the one that answered, and the first that ends above o
        const uint32_t qi = read_lane(uq, (int)u);
        const bool asked = qi < SEG_SHORT_Q;
        uint64_t x = asked ? xq[0] : xu[1];
#pragma unroll
        for (uint32_t k = 1; k < SEG_SHORT_Q; ++k)
            if (asked && qi == k) x = xq[k];
#pragma unroll
        for (uint32_t k = 2; k < SEG_SHORT_U; ++k)
            if (!asked && u == k) x = xu[k];
        const uint32_t at = asked ? read_lane(qat, (int)(qi & (SEG_SHORT_Q - 1))) : read_lane(uat, (int)u);
        const uint32_t pos = read_lane(qidx, (int)(qi & (SEG_SHORT_Q - 1)));
        uint32_t nlen = read_lane(ulen, (int)u), ntop = read_lane(utop, (int)u);
        wv_carve(pool + read_lane(ubase, (int)u), nlen, ntop, read_lane(ucap, (int)u), o, en, asked, pos, asked || at == 0,
                 l, at, x);
        if (l == u) {
            ulen = nlen;
            utop = ntop;
        }
    }
    if (l >= 1 && l < nu && ulen != ulen0) lens[uid] = ulen;
    if (l >= 1 && l < nu && utop != utop0) tops[uid] = utop;
    // the wave's later reads of these lists come after these writes (same wave: in order)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    return o;
}

// The blocks of the last group of few-list variables, taken out of the list of everything by one
// wave while the others place the next group (nothing but a variable that lives through the
// whole time line asks that list, and such a variable waits for this).
__device__ __forceinline__ void every_apply(const SegGeom &g, const uint32_t *__restrict__ lst, uint64_t *pool,
                                            uint32_t *lens, uint32_t *tops, const uint4 *pend, uint32_t n_pend,
                                            uint32_t l)
{
    const uint32_t id = 2 * g.K + g.T;
    const uint32_t base = read_lane(lst[id], 0), cap = read_lane(lst[id + 1], 0) - base;
    const uint32_t len0 = read_lane(lens[id], 0), top0 = read_lane(tops[id], 0);
    uint32_t len = len0, top = top0;
    uint64_t *L = pool + base;
    for (uint32_t m = 0; m < n_pend; ++m) {
        const uint4 pe = pend[m];
        const uint32_t o = read_lane(pe.x, 0), en = read_lane(pe.y, 0), at = (read_lane(pe.z, 0) && len > (uint32_t)WAVE) ? len - WAVE : 0u;
        const uint64_t x = wv_chunk(L, len, top, at, l);
        wv_carve(L, len, top, cap, o, en, false, 0u, at == 0, l, at, x);
    }
    if (l == 0 && len != len0) lens[id] = len;
    if (l == 0 && top != top0) tops[id] = top;
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
    uint32_t *lens;              // [slots][2 dir_cap]: lengths, then starts of the topmost ranges
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
    __shared__ uint32_t s_pos[SEG_THREADS];          // where the list a thread asked answered last
    __shared__ uint4 s_pend[2][SEG_GROUP];           // (offset, end, long-lived?, -) of the blocks of the last two groups
    __shared__ uint32_t s_fp[SEG_WAVES], s_rounds[SEG_WAVES], s_vars[SEG_WAVES];

    PlanHeader *hdr = A.hdr;
    if (!hdr->mode2) return;
    const uint32_t slots = TRIAL ? 1u : hdr->seg_slots;
    if (blockIdx.x >= slots) return;
    const SegGeom g{hdr->seg_shift, hdr->seg_K, A.T};
    const uint32_t nl = g.n_lists();
    const uint32_t sh = hdr->shift;
    const uint32_t n = TRIAL ? min(A.n, SEG_TRIAL_RANKS) : A.n;
    const uint32_t tid = threadIdx.x, l = tid & (WAVE - 1), wave = tid / WAVE;
    uint32_t trial_rounds = 0, trial_vars = 0;         // of the variables all threads place together ...
    uint32_t short_rounds = 0, short_vars = 0;         // ... and of those this wave places alone
    uint64_t *pool = A.pool + (size_t)blockIdx.x * hdr->seg_need;
    uint32_t *lens = A.lens + (size_t)blockIdx.x * 2 * A.dir_cap;    // per slot: the lists' lengths ...
    uint32_t *tops = lens + A.dir_cap;                               // ... and where their topmost ranges start
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
            lens[j] = 1;
            tops[j] = 0;
        }
        __syncthreads();
        uint32_t fp = 0, flip = 0;
        uint32_t pend = 0, ppar = 0;       // blocks the list of everything has not seen yet: s_pend[ppar][0 .. pend)
        for (uint32_t r0 = 0; r0 < n; r0 += WAVE) {
            // every wave holds the records of ranks r0 .. r0 + 63, lane i that of rank r0 + i
            uint4 rec = make_uint4(0u, 1u, 1u, 0u);
            if (r0 + l < n) rec = A.vrec[perm[r0 + l]];
            const uint32_t wn = min((uint32_t)WAVE, n - r0);
            for (uint32_t p = 0; p < wn;) {
                const uint32_t a = read_lane(rec.x, (int)p), f = read_lane(rec.y, (int)p), s = read_lane(rec.z, (int)p);
                const SegSpan sp = seg_span(g, a, f);
                const uint32_t nq = sp.n_query(), nu = sp.n_update();
                const bool longv = f - a > 1;         // long-lived blocks end up high, one-step ones low
                if (seg_is_short(sp)) {
                    // Few lists: one wave, all lanes on one list at a time.  Up to three such
                    // variables in a row whose segments differ share no list but that of
                    // everything and do not meet in time: three waves place them side by side,
                    // the fourth takes the last group's blocks out of the list of everything.
                    uint32_t gsz = 1, lo1 = 0, hi1 = 0;
                    const uint32_t lo0 = sp.k0, hi0 = sp.k0 + sp.nseg;
                    for (uint32_t m = 1; m < SEG_GROUP && p + m < wn; ++m) {
                        const SegSpan sm = seg_span(g, read_lane(rec.x, (int)(p + m)), read_lane(rec.y, (int)(p + m)));
                        if (!seg_is_short(sm)) break;
                        const uint32_t lo = sm.k0, hi = sm.k0 + sm.nseg;
                        if (lo < hi0 && lo0 < hi) break;
                        if (m == 2 && lo < hi1 && lo1 < hi) break;
                        lo1 = lo;
                        hi1 = hi;
                        ++gsz;
                    }
                    if (wave < gsz) {
                        const uint32_t q = p + wave;
                        const uint32_t aq = read_lane(rec.x, (int)q), fq = read_lane(rec.y, (int)q), sq = read_lane(rec.z, (int)q);
                        const SegSpan sq_ = seg_span(g, aq, fq);
                        const bool lq = fq - aq > 1;
                        const uint32_t o = place_short(g, sq_, sq_.n_query(), sq_.n_update(), sq, lq, l, lst, pool, lens, tops, short_rounds);
                        if (lq) ++short_vars;
                        fp = max(fp, o + sq);
                        if (l == 0) {
                            offs[r0 + q] = (uint64_t)o << sh;
                            s_pend[ppar ^ 1][wave] = make_uint4(o, o + sq, lq ? 1u : 0u, 0u);
                        }
                    } else if (wave == SEG_WAVES - 1 && pend) {
                        every_apply(g, lst, pool, lens, tops, s_pend[ppar], pend, l);
                    }
                    __syncthreads();
                    ppar ^= 1;
                    pend = gsz;
                    p += gsz;
                    continue;
                }
                // The list of everything has to see the last group's blocks before it is asked (by a
                // variable that lives through the whole time line) or written (by thread 0, below).
                // If the last wave has no list to ask, it does that during the first candidate's
                // search, whose barrier then covers it.
                const bool first_cand = nq >= 8;
                const bool drain_late = pend != 0 && first_cand && nq <= SEG_THREADS - WAVE;
                if (pend && !drain_late) {
                    if (wave == SEG_WAVES - 1) every_apply(g, lst, pool, lens, tops, s_pend[ppar], pend, l);
                    __syncthreads();
                }
                // lowest address that is free in every list of the variable: every thread asks its
                // lists for their lowest fit at or above the candidate, the maximum is the next
                // candidate, until no list moves it
                uint32_t memo[SEG_MEMO] = {0u, 0u};
                bool have = false;
                uint32_t o = 0;
                // what a thread needs of its first list in every round, and of the first list it will
                // take the block out of, is read once, ahead of the searches
                uint32_t q_len = 0, q_base = 0, q_top = 0, u_len = 0, u_base = 0, u_cap = 0, u_top = 0;
                if (tid < nq) {
                    const uint32_t id = seg_query_list(g, sp, tid);
                    q_len = lens[id];
                    q_top = tops[id];
                    q_base = lst[id];
                }
                if (tid < nu) {
                    const uint32_t id = seg_update_list(g, sp, tid);
                    u_len = lens[id];
                    u_top = tops[id];
                    u_base = lst[id];
                    u_cap = lst[id + 1] - u_base;
                }
                // A first candidate from one list, the one with most in it (the segment in the
                // middle of the lifetime), read by one wave 64 entries at a time: asked from there,
                // the others are spared the climb from address 0 over everything that does not
                // concern them (a walk over thousands of ranges too small, when large variables
                // come late).
                uint32_t x_last = 0xFFFFFFFFu, he_last = 0;     // this thread's first list: its last answer and where that range ends
                if (first_cand) {
                    uint32_t first = 0;
                    if (drain_late && wave == SEG_WAVES - 1) every_apply(g, lst, pool, lens, tops, s_pend[ppar], pend, l);
                    if (wave == 0) {
                        const uint32_t id = seg_query_list(g, sp, sp.nf / 2);
                        const uint32_t len = read_lane(lens[id], 0), top = read_lane(tops[id], 0);
                        const uint64_t *L = pool + read_lane(lst[id], 0);
                        uint32_t at = 0, idx;
                        uint64_t x = wv_chunk(L, len, top, 0u, l);
                        first = wv_fit(L, len, top, 0u, s, l, at, x, idx);
                    }
                    if (l == 0) s_max[flip][wave] = first;
                    __syncthreads();
                    o = max(max(s_max[flip][0], s_max[flip][1]), max(s_max[flip][2], s_max[flip][3]));
                    flip ^= 1;
                    have = o > 0;                     // (then start where the candidate would be, as in later rounds)
                    if (drain_late && tid == 0) {     // thread 0's list to write is the list of everything
                        u_len = lens[2 * g.K + g.T];
                        u_top = tops[2 * g.K + g.T];
                    }
                }
                pend = 0;
                for (;;) {
                    uint32_t best = o, j = 0;
                    for (uint32_t i = tid; i < nq; i += SEG_THREADS, ++j) {
                        // the range that answered last holds the new candidate as well: nothing to read
                        if (j == 0 && have && x_last <= o && he_last - o >= s && he_last >= o) continue;
                        // so does the topmost range (long-lived blocks end up high)
                        if (j == 0 && o >= q_top) continue;
                        uint32_t len = q_len, base = q_base, top = q_top;
                        if (j > 0) {
                            const uint32_t id = seg_query_list(g, sp, i);
                            len = lens[id];
                            top = tops[id];
                            base = lst[id];
                        }
                        // Where to look first.  The first round asks from address 0 and is answered
                        // low in the list.  Later rounds: where this list answered before, or, for a
                        // long-lived variable whose candidate has jumped up, further up at the
                        // place the candidate would have if the holes were spread evenly below the
                        // list's top (it saves most of the climb: a third fewer list reads in all).
                        const uint64_t *L = pool + base;
                        uint32_t idx = 0, he;
                        if (have) {
                            if (j < SEG_MEMO) idx = memo[j];
                            if (longv && len > 8) {
                                if (top) {
                                    const uint64_t at = (uint64_t)len * ((uint64_t)o + s) / top;
                                    idx = max(idx, (uint32_t)(at < len - 1 ? at : len - 1));
                                }
                            }
                        }
                        const uint32_t x = seg_fit(L, len, top, o, s, idx, he);
                        if (j < SEG_MEMO) memo[j] = idx;
                        if (j == 0) {
                            x_last = x;
                            he_last = he;
                        }
                        best = max(best, x);
                    }
                    best = seg_wave_max(best);
                    if (l == 0) s_max[flip][wave] = best;
                    s_pos[tid] = memo[0];             // after the last round: the range that holds the block
                    __syncthreads();
                    best = max(max(s_max[flip][0], s_max[flip][1]), max(s_max[flip][2], s_max[flip][3]));
                    flip ^= 1;
                    if (TRIAL && longv) ++trial_rounds;
                    if (best == o) break;             // every list accepts o
                    o = best;
                    if (nq == 1) break;               // one list: its answer is the answer
                    have = true;
                }
                if (TRIAL && longv) ++trial_vars;
                const uint32_t en = o + s;
                fp = max(fp, en);
                if (tid == 0) offs[r0 + p] = (uint64_t)o << sh;      // rank order; un-permuted at the end
                // One list per thread: where the block goes and what changes (seg_carve_plan); a
                // list's tail moves by its thread if it is short and by the whole wave, 256
                // entries per step, if it is long (large blocks that come late split ranges low
                // in lists of thousands: entry by entry that was most of a slow ordering's time).
                for (uint32_t i0 = 0; i0 < nu; i0 += SEG_THREADS) {
                    const uint32_t i = i0 + tid;
                    const bool mine = i < nu;
                    uint32_t base = u_base, cap = u_cap, len = u_len, top = u_top, id = 0;
                    SegCarve c;
                    c.i = c.j = 0;
                    c.delta = 0;
                    if (mine) {
                        id = seg_update_list(g, sp, i);
                        if (i0 > 0) {
                            base = lst[id];
                            cap = lst[id + 1] - base;
                            len = lens[id];
                            top = tops[id];
                        }
                        // Where to look first, if the block is not inside the topmost range (as most
                        // long-lived blocks are: then nothing is read).  A list that was asked: the
                        // range that answered holds the block.  Otherwise long-lived blocks end up
                        // high, one-step ones low (the place the address would have if the ranges
                        // were spread evenly below the top: measured worse).
                        uint32_t hint = longv ? len - 1 : 0u;
                        const uint32_t q = seg_update_query(sp, i);
                        if (q < SEG_THREADS) hint = s_pos[q];
                        c = seg_carve_plan(pool + base, len, top, o, en, hint);
                        // a list never outgrows its room (it sees at most cap - 1 blocks); the check
                        // keeps the stores inside the list whatever happens
                        if (c.delta > 0 && len + 1 > cap) c.j = c.i;
                    }
                    const bool act = c.j != c.i;
                    // of the entries from c.j on, those in memory (all but the last) move
                    const uint32_t mem = len - 1;
                    const uint32_t tail = act && c.delta != 0 && c.j < mem ? mem - c.j : 0u;
                    if (tail > 0 && tail <= SEG_TAIL_SELF) seg_carve_shift(pool + base, len, c.j, c.delta);
                    wv_shift_lanes(pool, base, tail > SEG_TAIL_SELF ? tail : 0u, c.delta > 0 ? mem : c.j, c.delta, l);
                    if (act) {
                        const uint32_t new_len = (uint32_t)((int32_t)len + c.delta), top0 = top;
                        seg_carve_finish(pool + base, new_len, top, c, o, en);
                        if (c.delta != 0) lens[id] = new_len;
                        if (top != top0) tops[id] = top;
                    }
                }
                __syncthreads();
                ++p;
            }
        }
        // what the waves placed on their own: highest end, rounds
        if (l == 0) {
            s_fp[wave] = fp;
            s_rounds[wave] = short_rounds;
            s_vars[wave] = short_vars;
        }
        __syncthreads();
        if (tid == 0) {
            for (int w = 0; w < SEG_WAVES; ++w) {
                fp = max(fp, s_fp[w]);
                trial_rounds += s_rounds[w];
                trial_vars += s_vars[w];
            }
            if (!TRIAL) {
                A.fps[b] = (uint64_t)fp << sh;
                A.ticks[b] = (uint64_t)(wall_clock64() - t_begin);
            }
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
