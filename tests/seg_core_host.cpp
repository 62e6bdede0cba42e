// Host build of the segment-list primitives (paper_1903_06631_amd/csrc/seg_core.h) for the CPU tests:
// the same functions the HIP kernel calls, compiled with the host compiler and its sanitizers, driven
// one "thread" after the other.  Test code only: the library never loads this.
#include <algorithm>
#include <cstdint>
#include <random>
#include <vector>

#include "../paper_1903_06631_amd/csrc/seg_core.h"

using namespace lap;

extern "C" {

// Randomised check of seg_lower_end / seg_fit / seg_carve against a bitmap of occupied addresses.
// Returns 0, or a positive code naming what disagreed.
int seg_host_unit(uint32_t seed, uint32_t iters, uint32_t max_blocks, uint32_t space)
{
    std::mt19937 rng(seed);
    for (uint32_t it = 0; it < iters; ++it) {
        std::vector<char> occ(space, 0);
        std::vector<uint64_t> L(max_blocks + 2);             // the ranges below the topmost one
        uint32_t len = 1, cap = 1, top = 0;
        auto full = [&]() {                                  // the list as a whole: memory, then (top, SEG_INF)
            std::vector<uint64_t> all(L.begin(), L.begin() + (len - 1));
            all.push_back(seg_pack(top, SEG_INF));
            return all;
        };
        const uint32_t nb = rng() % (max_blocks + 1);
        for (uint32_t k = 0; k < nb; ++k) {
            const uint32_t o = rng() % (space - 1);
            uint32_t e = o + 1 + rng() % std::max<uint32_t>(1, space / 8);
            if (e > space) e = space;
            ++cap;                                           // a block more: an entry more of room
            const uint32_t hint = rng() % 3 == 0 ? SEG_NOHINT : rng() % (len + 2);
            if (!seg_carve(L.data(), len, top, cap, o, e, hint)) return 1;
            for (uint32_t q = o; q < e; ++q) occ[q] = 1;
            std::vector<uint64_t> want;                      // the free runs of the bitmap
            for (uint32_t q = 0; q < space;) {
                if (occ[q]) { ++q; continue; }
                const uint32_t st = q;
                while (q < space && !occ[q]) ++q;
                want.push_back(seg_pack(st, q == space ? SEG_INF : q));
            }
            if (want.empty() || seg_end(want.back()) != SEG_INF) want.push_back(seg_pack(space, SEG_INF));
            if (full() != want) return 2;
        }
        for (int k = 0; k < 16; ++k) {
            const uint32_t o = rng() % space, s = 1 + rng() % std::max<uint32_t>(1, space / 6);
            uint32_t idx = rng() % 3 == 0 ? SEG_NOHINT : rng() % (len + 2), he = 0;
            const std::vector<uint64_t> F = full();
            const uint32_t got = seg_fit(L.data(), len, top, o, s, idx, he);
            uint32_t want = o;
            for (;;) {
                bool ok = true;
                for (uint32_t q = want; q < want + s && ok; ++q) ok = q >= space || !occ[q];
                if (ok) break;
                ++want;
            }
            if (got != want) return 3;
            if (idx >= len || seg_start(F[idx]) > got || seg_end(F[idx]) - got < s || he != seg_end(F[idx])) return 4;
            const uint32_t key = rng() % (space + 4);
            const uint32_t at = seg_lower_end(L.data(), len, top, key, rng() % 2 ? SEG_NOHINT : rng() % (len + 3));
            uint32_t lin = 0;
            while (seg_end(F[lin]) < key) ++lin;
            if (at != lin) return 5;
        }
    }
    return 0;
}

// First-fit placement of one ordering with the segment lists, the kernel's steps in sequence: every
// list of a variable is asked in rounds until none moves the candidate, then the block is taken out of
// its lists.  off_granules[v] receives the offsets.  Returns 0, or a positive code (list id out of
// range, duplicate list, list overflow).
int seg_host_place(uint32_t n, uint32_t T, const uint32_t *size_granules, const uint32_t *alloc, const uint32_t *free_,
                   const uint32_t *perm, uint32_t shift, uint32_t *off_granules, uint64_t *pool_entries,
                   uint64_t *rounds_out)
{
    const SegGeom g{shift, (uint32_t)(((uint64_t)T + (1u << shift) - 1) >> shift), T};
    const uint32_t nl = g.n_lists();
    std::vector<uint32_t> cnt(nl, 0);
    for (uint32_t v = 0; v < n; ++v) {
        const SegSpan sp = seg_span(g, alloc[v], free_[v]);
        std::vector<uint32_t> q, u;
        for (uint32_t i = 0; i < sp.n_query(); ++i) q.push_back(seg_query_list(g, sp, i));
        for (uint32_t i = 0; i < sp.n_update(); ++i) u.push_back(seg_update_list(g, sp, i));
        // seg_update_query: an update list maps to the asked list that it is, and to none otherwise
        for (uint32_t i = 0; i < u.size(); ++i) {
            const uint32_t qi = seg_update_query(sp, i);
            const bool asked = std::find(q.begin(), q.end(), u[i]) != q.end();
            if (qi == SEG_NOHINT ? asked : (qi >= q.size() || q[qi] != u[i])) return 6;
        }
        for (uint32_t id : q) if (id >= nl) return 1;
        for (uint32_t id : u) { if (id >= nl) return 1; ++cnt[id]; }
        std::sort(q.begin(), q.end());
        std::sort(u.begin(), u.end());
        if (std::adjacent_find(q.begin(), q.end()) != q.end() || std::adjacent_find(u.begin(), u.end()) != u.end()) return 2;
    }
    std::vector<uint64_t> lst(nl + 1, 0);
    for (uint32_t j = 0; j < nl; ++j) lst[j + 1] = lst[j] + cnt[j] + 1;
    *pool_entries = lst[nl];
    std::vector<uint64_t> pool(lst[nl]);
    std::vector<uint32_t> lens(nl, 1);
    std::vector<uint32_t> tops(nl, 0);
    uint64_t rounds = 0;
    for (uint32_t r = 0; r < n; ++r) {
        const uint32_t v = perm[r], a = alloc[v], f = free_[v], s = size_granules[v];
        const SegSpan sp = seg_span(g, a, f);
        const uint32_t nq = sp.n_query(), nu = sp.n_update();
        const bool longv = f - a > 1;
        std::vector<uint32_t> memo(nq, 0);
        bool have = false;
        uint32_t o = 0;
        for (;;) {
            uint32_t best = o;
            ++rounds;
            for (uint32_t i = 0; i < nq; ++i) {
                const uint32_t id = seg_query_list(g, sp, i), len = lens[id];
                const uint64_t *L = &pool[lst[id]];
                uint32_t idx = 0, he;
                if (have) {                                  // as in the kernel: last answer, or the evenly-spread estimate
                    idx = memo[i];
                    if (longv && len > 8) {
                        const uint32_t top = tops[id];
                        if (top) {
                            const uint64_t at = (uint64_t)len * ((uint64_t)o + s) / top;
                            idx = std::max(idx, (uint32_t)(at < len - 1 ? at : len - 1));
                        }
                    }
                }
                best = std::max(best, seg_fit(L, len, tops[id], o, s, idx, he));
                memo[i] = idx;
            }
            have = true;
            if (best == o) break;
            o = best;
        }
        off_granules[v] = o;
        for (uint32_t i = 0; i < nu; ++i) {
            const uint32_t id = seg_update_list(g, sp, i);
            if (!seg_carve(&pool[lst[id]], lens[id], tops[id], cnt[id] + 1, o, o + s, longv ? lens[id] - 1 : 0u)) return 3;
        }
    }
    *rounds_out = rounds;
    return 0;
}

}  // extern "C"
