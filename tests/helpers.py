"""Shared test helpers: fixture parsing and small independent brute-force checks.

Nothing here is used by the product path or by the oracle."""
import itertools
import os

import numpy as np

from traces.dnn import Trace

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    """'key v v v' lines -> dict key -> list of rows (each a list of strings)."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, *vals = line.split()
            out.setdefault(key, []).append(vals)
    return out


def mk_trace(size, alloc, free, T=None, gap_lo=None, gap_hi=None, step_ns=None, name="t"):
    size = np.asarray(size, np.uint64)
    alloc = np.asarray(alloc, np.uint32)
    free = np.asarray(free, np.uint32)
    T = int(free.max()) if T is None else T
    gap_lo = alloc.copy() if gap_lo is None else np.asarray(gap_lo, np.uint32)
    gap_hi = (free - 1).astype(np.uint32) if gap_hi is None else np.asarray(gap_hi, np.uint32)
    step_ns = None if step_ns is None else np.asarray(step_ns, np.uint64)
    return Trace(name, T, size, alloc, free, gap_lo, gap_hi, step_ns, {})


def overlaps(tr, i, j):
    return tr.alloc[i] < tr.free[j] and tr.alloc[j] < tr.free[i]


def check_valid(tr, off):
    """Section III-B: a block's address range is never shared with a neighbour."""
    n = tr.n_vars
    a, f = tr.alloc.astype(np.int64), tr.free.astype(np.int64)
    o = off.astype(object)
    e = o + tr.size.astype(object)
    for i in range(n):
        tl = (a[i] < f) & (a < f[i])
        tl[i] = False
        idx = np.nonzero(tl)[0]
        for j in idx:
            if o[i] < e[j] and o[j] < e[i]:
                return False
    return True


def check_valid_fast(tr, off):
    """Same invariant by a sweep over time steps (O(T * live log live))."""
    a, f = tr.alloc.astype(np.int64), tr.free.astype(np.int64)
    o = off.astype(np.uint64)
    e = o + tr.size
    order = np.argsort(a, kind="stable")
    for t in range(tr.n_steps):
        live = np.nonzero((a <= t) & (t < f))[0]
        if len(live) < 2:
            continue
        s = live[np.argsort(o[live], kind="stable")]
        if np.any(e[s][:-1] > o[s][1:]):
            return False
    return True


def grid_first_fit(tr, perm, granule):
    """First-fit by a time x address occupancy grid: lowest address at which the
    whole rectangle (lifetime x size) is free.  Independent of interval lists."""
    n, T = tr.n_vars, tr.n_steps
    sz = (tr.size // np.uint64(granule)).astype(np.int64)
    assert np.all(sz * granule == tr.size.astype(np.int64))
    H = int(sz.sum()) + 1
    occ = np.zeros((T, H), bool)
    off = np.zeros(n, np.uint64)
    for v in perm:
        a, f, s = int(tr.alloc[v]), int(tr.free[v]), int(sz[v])
        col = occ[a:f].any(axis=0)
        o = 0
        while col[o:o + s].any():
            o += 1
        occ[a:f, o:o + s] = True
        off[v] = o * granule
    return off


def optimal_footprint(tr, granule):
    """True offline-DSA optimum by exhaustive search over granule offsets."""
    n = tr.n_vars
    sz = [int(x) // granule for x in tr.size]
    total = sum(sz)
    nb = [[j for j in range(n) if j != i and overlaps(tr, i, j)] for i in range(n)]
    best = [total]
    off = [None] * n

    def rec(i, top):
        if top >= best[0]:
            return
        if i == n:
            best[0] = top
            return
        for o in range(0, best[0] - sz[i]):
            ok = True
            for j in nb[i]:
                if off[j] is not None and o < off[j] + sz[j] and off[j] < o + sz[i]:
                    ok = False
                    break
            if ok:
                off[i] = o
                rec(i + 1, max(top, o + sz[i]))
                off[i] = None

    rec(0, 0)
    return best[0] * granule


def all_perms(n):
    return itertools.permutations(range(n))


def validate_cases():
    """(name, trace, status) triples for trace validation.  The status of every case is written
    out here from the documented rules (the error list of the library's header), not taken from
    either implementation: -6 = invalid content (size 0, alloc >= free, free > n_steps, gap outside
    [alloc, free-1], step_ns 0), -7 = out of range (a size >= 2^53, sum of sizes >= 2^63, sum of
    step_ns >= 2^53, max size * n_steps >= 2^64), 0 = valid.  Invalid content is reported before
    a range problem of the same trace."""
    from traces import random_trace

    def base(n=1000, T=40, step=True):
        return random_trace(3, n, T, with_step_ns=step)

    def edit(field, i, v, **kw):
        t = base(**kw)
        getattr(t, field)[i] = v
        return t

    cases = [("valid", base(), 0), ("valid without step times", base(step=False), 0)]
    cases.append(("size 0", edit("size", 5, 0), -6))
    t = base(); t.alloc[9] = t.free[9]; cases.append(("alloc == free", t, -6))
    t = base(); t.alloc[9] = 39; t.free[9] = 12; cases.append(("alloc > free", t, -6))
    cases.append(("free > n_steps", edit("free", 7, 41), -6))
    t = base(); t.alloc[7] = 39; t.free[7] = 40; t.gap_lo[7] = t.gap_hi[7] = 39
    cases.append(("free == n_steps is allowed", t, 0))
    t = base(); i = int(np.argmax(t.alloc > 0)); t.gap_lo[i] = t.alloc[i] - 1
    cases.append(("gap_lo below alloc", t, -6))
    t = base(); t.gap_hi[4] = t.free[4]; cases.append(("gap_hi above free-1", t, -6))
    t = base(); i = int(np.argmax(t.free - t.alloc > 2)); t.gap_lo[i] = t.alloc[i] + 1; t.gap_hi[i] = t.alloc[i]
    cases.append(("gap_lo above gap_hi", t, -6))
    cases.append(("step_ns 0", edit("step_ns", 3, 0), -6))
    cases.append(("size 2^53", edit("size", 11, 1 << 53), -7))
    cases.append(("size 2^53 - 1 is allowed", edit("size", 11, (1 << 53) - 1), 0))
    cases.append(("one step_ns of 2^53", edit("step_ns", 2, 1 << 53), -7))
    t = base(); t.step_ns[:] = 1; t.step_ns[0] = (1 << 53) - 39
    cases.append(("sum of step_ns == 2^53", t, -7))
    t = base(); t.step_ns[:] = 1; t.step_ns[0] = (1 << 53) - 40
    cases.append(("sum of step_ns == 2^53 - 1 is allowed", t, 0))
    for n, st in ((1024, 0), (1025, -7)):          # 1024 * (2^53 - 1) = 2^63 - 1024; one more reaches 2^63
        t = base(n=n); t.size[:] = (1 << 53) - 1
        cases.append((f"sum of {n} sizes of 2^53 - 1", t, st))
    for T, st in ((4095, 0), (4096, -7)):          # 2^52 * 4096 = 2^64
        t = base(T=T); t.size[17] = 1 << 52
        cases.append((f"size 2^52 over {T} steps", t, st))
    t = base(); t.size[5] = 0; t.size[6] = 1 << 53
    cases.append(("invalid content comes before a range problem", t, -6))
    return cases


# ---- the full-size ordering batches and their stored oracle results -------------------------
# The two largest configurations are planned for every ordering on the GPU; the oracle needs a
# minute or more per ordering there, so its results are computed ahead of time by
# tests/golden/make_fullsize_hashes.py (which calls only the oracle) and stored as one line per
# ordering: footprint and a SHA-256 prefix of the offsets.

def fullsize_batch(cfg):
    """(kinds, seeds) of the batch planned at full size: the benchmark's own batch (4 fixed orders,
    then seeded shuffles with seeds 631 + b) with every 64th ordering (b % 64 == 63) turned into a
    shuffle inside size classes (kind 6) of the same seed, so that every kind is covered."""
    from traces import make_config, make_orderings
    B = make_config(cfg).meta["B"]
    kinds, seeds = make_orderings(B)
    kinds = kinds.copy()
    kinds[63::64] = 6
    return kinds, seeds


def offsets_digest(off):
    """16 hex digits of SHA-256 over the little-endian u64 offsets of one ordering."""
    import hashlib
    return hashlib.sha256(np.ascontiguousarray(off, dtype="<u8").tobytes()).hexdigest()[:16]


def fullsize_golden_path(cfg, best_fit):
    return os.path.join(GOLDEN, f"fullsize_cfg{cfg}_{'best' if best_fit else 'first'}_fit.txt")


def read_fullsize_golden(cfg, best_fit):
    """ordering index -> (kind, seed, footprint, digest) for the orderings the oracle has done."""
    out = {}
    path = fullsize_golden_path(cfg, best_fit)
    if not os.path.exists(path):
        return out
    with open(path) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if len(line) == 5:
                out[int(line[0])] = (int(line[1]), int(line[2]), int(line[3]), line[4])
    return out
