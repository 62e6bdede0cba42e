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
