"""Pins for the oracle's best-fit placement (Section III-C, the policy the paper runs by default)."""
import numpy as np
import pytest

from helpers import check_valid, mk_trace, read_golden, all_perms
from traces import make_config, random_trace

G = 512


def _golden():
    g = read_golden("e4_best_fit.txt")
    tr = mk_trace([int(x) * G for x in g["size"][0]], g["alloc"][0], g["free"][0], T=3)
    return g, tr


def test_e4_golden(oracle_mod):
    g, tr = _golden()
    perm = np.arange(tr.n_vars, dtype=np.uint32)
    off, fp = oracle_mod.place(tr, perm)
    assert (off // G).tolist() == [int(x) for x in g["first_fit"][0]] and fp == int(g["first_fit_footprint"][0][0]) * G
    off, fp = oracle_mod.place(tr, perm, best_fit=True)
    assert (off // G).tolist() == [int(x) for x in g["best_fit"][0]] and fp == int(g["best_fit_footprint"][0][0]) * G
    _, peak, _ = oracle_mod.load_profile(tr)
    assert peak == int(g["peak"][0][0]) * G


def grid_best_fit(tr, perm, granule):
    """Best-fit on a time x address occupancy bitmap: list the maximal free runs below the
    highest occupied granule of the variable's lifetime, take the smallest that fits."""
    n, T = tr.n_vars, tr.n_steps
    sz = (tr.size // np.uint64(granule)).astype(np.int64)
    H = int(sz.sum()) + 1
    occ = np.zeros((T, H), bool)
    off = np.zeros(n, np.uint64)
    for v in perm:
        a, f, s = int(tr.alloc[v]), int(tr.free[v]), int(sz[v])
        col = occ[a:f].any(axis=0)
        used = np.nonzero(col)[0]
        top = int(used[-1]) + 1 if len(used) else 0
        runs, x = [], 0
        while x < top:
            if col[x]:
                x += 1
                continue
            y = x
            while y < top and not col[y]:
                y += 1
            runs.append((y - x, x))
            x = y
        fits = [r for r in runs if r[0] >= s]
        o = min(fits)[1] if fits else top
        occ[a:f, o:o + s] = True
        off[v] = o * granule
    return off


@pytest.mark.parametrize("seed", range(12))
def test_against_bitmap_brute_force(oracle_mod, seed):
    tr = random_trace(4000 + seed, n=30 + 5 * seed, T=6 + seed, size_choices=(512, 1024, 1536, 2560, 4096),
                      max_life=5, one_step_frac=0.4)
    rng = np.random.default_rng(seed)
    for kind in (0, 1, 2, 3):
        perm = oracle_mod.make_perm(tr, kind)
        off, fp = oracle_mod.place(tr, perm, best_fit=True)
        assert np.array_equal(off, grid_best_fit(tr, perm, G))
        assert fp == int((off + tr.size).max())
    perm = rng.permutation(tr.n_vars).astype(np.uint32)
    off, _ = oracle_mod.place(tr, perm, best_fit=True)
    assert np.array_equal(off, grid_best_fit(tr, perm, G))


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_valid_and_bounded(oracle_mod, cfg):
    tr = make_config(cfg)
    _, peak, _ = oracle_mod.load_profile(tr)
    differs = False
    for kind in (0, 1, 2, 3, 4):
        perm = oracle_mod.make_perm(tr, kind, 631)
        off, fp = oracle_mod.place(tr, perm, best_fit=True)
        if cfg < 3:
            assert check_valid(tr, off)
        assert fp >= peak and fp == int((off + tr.size).max())            # Eq. 2
        off_ff, _ = oracle_mod.place(tr, perm)
        differs |= not np.array_equal(off, off_ff)
    assert differs or cfg == 1          # the two policies are not the same function


def test_special_cases(oracle_mod):
    # everything overlaps: no holes ever, both policies stack in order
    tr = mk_trace([G * k for k in (3, 1, 4, 1, 5)], [0] * 5, [2] * 5, T=2)
    perm = np.array([2, 0, 4, 1, 3], np.uint32)
    a, _ = oracle_mod.place(tr, perm)
    b, _ = oracle_mod.place(tr, perm, best_fit=True)
    assert np.array_equal(a, b) and b.tolist() == [4 * G, 12 * G, 0, 13 * G, 7 * G]
    # disjoint lifetimes: everything at 0
    tr = mk_trace([G, 2 * G, 3 * G], [0, 1, 2], [1, 2, 3], T=3)
    assert oracle_mod.place(tr, np.arange(3, dtype=np.uint32), best_fit=True)[0].tolist() == [0, 0, 0]
    # two holes of the same size: the lower one; a hole of exactly the size beats a larger one below it
    #   step 0: a [0,2) b [2,3) c [3,5) d [5,6) e [6,9) f [9,10); b, d, f live on to step 1
    tr = mk_trace([2 * G, G, 2 * G, G, 3 * G, G, G, 2 * G, 3 * G],
                  [0, 0, 0, 0, 0, 0, 1, 1, 1], [1, 2, 1, 2, 1, 2, 2, 2, 2], T=2)
    off, _ = oracle_mod.place(tr, np.arange(9, dtype=np.uint32), best_fit=True)
    assert (off // G).tolist()[:6] == [0, 2, 3, 5, 6, 9]
    # step 1 sees b [2,3) d [5,6) f [9,10): holes [0,2) 2, [3,5) 2, [6,9) 3
    # v6 (1): smallest fitting hole size 2, two of them -> the lower, 0; then holes [1,2) 1, [3,5) 2, [6,9) 3
    # v7 (2): exact hole [3,5) -> 3;  v8 (3): exact hole [6,9) -> 6
    assert (off // G).tolist()[6:] == [0, 3, 6]


def test_exhaustive_small_orders(oracle_mod):
    """On every order of a 6-variable trace best-fit stays valid, above the peak, and equal to the
    bitmap brute force."""
    g = read_golden("e1_placement.txt")
    tr = mk_trace([int(x) * G for x in g["size"][0]], g["alloc"][0], g["free"][0], T=5)
    _, peak, _ = oracle_mod.load_profile(tr)
    for perm in all_perms(6):
        perm = np.array(perm, np.uint32)
        off, fp = oracle_mod.place(tr, perm, best_fit=True)
        assert check_valid(tr, off) and fp >= peak
        assert np.array_equal(off, grid_best_fit(tr, perm, G))
