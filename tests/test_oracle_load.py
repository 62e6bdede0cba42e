"""Pins for the oracle's load profile (Section II Def. 2/4, Eq. 1)."""
import itertools

import numpy as np
import pytest

from helpers import mk_trace, overlaps, read_golden
from traces import make_config, random_trace


def test_e1_golden(oracle_mod):
    g = read_golden("e1_placement.txt")
    tr = mk_trace(np.array(g["size"][0], dtype=np.uint64) * 512, g["alloc"][0], g["free"][0], T=int(g["n_steps"][0][0]))
    load, peak, tpk = oracle_mod.load_profile(tr)
    assert (load // 512).tolist() == [int(x) for x in g["load"][0]]
    assert peak == int(g["peak"][0][0]) * 512 and tpk == int(g["t_peak"][0][0])
    assert oracle_mod.count_edges(tr) == int(g["edges"][0][0])


def test_e2_golden(oracle_mod):
    g = read_golden("e2_swaps.txt")
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=8)
    load, peak, tpk = oracle_mod.load_profile(tr)
    assert load.tolist() == [int(x) for x in g["load"][0]]
    assert peak == int(g["peak"][0][0]) and tpk == int(g["t_peak"][0][0])


@pytest.mark.parametrize("seed", range(8))
def test_event_sort_prefix_sum(oracle_mod, seed):
    """A different algorithm: +size/-size events ordered by time, running sum."""
    tr = random_trace(seed, 300, 37, size_choices=[1, 2, 3, 8, 100])
    ev = [(int(a), int(s)) for a, s in zip(tr.alloc, tr.size)] + [(int(f), -int(s)) for f, s in zip(tr.free, tr.size)]
    ev.sort()
    run, k, want = 0, 0, []
    for t in range(tr.n_steps):
        while k < len(ev) and ev[k][0] <= t:
            run += ev[k][1]
            k += 1
        want.append(run)
    load, peak, tpk = oracle_mod.load_profile(tr)
    assert load.tolist() == want
    assert peak == max(want) and tpk == want.index(max(want))


@pytest.mark.parametrize("seed", range(6))
def test_peak_is_max_weight_clique(oracle_mod, seed):
    """Eq. 1: the peak load is the largest total weight of a clique of G."""
    tr = random_trace(100 + seed, 9, 6, size_choices=[1, 2, 3, 5, 7])
    n = tr.n_vars
    best = 0
    for mask in range(1, 1 << n):
        idx = [i for i in range(n) if mask >> i & 1]
        if all(overlaps(tr, i, j) for i, j in itertools.combinations(idx, 2)):
            best = max(best, int(tr.size[idx].sum()))
    assert oracle_mod.load_profile(tr)[1] == best


def test_disjoint_lifetimes_peak_is_max_size(oracle_mod):
    # Section VI-A: exact per-variable allocation consumes the peak load; with no two
    # variables alive together that is the largest variable.
    tr = mk_trace([512 * k for k in (3, 9, 1, 4)], [0, 1, 2, 3], [1, 2, 3, 4])
    load, peak, tpk = oracle_mod.load_profile(tr)
    assert peak == 9 * 512 and tpk == 1 and load.tolist() == [3 * 512, 9 * 512, 512, 4 * 512]


def test_all_overlapping_peak_is_sum(oracle_mod):
    tr = mk_trace([512, 1024, 1536], [0, 1, 2], [5, 4, 3], T=6)
    load, peak, tpk = oracle_mod.load_profile(tr)
    assert peak == 3072 and tpk == 2 and load[5] == 0


def test_peak_time_is_earliest(oracle_mod):
    tr = mk_trace([512, 512], [0, 3], [1, 4], T=5)
    assert oracle_mod.load_profile(tr)[2] == 0


def test_free_before_alloc_at_same_step(oracle_mod):
    # half-open lifetimes: a variable freed at step 2 and one allocated at step 2 never coexist
    tr = mk_trace([1000, 1000], [0, 2], [2, 4])
    load, peak, _ = oracle_mod.load_profile(tr)
    assert peak == 1000 and oracle_mod.count_edges(tr) == 0


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_configs_shape(oracle_mod, cfg):
    """Section II-D: load rises in forward, peaks near the end of forward, falls in backward."""
    tr = make_config(cfg)
    load, peak, tpk = oracle_mod.load_profile(tr)
    F = tr.n_steps // 2
    assert abs(tpk - F) <= max(3, F // 3)
    assert load[0] < peak and load[-1] < peak
    assert oracle_mod.validate_trace(tr) == 0
