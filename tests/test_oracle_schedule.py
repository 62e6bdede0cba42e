"""Pins for the oracle's swap schedule (Section IV-E)."""
import numpy as np
import pytest

from helpers import mk_trace, read_golden
from traces import make_config, random_trace


def _ints(r):
    return [int(x) for x in r]


def test_e5_golden(oracle_mod):
    g = read_golden("e5_schedule.txt")
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=10, gap_lo=_ints(g["gap_lo"][0]),
                  gap_hi=_ints(g["gap_hi"][0]), step_ns=[100] * 10)
    r = oracle_mod.schedule_swaps(tr, 1.0, _ints(g["swap_list"][0]))
    for k in ("out_start", "out_end", "in_start", "in_end", "load"):
        assert r[k].tolist() == _ints(g[k][0]), k
    assert r["peak"] == 620 and r["late_ns"] == 0
    # the order of the list does not matter, results follow the positions
    r2 = oracle_mod.schedule_swaps(tr, 1.0, [0, 1, 2])
    assert r2["out_start"].tolist() == [100, 250, 370] and r2["in_start"].tolist() == [750, 570, 690]
    assert r2["load"].tolist() == r["load"].tolist()
    # nothing selected: the plain load curve
    r0 = oracle_mod.schedule_swaps(tr, 1.0, [])
    assert r0["load"].tolist() == [330] * 4 + [830, 830] + [330] * 4 and r0["late_ns"] == 0


def _check_defining_properties(tr, link, sl, r):
    """An as-soon-as-possible stream schedule is the only one in which every job starts at its
    ready time or exactly when its predecessor ends; an as-late-as-possible one the only one in
    which every job ends at its due time or exactly when its successor starts."""
    ns = np.full(tr.n_steps, 1_000_000, np.int64) if tr.step_ns is None else tr.step_ns.astype(np.int64)
    start = np.concatenate([[0], np.cumsum(ns)])
    bpus = round(link * 1000)
    delta = [-(-int(tr.size[v]) * 1000 // bpus) for v in sl]
    k = len(sl)
    assert all(r["out_end"][j] - r["out_start"][j] == delta[j] for j in range(k))
    assert all(r["in_end"][j] - r["in_start"][j] == delta[j] for j in range(k))
    o = sorted(range(k), key=lambda j: (int(tr.gap_lo[sl[j]]), sl[j]))
    for a, j in enumerate(o):
        ready = int(start[tr.gap_lo[sl[j]] + 1])
        prev_end = int(r["out_end"][o[a - 1]]) if a else None
        assert r["out_start"][j] >= ready and (prev_end is None or r["out_start"][j] >= prev_end)
        assert r["out_start"][j] == ready or r["out_start"][j] == prev_end
    i = sorted(range(k), key=lambda j: (int(tr.gap_hi[sl[j]]), sl[j]))
    for a, j in enumerate(i):
        due = int(start[tr.gap_hi[sl[j]]])
        nxt = int(r["in_start"][i[a + 1]]) if a + 1 < k else None
        assert r["in_end"][j] <= due and (nxt is None or r["in_end"][j] <= nxt)
        assert r["in_end"][j] == due or r["in_end"][j] == nxt
    # load: exact re-derivation, step by step
    T = tr.n_steps
    load = [sum(int(tr.size[v]) for v in range(tr.n_vars) if tr.alloc[v] <= t < tr.free[v]) for t in range(T)]
    late = 0
    for j, v in enumerate(sl):
        if r["out_end"][j] > r["in_start"][j]:
            late += int(r["out_end"][j] - r["in_start"][j])
            continue
        for t in range(T):
            if start[t] >= r["out_end"][j] and start[t + 1] <= r["in_start"][j]:
                load[t] -= int(tr.size[v])
    assert [int(x) for x in r["load"]] == load and r["peak"] == max(load) and r["late_ns"] == late


def _event_queue_out_stream(tr, link, sl):
    """The swap-out stream as a machine with a clock: jobs arrive when their access completes and
    are served first come first served (ties by variable index)."""
    ns = np.full(tr.n_steps, 1_000_000, np.int64) if tr.step_ns is None else tr.step_ns.astype(np.int64)
    start = np.concatenate([[0], np.cumsum(ns)])
    bpus = round(link * 1000)
    arrivals = sorted((int(start[tr.gap_lo[v] + 1]), int(tr.gap_lo[v]), v, j) for j, v in enumerate(sl))
    clock, res = 0, {}
    for at, _, v, j in arrivals:
        clock = max(clock, at)
        res[j] = clock
        clock += -(-int(tr.size[v]) * 1000 // bpus)
    return [res[j] for j in range(len(sl))]


@pytest.mark.parametrize("seed", range(10))
def test_properties_on_random_traces(oracle_mod, seed):
    tr = random_trace(8000 + seed, n=60 + 11 * seed, T=20 + 2 * seed, size_choices=(512, 1024, 4096, 1 << 14),
                      max_life=18, with_step_ns=bool(seed % 2))
    rng = np.random.default_rng(seed)
    cand = np.nonzero(tr.gap_hi > tr.gap_lo)[0]
    for link in (0.002, 0.05, 64.0):
        sl = rng.permutation(cand)[: max(1, len(cand) * 2 // 3)].astype(np.uint32).tolist()
        r = oracle_mod.schedule_swaps(tr, link, sl)
        _check_defining_properties(tr, link, sl, r)
        assert r["out_start"].tolist() == _event_queue_out_stream(tr, link, sl)
    # the slow links overbook the streams somewhere in these cases, the fast one hides everything
    assert oracle_mod.schedule_swaps(tr, 0.002, sl)["late_ns"] > 0


def test_fast_link_matches_the_selection_walk(oracle_mod):
    """With a link so fast that no transfer waits for another, the schedule's windows are the ones
    the selection walk assumes, so the peak under the schedule is the walk's peak."""
    tr = make_config(2)
    sel = oracle_mod.select_swaps(tr, 1e6, 1 << 20, 2, [0])
    k = sel["n_cand"]
    r = oracle_mod.schedule_swaps(tr, 1e6, sel["order"][:k])
    assert r["peak"] == int(sel["peaks"][k])          # (variables with adjacent accesses are late in both)
    r1 = oracle_mod.schedule_swaps(tr, 1e6, sel["order"][:3])
    assert r1["peak"] == int(sel["peaks"][3])
