"""Pins for the oracle's selection of swap variables (Section IV-D), the SWDOA order
(Section IV-B iv) and load_min (Section VI-B1)."""
import numpy as np
import pytest

from helpers import mk_trace, read_golden
from traces import make_config, random_trace

KINDS = {"doa": 0, "aoa": 1, "wdoa": 2, "swdoa": 3, "peak_cut": 4}


def _ints(row):
    return [int(x) for x in row]


def test_e3_golden(oracle_mod):
    g = read_golden("e3_select.txt")
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=int(g["n_steps"][0][0]),
                  gap_lo=_ints(g["gap_lo"][0]), gap_hi=_ints(g["gap_hi"][0]))
    limits = _ints(g["limits"][0])
    for name, kind in KINDS.items():
        r = oracle_mod.select_swaps(tr, 64.0, 1, kind, limits)
        assert r["n_cand"] == int(g["n_cand"][0][0])
        assert r["order"].tolist() == _ints(g["order_" + name][0]), name
        assert r["peaks"].tolist() == _ints(g["peaks"][0])
        assert r["n_selected"].tolist() == _ints(g["n_selected"][0])
        assert r["peak_after"].tolist() == _ints(g["peak_after"][0])
        assert r["load_min"] == int(g["load_min"][0][0])
        assert r["rank"][4] == 0xFFFFFFFF and r["rank"][5] == 0xFFFFFFFF
        assert [int(r["rank"][v]) for v in r["order"]] == list(range(r["n_cand"]))


def test_e2_golden(oracle_mod):
    g = read_golden("e2_swaps.txt")
    s = read_golden("e2_select.txt")
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=8, step_ns=g["step_ns"][0])
    for kind in range(5):
        r = oracle_mod.select_swaps(tr, 64.0, 1 << 20, kind, _ints(s["limits"][0]))
        assert r["order"].tolist() == _ints(s["order"][0])
        assert r["peaks"].tolist() == _ints(s["peaks"][0])
        assert r["n_selected"].tolist() == _ints(s["n_selected"][0])
        assert r["peak_after"].tolist() == _ints(s["peak_after"][0])
        assert r["load_min"] == int(s["load_min"][0][0])


def _matrix_resimulation(tr, sc, kind, link_GBps):
    """Independent formulation: residency as dense 0/1 matrices, exact Python integers.
    The away window is found from step start times with searchsorted; scores other than
    SWDOA come from the (separately pinned) score function and a library sort."""
    n, T = tr.n_vars, tr.n_steps
    ns = np.full(T, 1_000_000, np.int64) if tr.step_ns is None else tr.step_ns.astype(np.int64)
    start = np.concatenate([[0], np.cumsum(ns)])
    steps = np.arange(T)
    live = (tr.alloc[:, None] <= steps[None, :]) & (steps[None, :] < tr.free[:, None])
    idle = (tr.gap_lo[:, None] < steps[None, :]) & (steps[None, :] < tr.gap_hi[:, None])
    size = [int(x) for x in tr.size]
    load = [sum(size[i] for i in range(n) if live[i, t]) for t in range(T)]
    bpus = round(link_GBps * 1000)
    away = np.zeros((n, T), bool)
    for i in range(n):
        if tr.gap_hi[i] <= tr.gap_lo[i]:
            continue
        delta = -(-size[i] * 1000 // bpus)
        w0 = int(start[tr.gap_lo[i] + 1]) + delta
        w1 = int(start[tr.gap_hi[i]]) - delta
        if w1 - w0 < 0:
            continue
        # whole steps [start[t], start[t+1]) inside [w0, w1)
        lo = int(np.searchsorted(start, w0, side="left"))
        hi = int(np.searchsorted(start, w1, side="right")) - 1
        if hi > lo:
            away[i, lo:hi] = True
    cands = [i for i in range(n) if sc["candidate"][i]]
    load_min = max(load[t] - sum(size[i] for i in cands if idle[i, t]) for t in range(T))
    cur = list(load)
    order, peaks = [], [max(cur)]
    if kind != 3:
        key = {0: sc["doa_ns"], 1: sc["aoa"], 2: sc["wdoa"], 4: sc["peak_cut"]}[kind]
        conv = float if kind == 1 else int
        order = sorted(cands, key=lambda i: (-conv(key[i]), i))
        for v in order:
            cur = [cur[t] - size[v] * int(away[v, t]) for t in range(T)]
            peaks.append(max(cur))
    else:
        rest = list(cands)
        while rest:
            w = {i: sum(cur[t] for t in range(T) if idle[i, t]) for i in rest}
            v = min(rest, key=lambda i: (-w[i], i))
            rest.remove(v)
            order.append(v)
            cur = [cur[t] - size[v] * int(away[v, t]) for t in range(T)]
            peaks.append(max(cur))
    return order, peaks, load_min


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("kind", range(5))
def test_against_matrix_resimulation(oracle_mod, seed, kind):
    tr = random_trace(7000 + seed, n=40 + 7 * seed, T=24 + 3 * seed, size_choices=(512, 1024, 4096, 1 << 14, 3 << 13),
                      max_life=20, with_step_ns=bool(seed % 2))
    link = [0.004, 0.05, 1.0][seed % 3]      # slow links so that transfers span several steps
    sc = oracle_mod.score_swaps(tr, link, 1024)
    r = oracle_mod.select_swaps(tr, link, 1024, kind, [0])
    order, peaks, load_min = _matrix_resimulation(tr, sc, kind, link)
    assert r["n_cand"] == len(order) and r["n_cand"] >= 3
    assert r["order"].tolist() == order
    assert [int(x) for x in r["peaks"]] == peaks
    assert r["load_min"] == load_min


def test_orders_really_differ(oracle_mod):
    """The fixtures above would not tell the score kinds apart if every kind gave one order."""
    seen = set()
    g = read_golden("e3_select.txt")
    cases = [(mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=12, gap_lo=_ints(g["gap_lo"][0]),
                       gap_hi=_ints(g["gap_hi"][0])), 64.0)]
    for seed in range(6):
        cases.append((random_trace(7000 + seed, n=40 + 7 * seed, T=24 + 3 * seed,
                                   size_choices=(512, 1024, 4096, 1 << 14, 3 << 13), max_life=20,
                                   with_step_ns=bool(seed % 2)), [0.004, 0.05, 1.0][seed % 3]))
    for tr, link in cases:
        orders = [tuple(oracle_mod.select_swaps(tr, link, 1, k, [0])["order"].tolist()) for k in range(5)]
        for a in range(5):
            for b in range(a + 1, 5):
                if orders[a] != orders[b]:
                    seen.add((a, b))
    assert len(seen) == 10


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_walk_properties(oracle_mod, cfg):
    tr = make_config(cfg)
    link, mb = tr.meta["link_GBps"], tr.meta["min_bytes"]
    load, peak, _ = oracle_mod.load_profile(tr)
    sc = oracle_mod.score_swaps(tr, link, mb)
    for kind in range(5):
        limits = [peak, peak - 1, (peak * 3) // 4, peak // 2, 0]
        r = oracle_mod.select_swaps(tr, link, mb, kind, limits)
        pk = r["peaks"].astype(object)
        assert r["n_cand"] == int(sc["candidate"].sum())
        assert sorted(r["order"].tolist()) == np.nonzero(sc["candidate"])[0].tolist()
        assert pk[0] == peak
        assert all(pk[k + 1] <= pk[k] for k in range(len(pk) - 1))        # removing load never raises the peak
        assert r["load_min"] <= pk[-1]                                    # idle steps contain the away steps
        for q, lim in enumerate(limits):
            k = int(r["n_selected"][q])
            assert r["peak_after"][q] == pk[k]
            assert all(pk[j] > lim for j in range(k))                     # the walk did not stop earlier
            assert pk[k] <= lim or k == r["n_cand"]
        assert r["n_selected"][0] == 0
        if kind == 2 or kind == 3:      # first SWDOA pick is the WDOA maximum
            c = np.nonzero(sc["candidate"])[0]
            if len(c):
                assert r["order"][0] == c[np.argmax(sc["wdoa"][c])]
        if kind == 4 and r["n_cand"]:
            assert pk[1] == peak - int(sc["peak_cut"][r["order"][0]])


def test_planted_mistakes_are_caught(oracle_mod):
    """A walk that forgets to update the curve (plain WDOA instead of SWDOA) or that takes the
    idle steps for the away steps fails the hand-worked example."""
    g = read_golden("e3_select.txt")
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=12, gap_lo=_ints(g["gap_lo"][0]),
                  gap_hi=_ints(g["gap_hi"][0]))
    r2 = oracle_mod.select_swaps(tr, 64.0, 1, 2, [0])
    r3 = oracle_mod.select_swaps(tr, 64.0, 1, 3, [0])
    assert r2["order"].tolist() != r3["order"].tolist()
    # idle steps instead of away steps would have taken v0 out of steps 1..7 and v2 out of 8..10:
    # the peak after all four would be 78, not 84
    assert r3["peaks"][-1] == 84 and r3["load_min"] == 78


def test_no_candidates(oracle_mod):
    tr = mk_trace([100, 200], [0, 1], [1, 2], T=2)
    r = oracle_mod.select_swaps(tr, 64.0, 1, 3, [50])
    assert r["n_cand"] == 0 and r["peaks"].tolist() == [200]
    assert r["n_selected"].tolist() == [0] and r["peak_after"].tolist() == [200] and r["load_min"] == 200
