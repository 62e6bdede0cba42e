"""Pins for the oracle's simulation of the swap schedule under a memory-load limit (Section IV-E)."""
import numpy as np
import pytest

from helpers import mk_trace, read_golden
from traces import make_config, random_trace


def _e5():
    g = read_golden("e5_schedule.txt")
    ints = lambda r: [int(x) for x in r]
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=10, gap_lo=ints(g["gap_lo"][0]),
                  gap_hi=ints(g["gap_hi"][0]), step_ns=[100] * 10)
    return tr, ints(g["swap_list"][0])


def test_e6_golden(oracle_mod):
    tr, sl = _e5()
    g = read_golden("e6_simulate.txt")
    for q, lim in enumerate(g["limits"][0]):
        r = oracle_mod.simulate_swaps(tr, 1.0, sl, int(lim))
        assert r["total_ns"] == int(g["total_ns"][0][q]) and r["overhead_ns"] == r["total_ns"] - 1000
        assert r["peak_resident"] == int(g["peak_resident"][0][q]) and r["forced"] == int(g["forced"][0][q])
    r = oracle_mod.simulate_swaps(tr, 1.0, [], 829)
    assert r == dict(total_ns=1000, overhead_ns=0, peak_resident=830, forced=1)
    assert oracle_mod.simulate_swaps(tr, 1.0, [], 830)["forced"] == 0


def test_e6_listed_variable_without_idle_gap(oracle_mod):
    """Section IV-E, reading: a listed variable whose two accesses coincide is never swapped and takes
    no time on the streams of the plan, so its presence moves no other variable's swap-in."""
    g = read_golden("e6_simulate.txt")
    ints = lambda key: [int(x) for x in g[key][0]]
    tr = mk_trace(ints("nogap_size"), ints("nogap_alloc"), ints("nogap_free"), T=10, gap_lo=ints("nogap_gap_lo"),
                  gap_hi=ints("nogap_gap_hi"), step_ns=[100] * 10)
    sl = ints("nogap_swap_list")
    for q, lim in enumerate(ints("nogap_limits")):
        r = oracle_mod.simulate_swaps(tr, 1.0, sl, lim)
        assert r["total_ns"] == ints("nogap_total_ns")[q], lim
        assert r["peak_resident"] == ints("nogap_peak_resident")[q] and r["forced"] == ints("nogap_forced")[q]
        # and the variable's place in the list does not matter
        for other in ([4, 2, 0, 1], [2, 0, 1, 4], [2, 0, 1]):
            assert oracle_mod.simulate_swaps(tr, 1.0, other, lim) == r


def tick_simulation(tr, link, sl, limit, plan):
    """The same machine advanced one nanosecond at a time, written around per-variable states
    instead of event times."""
    n, T = tr.n_vars, tr.n_steps
    ns = [1_000_000] * T if tr.step_ns is None else [int(x) for x in tr.step_ns]
    start = [0]
    for x in ns:
        start.append(start[-1] + x)
    bpus = round(link * 1000)
    size = [int(x) for x in tr.size]
    dur = {v: -(-size[v] * 1000 // bpus) for v in sl}
    jobs = [j for j, v in enumerate(sl) if tr.gap_hi[v] > tr.gap_lo[v]]
    outq = sorted(jobs, key=lambda j: (int(tr.gap_lo[sl[j]]), sl[j]))
    inq = sorted(jobs, key=lambda j: (int(tr.gap_hi[sl[j]]), sl[j]))
    kb = {}
    for j in jobs:
        v = sl[j]
        b = max([t for t in range(int(tr.gap_hi[v]) + 1) if start[t] <= plan["in_start"][j]] or [0])
        kb[j] = max(b, int(tr.gap_lo[v]) + 1)
    state = {j: "resident" for j in jobs}        # resident -> queued_out -> going_out -> away -> coming_in -> back
    left = {}                                    # remaining ns of a running transfer
    R = peak = forced = 0
    t, step_left, now = 0, None, 0
    boundary = 0
    while True:
        # ends
        if step_left == 0:
            R -= sum(size[v] for v in range(n) if tr.free[v] - 1 == t)
            for j in outq:
                if tr.gap_lo[sl[j]] == t:
                    state[j] = "queued_out"
            t += 1
            boundary = t
            step_left = None
        for j in jobs:
            if state[j] == "going_out" and left[j] == 0:
                state[j] = "away"; R -= size[sl[j]]
            if state[j] == "coming_in" and left[j] == 0:
                state[j] = "back"
        if t == T and step_left is None:
            break
        # starts
        if not any(state[j] == "going_out" for j in jobs):
            q = [j for j in outq if state[j] == "queued_out"]
            if q:
                state[q[0]] = "going_out"; left[q[0]] = dur[sl[q[0]]]
        need = sum(size[v] for v in range(n) if tr.alloc[v] == t) if t < T else 0
        ready = t < T and all(state[j] in ("back",) or tr.gap_hi[sl[j]] != t for j in jobs)
        step_blocked = in_blocked = False
        if step_left is None and ready:
            if need == 0 or R + need <= limit:
                R += need; peak = max(peak, R); step_left = ns[t]
            else:
                step_blocked = True
        head = next((j for j in inq if state[j] not in ("coming_in", "back")), None)
        in_busy = any(state[j] == "coming_in" for j in jobs)
        if not in_busy and head is not None and kb[head] <= boundary and state[head] == "away":
            if R + size[sl[head]] <= limit:
                R += size[sl[head]]; peak = max(peak, R); state[head] = "coming_in"; left[head] = dur[sl[head]]
            else:
                in_blocked = True
        running = step_left is not None or any(state[j] in ("going_out", "coming_in") for j in jobs)
        if not running:
            forced += 1
            if step_blocked:
                R += need; step_left = ns[t]
            else:
                assert in_blocked
                R += size[sl[head]]; state[head] = "coming_in"; left[head] = dur[sl[head]]
            peak = max(peak, R)
        # one nanosecond passes
        now += 1
        if step_left is not None:
            step_left -= 1
        for j in jobs:
            if state[j] in ("going_out", "coming_in"):
                left[j] -= 1
    return dict(total_ns=now, overhead_ns=now - start[T], peak_resident=peak, forced=forced)


@pytest.mark.parametrize("seed", range(16))
def test_against_tick_simulation(oracle_mod, seed):
    rng = np.random.default_rng(seed)
    n, T = 14 + seed, 8 + seed % 5
    tr = random_trace(9000 + seed, n=n, T=T, size_choices=(1000, 2000, 3000, 5000), max_life=T, granule=1000)
    tr.step_ns = rng.integers(2, 9, T).astype(np.uint64)
    link = 1000.0                               # 1000 bytes per ns: transfers take 1..5 ns
    cand = [int(v) for v in np.nonzero(tr.gap_hi > tr.gap_lo)[0]]
    sl = [int(x) for x in rng.permutation(cand)[: max(1, len(cand) * 2 // 3)]]
    sl += [int(v) for v in np.nonzero(tr.gap_hi == tr.gap_lo)[0][:1]]      # one that is never swapped
    movable = [v for v in sl if tr.gap_hi[v] > tr.gap_lo[v]]
    plan = oracle_mod.schedule_swaps(tr, link, movable)          # the plan covers the variables that move
    _, peak, _ = oracle_mod.load_profile(tr)
    for lim in (10 ** 12, peak, plan["peak"], (plan["peak"] * 4) // 5, peak // 2, 0):
        got = oracle_mod.simulate_swaps(tr, link, sl, lim)
        assert got == tick_simulation(tr, link, movable, lim, plan), (seed, lim)


@pytest.mark.parametrize("cfg", [2, 3])
def test_loose_limit_costs_nothing(oracle_mod, cfg):
    tr = make_config(cfg)
    link, mb = tr.meta["link_GBps"], tr.meta["min_bytes"]
    _, peak, _ = oracle_mod.load_profile(tr)
    sel = oracle_mod.select_swaps(tr, link, mb, 0, [0])
    # variables with room for both transfers only: nothing is late, nothing waits
    sc = oracle_mod.score_swaps(tr, link, mb)
    sl = [int(v) for v in sel["order"] if sc["doa_ns"][v] > 0][:5]
    plan = oracle_mod.schedule_swaps(tr, link, sl)
    r = oracle_mod.simulate_swaps(tr, link, sl, peak)
    if plan["late_ns"] == 0:
        assert r["overhead_ns"] == 0 and r["forced"] == 0
    assert r["peak_resident"] <= peak
    # no list at all: the run is the plain iteration
    r0 = oracle_mod.simulate_swaps(tr, link, [], peak)
    assert r0["overhead_ns"] == 0 and r0["forced"] == 0 and r0["peak_resident"] == peak
    # a tighter limit never makes the iteration shorter
    prev = 0
    for lim in (peak, peak * 9 // 10, peak * 3 // 4, peak // 2):
        o = oracle_mod.simulate_swaps(tr, link, [int(v) for v in sel["order"]], lim)
        assert o["peak_resident"] <= max(lim, 0) or o["forced"] > 0
        prev = o["overhead_ns"]
