"""Pins for the oracle's swap-candidate scores (Section IV-A, IV-B)."""
import numpy as np
import pytest

from helpers import mk_trace, read_golden
from traces import make_config, random_trace
from traces.dnn import Trace


def test_e2_golden(oracle_mod):
    g = read_golden("e2_swaps.txt")
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=8, step_ns=g["step_ns"][0])
    s = oracle_mod.score_swaps(tr, float(g["link_GBps"][0][0]), int(g["min_bytes"][0][0]))
    assert s["candidate"].tolist() == [int(x) for x in g["candidate"][0]]
    assert s["doa_ns"].tolist() == [int(x) for x in g["doa_ns"][0]]
    assert s["aoa"].tolist() == [float(x) for x in g["aoa"][0]]
    assert s["wdoa"].tolist() == [int(x) for x in g["wdoa"][0]]
    assert s["peak_cut"].tolist() == [int(x) for x in g["peak_cut"][0]]
    # default accesses (alloc, free-1) == passing them explicitly
    s2 = oracle_mod.score_swaps(tr, 64.0, 1 << 20, use_gaps=False)
    for k in s:
        assert s[k].tolist() == s2[k].tolist()


def _literal_scores(tr, load, peak, t_peak, link_GBps, min_bytes):
    """Scores re-derived with exact Python integers / Fractions and a literal re-simulation
    of the load curve with the variable taken out."""
    from fractions import Fraction
    T = tr.n_steps
    ns = [1_000_000] * T if tr.step_ns is None else [int(x) for x in tr.step_ns]
    start = [sum(ns[:t]) for t in range(T + 1)]
    rate = Fraction(round(link_GBps * 1000)) / 1000           # bytes per ns
    out = []
    for i in range(tr.n_vars):
        s, a, f = int(tr.size[i]), int(tr.alloc[i]), int(tr.free[i])
        tl, th = int(tr.gap_lo[i]), int(tr.gap_hi[i])
        if th <= tl:
            out.append((0, 0, 0.0, 0, 0))
            continue
        cand = int(s >= min_bytes and a <= t_peak < f)
        xfer = -((-Fraction(s)) // rate)                       # ceil(size / rate) ns
        idle_from, idle_to = start[tl + 1], start[th]          # first access ends, second begins
        doa = idle_to - idle_from - 2 * int(xfer)
        aoa = float(doa) * float(s) if doa >= 0 else float(doa) / float(s)
        wdoa = sum(int(load[t]) for t in range(tl + 1, th))
        cut = 0
        if doa >= 0:
            gone = [t for t in range(T) if start[t] >= idle_from + xfer and start[t + 1] <= idle_to - xfer]
            if gone:
                new = [int(load[t]) - (s if t in gone else 0) for t in range(T)]
                cut = peak - max(new)
        out.append((cand, doa, aoa, wdoa, cut))
    return out


@pytest.mark.parametrize("seed,link", [(0, 64.0), (1, 64.0), (2, 0.5), (3, 1e-3), (4, 900.0), (5, 12.345)])
def test_scores_match_literal_resimulation(oracle_mod, seed, link):
    tr = random_trace(500 + seed, 120, 17, with_step_ns=(seed % 2 == 0))
    load, peak, tpk = oracle_mod.load_profile(tr)
    s = oracle_mod.score_swaps(tr, link, 1 << 14)
    want = _literal_scores(tr, load, peak, tpk, link, 1 << 14)
    got = list(zip(s["candidate"].tolist(), s["doa_ns"].tolist(), s["aoa"].tolist(),
                   s["wdoa"].tolist(), s["peak_cut"].tolist()))
    assert got == want


def test_peak_cut_literal_small_traces(oracle_mod):
    """Few variables, so single variables move the peak: many non-zero cuts to compare."""
    nonzero = 0
    for seed in range(80):
        tr = random_trace(900 + seed, 12, 9, one_step_frac=0.1, with_step_ns=(seed % 3 == 0))
        load, peak, tpk = oracle_mod.load_profile(tr)
        s = oracle_mod.score_swaps(tr, 64.0, 1)
        want = _literal_scores(tr, load, peak, tpk, 64.0, 1)
        assert s["peak_cut"].tolist() == [w[4] for w in want]
        assert s["doa_ns"].tolist() == [w[1] for w in want]
        nonzero += sum(w[4] > 0 for w in want)
    assert nonzero >= 15


def test_negative_doa_uses_inverse_size(oracle_mod):
    # Section IV-B: when the transfers take longer than the gap, AOA = DOA / size, and a larger
    # (less negative) value still means a relatively better candidate.
    tr = mk_trace([1 << 30, 1 << 20], [0, 0], [3, 3], T=3)
    s = oracle_mod.score_swaps(tr, 1.0, 1)
    assert (s["doa_ns"] < 0).all()
    assert s["aoa"].tolist() == [s["doa_ns"][0] / float(1 << 30), s["doa_ns"][1] / float(1 << 20)]
    assert s["peak_cut"].tolist() == [0, 0]


def test_adjacent_accesses(oracle_mod):
    # accesses at consecutive steps: nothing idle -> DOA = -2*delta, WDOA = 0, cut = 0
    tr = mk_trace([64000, 512], [0, 0], [2, 2], T=2)
    s = oracle_mod.score_swaps(tr, 64.0, 1)
    assert s["doa_ns"].tolist() == [-2000, -16] and s["wdoa"].tolist() == [0, 0]
    assert s["peak_cut"].tolist() == [0, 0]


def test_fast_link_limit(oracle_mod):
    # transfer time -> 1 ns: the variable is away for every idle step except the first and the
    # last one (a step counts only if it lies wholly between swap-out end and swap-in start)
    tr = mk_trace([4096, 1024, 2048], [0, 1, 3], [7, 2, 4], T=7)
    load, peak, tpk = oracle_mod.load_profile(tr)
    assert load.tolist() == [4096, 5120, 4096, 6144, 4096, 4096, 4096] and (peak, tpk) == (6144, 3)
    s = oracle_mod.score_swaps(tr, 9.0e6, 1)
    # v0: accesses 0 and 6, idle steps 1..5, away on 2..4 -> curve 4096,5120,0,2048,0,4096,4096
    assert s["doa_ns"][0] == 5_000_000 - 2
    assert s["wdoa"][0] == 5120 + 4096 + 6144 + 4096 + 4096
    assert s["peak_cut"][0] == 6144 - 5120
    assert s["candidate"].tolist() == [1, 0, 0]          # v1, v2 have no gap
    # shrink the gap to accesses 1 and 5: idle 2..4, away on step 3 only -> 4096+... peak 5120
    tr2 = mk_trace([4096, 1024, 2048], [0, 1, 3], [7, 2, 4], T=7, gap_lo=[1, 1, 3], gap_hi=[5, 1, 3])
    s2 = oracle_mod.score_swaps(tr2, 9.0e6, 1)
    assert s2["peak_cut"][0] == 1024 and s2["wdoa"][0] == 4096 + 6144 + 4096
    # accesses 2 and 4: idle step 3 only, and it is not wholly inside the window -> no cut
    tr3 = mk_trace([4096, 1024, 2048], [0, 1, 3], [7, 2, 4], T=7, gap_lo=[2, 1, 3], gap_hi=[4, 1, 3])
    s3 = oracle_mod.score_swaps(tr3, 9.0e6, 1)
    assert s3["peak_cut"][0] == 0 and s3["wdoa"][0] == 6144 and s3["doa_ns"][0] == 1_000_000 - 2


def test_bad_link_rejected(oracle_mod):
    tr = mk_trace([512], [0], [2])
    for link in (0.0, -1.0, float("nan"), float("inf"), 1e-9):
        assert oracle_mod.score_swaps(tr, link, 1, check=False) == -5


@pytest.mark.parametrize("cfg", [1, 3])
def test_configs_have_useful_candidates(oracle_mod, cfg):
    tr = make_config(cfg)
    s = oracle_mod.score_swaps(tr, tr.meta["link_GBps"], tr.meta["min_bytes"])
    assert (s["peak_cut"] > 0).any()
    if cfg == 3:       # the tiny net has no variable of 1 MiB; ResNet-50 has many
        assert s["candidate"].sum() > 0
        assert (s["peak_cut"][s["candidate"] == 1] > 0).any()
    assert (s["peak_cut"] <= tr.size).all()
