"""Pins for the oracle's evaluation of aggregated-score weight vectors (Section IV-C, Eq. 3)."""
import numpy as np
import pytest

from helpers import mk_trace, read_golden
from traces import make_config, random_trace


def _e3():
    g = read_golden("e3_select.txt")
    ints = lambda r: [int(x) for x in r]
    return mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=12, gap_lo=ints(g["gap_lo"][0]),
                    gap_hi=ints(g["gap_hi"][0]))


UNIT = [[1, 0, 0, 0], [0, 1, 0, 0], [0, 0, 1, 0], [0, 0, 0, 1]]      # AOA, DOA, WDOA, SWDOA


def test_e3_unit_vectors(oracle_mod):
    """The hand-worked orders of e3_select.txt: AOA 0 3 1 2, DOA 0 1 2 3, WDOA 0 1 2 3, SWDOA 0 2 1 3, and the
    SWDOA values worked out there: 418 when v0 is picked, then v2 252, v1 226; v3 stood at 128 while v1 was
    picked, and v1's removal (8 bytes off step 5) leaves it 84 + 36 = 120 at its own pick."""
    tr = _e3()
    r = oracle_mod.evaluate_weights(tr, 64.0, 1, UNIT, 84)
    assert r["swdoa"].tolist() == [418, 226, 252, 120, 0, 0]
    assert r["order"].tolist() == [[0, 3, 1, 2], [0, 1, 2, 3], [0, 1, 2, 3], [0, 2, 1, 3]]
    assert r["n_selected"].tolist() == [1, 1, 1, 1] and r["peak_after"].tolist() == [84] * 4
    # a negative weight reverses an order
    r = oracle_mod.evaluate_weights(tr, 64.0, 1, [[0, -1, 0, 0]], 0)
    assert r["order"].tolist() == [[3, 2, 1, 0]] and r["n_selected"].tolist() == [4]


@pytest.mark.parametrize("seed", range(5))
def test_unit_vectors_reproduce_the_basic_orders(oracle_mod, seed):
    tr = random_trace(9500 + seed, n=80 + 20 * seed, T=30 + seed, size_choices=(512, 1024, 4096, 1 << 14, 3 << 13),
                      max_life=25, with_step_ns=bool(seed % 2))
    link = [0.004, 0.05, 1.0][seed % 3]
    _, peak, _ = oracle_mod.load_profile(tr)
    limit = peak * 2 // 3
    r = oracle_mod.evaluate_weights(tr, link, 1024, UNIT, limit)
    for row, kind in enumerate((1, 0, 2)):                   # AOA, DOA, WDOA walks of the selection oracle
        s = oracle_mod.select_swaps(tr, link, 1024, kind, [limit])
        assert r["order"][row].tolist() == s["order"].tolist()
        assert r["n_selected"][row] == s["n_selected"][0] and r["peak_after"][row] == s["peak_after"][0]
        sim = oracle_mod.simulate_swaps(tr, link, s["order"][: int(s["n_selected"][0])], limit)
        assert r["overhead_ns"][row] == sim["overhead_ns"] and r["forced"][row] == sim["forced"]
    # SWDOA values are non-increasing along the SWDOA walk, so sorting by them gives that walk
    s = oracle_mod.select_swaps(tr, link, 1024, 3, [limit])
    vals = r["swdoa"][s["order"]].astype(np.int64)
    assert np.all(np.diff(vals) <= 0)
    if len(set(vals.tolist())) == len(vals):
        assert r["order"][3].tolist() == s["order"].tolist()
    # the values themselves: the first pick's is its plain WDOA
    sc = oracle_mod.score_swaps(tr, link, 1024)
    if len(s["order"]):
        assert r["swdoa"][s["order"][0]] == sc["wdoa"][s["order"][0]]
    assert all(r["swdoa"][v] <= sc["wdoa"][v] for v in s["order"])
    # scaling all weights by a power of two changes no decision; best is the arg-min
    rng = np.random.default_rng(seed)
    wv = rng.uniform(-1, 1, (12, 4))
    scale = np.array([1.0 / max(1.0, float(np.std(sc[k][sc["candidate"] == 1].astype(np.float64))))
                      for k in ("aoa", "doa_ns", "wdoa")] + [1.0 / max(1.0, float(np.std(r["swdoa"].astype(np.float64))))])
    wv = wv * scale
    r1 = oracle_mod.evaluate_weights(tr, link, 1024, wv, limit)
    r2 = oracle_mod.evaluate_weights(tr, link, 1024, wv * 4.0, limit)
    assert np.array_equal(r1["order"], r2["order"]) and np.array_equal(r1["overhead_ns"], r2["overhead_ns"])
    assert r1["best"] == int(np.argmin(r1["overhead_ns"]))
    assert len({tuple(o) for o in r1["order"].tolist()}) > 3          # the vectors really give different orders
