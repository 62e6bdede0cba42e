"""GPU parity: lap_simulate_swaps against the oracle's discrete-event run, value by value."""
import numpy as np
import pytest

from gpu_util import u64
from helpers import mk_trace, read_golden
from traces import make_config, random_trace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lap():
    import paper_1903_06631_amd as lap
    lap.load_library()
    return lap


def _check(lap, oracle, tr, link, sl, runs, use_gaps=True):
    """runs: list of (prefix length, limit)"""
    import torch
    dt = lap.DeviceTrace(tr, use_gaps=use_gaps)
    lst = torch.from_numpy(np.asarray(sl, dtype=np.uint32).view(np.int32)).to(dt.device)
    got = lap.simulate_swaps(dt, link, lst, [r[0] for r in runs], [r[1] for r in runs])
    tot, ovh, pk = u64(got["total_ns"]), u64(got["overhead_ns"]), u64(got["peak_resident"])
    forced = got["forced"].cpu().numpy().view(np.uint32)
    refs = []
    for q, (k, lim) in enumerate(runs):
        ref = oracle.simulate_swaps(tr, link, list(sl[:k]), lim, use_gaps=use_gaps)
        mine = (int(tot[q]), int(ovh[q]), int(pk[q]), int(forced[q]))
        assert mine == (ref["total_ns"], ref["overhead_ns"], ref["peak_resident"], ref["forced"]), (q, k, lim)
        refs.append(ref)
    return refs


def test_simulate_golden(lap, oracle_mod):
    g = read_golden("e5_schedule.txt")
    ints = lambda r: [int(x) for x in r]
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=10, gap_lo=ints(g["gap_lo"][0]),
                  gap_hi=ints(g["gap_hi"][0]), step_ns=[100] * 10)
    sl = ints(g["swap_list"][0])
    refs = _check(lap, oracle_mod, tr, 1.0, sl, [(3, 10 ** 9), (3, 620), (3, 560), (3, 520), (3, 499), (3, 100),
                                                 (0, 829), (0, 830), (1, 560), (2, 520)])
    assert [r["total_ns"] for r in refs[:4]] == [1000, 1000, 1030, 1060]


def test_simulate_golden_listed_variable_without_idle_gap(lap, oracle_mod):
    g = read_golden("e6_simulate.txt")
    ints = lambda key: [int(x) for x in g[key][0]]
    tr = mk_trace(ints("nogap_size"), ints("nogap_alloc"), ints("nogap_free"), T=10, gap_lo=ints("nogap_gap_lo"),
                  gap_hi=ints("nogap_gap_hi"), step_ns=[100] * 10)
    refs = _check(lap, oracle_mod, tr, 1.0, ints("nogap_swap_list"), [(4, lim) for lim in ints("nogap_limits")])
    assert [r["total_ns"] for r in refs] == ints("nogap_total_ns")
    assert [r["peak_resident"] for r in refs] == ints("nogap_peak_resident")


@pytest.mark.parametrize("seed,n,T", [(0, 1, 1), (1, 30, 9), (2, 400, 25), (3, 3000, 120), (4, 12000, 700)])
def test_simulate_random(lap, oracle_mod, seed, n, T):
    tr = random_trace(1900 + seed, n, T, with_step_ns=(seed % 2 == 0))
    rng = np.random.default_rng(seed)
    cand = np.nonzero(tr.gap_hi > tr.gap_lo)[0]
    sl = rng.permutation(n)[: max(1, n * 2 // 3)].astype(np.uint32)      # includes variables without a gap
    _, peak, _ = oracle_mod.load_profile(tr)
    for link in (0.004, 1.0, 64.0):
        runs = [(len(sl), 10 ** 15), (len(sl), peak), (len(sl), peak * 3 // 4), (len(sl) // 2, peak // 2),
                (len(sl) // 3, peak * 9 // 10), (0, peak), (0, peak - 1), (len(sl), 0), (1, peak // 3)]
        _check(lap, oracle_mod, tr, link, sl, runs)
    _check(lap, oracle_mod, tr, 1.0, sl, [(len(sl), peak * 2 // 3)], use_gaps=False)


@pytest.mark.parametrize("cfg", [2, 3, 5])
def test_simulate_limit_sweep_on_configs(lap, oracle_mod, cfg):
    """what the planner is for: the selection's prefixes for a sweep of limits, each replayed under its limit"""
    tr = make_config(cfg)
    link, mb = tr.meta["link_GBps"], tr.meta["min_bytes"]
    _, peak, _ = oracle_mod.load_profile(tr)
    limits = [peak * q // 10 for q in range(3, 11)]
    sel = oracle_mod.select_swaps(tr, link, mb, 3, limits)
    runs = [(int(sel["n_selected"][q]), limits[q]) for q in range(len(limits))]
    refs = _check(lap, oracle_mod, tr, link, sel["order"], runs)
    assert refs[-1]["overhead_ns"] == 0 and refs[-1]["forced"] == 0          # limit = peak, nothing swapped


def test_simulate_argument_errors(lap):
    import torch
    tr = random_trace(1, 100, 10)
    dt = lap.DeviceTrace(tr)
    lst = torch.arange(4, dtype=torch.int32, device="cuda")
    with pytest.raises(lap.LapError) as e:
        lap.simulate_swaps(dt, 1.0, lst, [5], [100])
    assert e.value.status == -2
    with pytest.raises(lap.LapError) as e:
        lap.simulate_swaps(dt, float("nan"), lst, [4], [100])
    assert e.value.status == -5
