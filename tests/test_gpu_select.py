"""GPU parity: lap_select_swaps against the oracle's selection walk, bit for bit."""
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


def _check(lap, oracle, tr, link, min_bytes, kinds, limits, use_gaps=True, pass_load=False, want_rank=True):
    dt = lap.DeviceTrace(tr, use_gaps=use_gaps)
    load = lap.load_profile(dt)["load"] if pass_load else None
    got = lap.select_swaps(dt, link, min_bytes, kinds, limits, load=load, want_rank=want_rank)
    nc = int(got["n_cand"].cpu().numpy().view(np.uint32)[0])
    order = got["order"].cpu().numpy().view(np.uint32)
    peaks = u64(got["peaks"])
    for row, kind in enumerate(kinds):
        ref = oracle.select_swaps(tr, link, min_bytes, kind, limits, use_gaps=use_gaps)
        assert nc == ref["n_cand"]
        assert np.array_equal(order[row, :nc], ref["order"]), kind
        assert np.array_equal(peaks[row, :nc + 1], ref["peaks"]), kind
        if want_rank:
            assert np.array_equal(got["rank"].cpu().numpy().view(np.uint32)[row], ref["rank"]), kind
        if len(limits):
            assert np.array_equal(got["n_selected"].cpu().numpy().view(np.uint32)[row], ref["n_selected"]), kind
            assert np.array_equal(u64(got["peak_after"])[row], ref["peak_after"]), kind
        assert int(u64(got["load_min"])[0]) == ref["load_min"]
    return nc


def test_select_golden_examples(lap, oracle_mod):
    g = read_golden("e3_select.txt")
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=12, gap_lo=[int(x) for x in g["gap_lo"][0]],
                  gap_hi=[int(x) for x in g["gap_hi"][0]])
    assert _check(lap, oracle_mod, tr, 64.0, 1, [0, 1, 2, 3, 4], [90, 84, 83, 94]) == 4
    g = read_golden("e2_swaps.txt")
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=8, step_ns=g["step_ns"][0])
    assert _check(lap, oracle_mod, tr, 64.0, 1 << 20, [3, 2], [8388608, 1 << 40, 0]) == 4


@pytest.mark.parametrize("seed,n,T,link", [(0, 1, 1, 64.0), (1, 40, 24, 0.004), (2, 300, 17, 0.05), (3, 5000, 300, 0.5),
                                           (4, 20000, 1025, 12.345), (5, 3000, 5000, 900.0), (6, 2500, 2049, 1e-3)])
def test_select_random(lap, oracle_mod, seed, n, T, link):
    tr = random_trace(900 + seed, n, T, with_step_ns=(seed % 2 == 0))
    _, peak, _ = oracle_mod.load_profile(tr)
    limits = [peak, peak - 1, peak * 9 // 10, peak * 3 // 4, peak // 2, 0]
    _check(lap, oracle_mod, tr, link, 1 << 14, [0, 1, 2, 3, 4], limits, pass_load=(seed % 3 == 0))
    _check(lap, oracle_mod, tr, link, 1 << 14, [3], [], use_gaps=False, want_rank=False)


def test_select_many_candidates_more_than_one_slot_per_thread(lap, oracle_mod):
    # every variable large enough: thousands of candidates around the peak, several per thread
    tr = random_trace(950, 12000, 40, size_choices=(1 << 16, 1 << 17, 3 << 16), max_life=40, with_step_ns=True)
    nc = _check(lap, oracle_mod, tr, 0.5, 1, [3, 0, 4], [0])
    assert nc > 2048


def test_select_equal_scores_take_the_lower_index(lap, oracle_mod):
    n = 200
    tr = mk_trace([1 << 20] * n, [0] * n, [10] * n, T=10, gap_lo=[1] * n, gap_hi=[8] * n)
    nc = _check(lap, oracle_mod, tr, 64.0, 1, [0, 1, 2, 3, 4], [150 << 20, 0])
    assert nc == n


def test_select_no_candidates_and_kind_repeats(lap, oracle_mod):
    tr = mk_trace([100, 200], [0, 1], [1, 2], T=2)
    assert _check(lap, oracle_mod, tr, 64.0, 1, [3, 3, 0], [50]) == 0


@pytest.mark.parametrize("cfg", [1, 2, 3, 5])
def test_select_configs(lap, oracle_mod, cfg):
    tr = make_config(cfg)
    _, peak, _ = oracle_mod.load_profile(tr)
    limits = [peak * q // 20 for q in range(21)]
    _check(lap, oracle_mod, tr, tr.meta["link_GBps"], tr.meta["min_bytes"], [0, 1, 2, 3, 4], limits)


def test_select_config4_static_scores(lap, oracle_mod):
    # 11000 candidates over 14000 steps; the oracle's SWDOA walk takes minutes there, the static orders seconds
    tr = make_config(4)
    _, peak, _ = oracle_mod.load_profile(tr)
    _check(lap, oracle_mod, tr, tr.meta["link_GBps"], tr.meta["min_bytes"], [2, 4], [peak // 2, peak // 50])


def test_select_argument_errors(lap):
    tr = random_trace(1, 100, 10)
    dt = lap.DeviceTrace(tr)
    with pytest.raises(lap.LapError) as e:
        lap.select_swaps(dt, 64.0, 1, [5], [0])
    assert e.value.status == -4
    with pytest.raises(lap.LapError) as e:
        lap.select_swaps(dt, 0.0, 1, [3], [0])
    assert e.value.status == -5
    with pytest.raises(lap.LapError) as e:
        lap.select_swaps(dt, 64.0, 1, [3], list(range(1025)))
    assert e.value.status == -2
    with pytest.raises(lap.LapError) as e:
        lap.select_swaps(dt, 64.0, 1, [], [0])
    assert e.value.status in (-1, -2)      # the empty output tensors have a null address
