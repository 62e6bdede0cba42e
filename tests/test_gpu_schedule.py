"""GPU parity: lap_schedule_swaps against the oracle's swap schedule, bit for bit."""
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


def _check(lap, oracle, tr, link, sl, use_gaps=True, pass_load=False):
    import torch
    dt = lap.DeviceTrace(tr, use_gaps=use_gaps)
    load = lap.load_profile(dt)["load"] if pass_load else None
    lst = torch.from_numpy(np.asarray(sl, dtype=np.uint32).view(np.int32)).to(dt.device)
    got = lap.schedule_swaps(dt, link, lst, load=load)
    ref = oracle.schedule_swaps(tr, link, sl, use_gaps=use_gaps)
    for k in ("out_start", "out_end", "in_start", "in_end"):
        assert np.array_equal(got[k].cpu().numpy(), ref[k]), k
    assert np.array_equal(u64(got["load"]), ref["load"])
    assert int(u64(got["peak"])[0]) == ref["peak"] and int(u64(got["late_ns"])[0]) == ref["late_ns"]
    return ref


def test_schedule_golden(lap, oracle_mod):
    g = read_golden("e5_schedule.txt")
    ints = lambda r: [int(x) for x in r]
    tr = mk_trace(g["size"][0], g["alloc"][0], g["free"][0], T=10, gap_lo=ints(g["gap_lo"][0]),
                  gap_hi=ints(g["gap_hi"][0]), step_ns=[100] * 10)
    r = _check(lap, oracle_mod, tr, 1.0, ints(g["swap_list"][0]))
    assert r["peak"] == 620
    _check(lap, oracle_mod, tr, 1.0, [])
    _check(lap, oracle_mod, tr, 1.0, [1])


@pytest.mark.parametrize("seed,n,T", [(0, 1, 1), (1, 40, 12), (2, 700, 33), (3, 5000, 300), (4, 30000, 1025),
                                      (5, 2000, 5000)])
def test_schedule_random(lap, oracle_mod, seed, n, T):
    tr = random_trace(1700 + seed, n, T, with_step_ns=(seed % 2 == 0))
    rng = np.random.default_rng(seed)
    cand = np.nonzero(tr.gap_hi > tr.gap_lo)[0]
    if len(cand) == 0:
        cand = np.arange(n)
    for link in (0.003, 0.5, 64.0):
        sl = rng.permutation(cand)[: max(1, len(cand) * 3 // 5)].astype(np.uint32)
        _check(lap, oracle_mod, tr, link, sl, pass_load=(seed % 2 == 1))
    _check(lap, oracle_mod, tr, 1.0, rng.permutation(n)[: max(1, n // 2)].astype(np.uint32), use_gaps=False)
    _check(lap, oracle_mod, tr, 1.0, np.arange(n, dtype=np.uint32))             # everything, several chunks of 1024


@pytest.mark.parametrize("cfg", [2, 3, 5])
def test_schedule_of_selected_variables(lap, oracle_mod, cfg):
    """the lists the selection produces: a prefix of the SWDOA order and all candidates"""
    tr = make_config(cfg)
    link, mb = tr.meta["link_GBps"], tr.meta["min_bytes"]
    sel = oracle_mod.select_swaps(tr, link, mb, 3, [0])
    order = sel["order"]
    for k in (len(order), len(order) // 3):
        r = _check(lap, oracle_mod, tr, link, order[:k])
        assert r["peak"] >= sel["load_min"]
    _check(lap, oracle_mod, tr, link / 50, order)      # a slow link: the streams are overbooked


def test_schedule_argument_errors(lap):
    import torch
    tr = random_trace(1, 100, 10)
    dt = lap.DeviceTrace(tr)
    lst = torch.arange(4, dtype=torch.int32, device="cuda")
    with pytest.raises(lap.LapError) as e:
        lap.schedule_swaps(dt, 0.0, lst)
    assert e.value.status == -5
    with pytest.raises(lap.LapError) as e:
        lap.schedule_swaps(dt, 1.0, torch.arange(101, dtype=torch.int32, device="cuda"))
    assert e.value.status == -2
