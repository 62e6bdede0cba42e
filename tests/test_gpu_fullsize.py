"""Parity at the benchmark configurations' full sizes, in the launch configuration bench.py times: every ordering is
planned on the GPU; a sample of orderings is recomputed by the oracle and compared offset by offset,
and properties that hold for any ordering are checked on all of them."""
import numpy as np
import pytest

from gpu_util import oracle_all_orderings, u64
from traces import make_config, make_orderings

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


@pytest.fixture(scope="module")
def lap():
    import paper_1903_06631_amd as lap
    lap.load_library()
    return lap


def _neighbours_disjoint(tr, off, steps):
    """No two variables alive at the same step share addresses (checked at the given steps)."""
    a, f = tr.alloc.astype(np.int64), tr.free.astype(np.int64)
    e = off + tr.size
    for t in steps:
        live = np.nonzero((a <= t) & (t < f))[0]
        s = live[np.argsort(off[live], kind="stable")]
        if np.any(e[s][:-1] > off[s][1:]):
            return False
    return True


@pytest.mark.parametrize("cfg,sample,step_stride", [(5, [0, 1, 3, 4, 517, 1023], 1), (4, [0, 2, 3, 4, 2048, 4095], 97)])
def test_full_size_plan(lap, oracle_mod, cfg, sample, step_stride):
    tr = make_config(cfg)
    B = tr.meta["B"]
    kinds, seeds = make_orderings(B)
    dt = lap.DeviceTrace(tr)
    got = lap.plan_pool(dt, kinds, seeds)
    fps = u64(got["footprints"])
    best = int(got["best_ordering"].item())
    all_off = got["all_offsets"]
    # sampled orderings, element by element
    ref = oracle_all_orderings(oracle_mod, tr, kinds, seeds, which=sample)
    for b, (_, off, fp) in ref.items():
        assert np.array_equal(u64(all_off[b]), off), f"cfg {cfg} ordering {b}"
        assert fps[b] == fp
    # every ordering: footprint = highest block end, never below the peak load (Eq. 2)
    _, peak, _ = oracle_mod.load_profile(tr)
    size_dev = dt.size
    top = (all_off + size_dev[None, :]).max(dim=1).values        # sums stay far below 2^63
    assert np.array_equal(u64(top), fps)
    assert (fps >= peak).all()
    assert best == int(np.argmin(fps)) and int(u64(got["best_footprint"])[0]) == int(fps.min())
    assert np.array_equal(u64(got["best_offsets"]), u64(all_off[best]))
    # validity of orderings the oracle did not recompute
    steps = range(0, tr.n_steps, step_stride)
    for b in (best, 7, B // 2 + 1):
        assert _neighbours_disjoint(tr, u64(all_off[b]), steps), f"cfg {cfg} ordering {b}"


def test_full_size_best_fit(lap, oracle_mod):
    """Config 5 with every ordering planned best-fit: sampled orderings against the oracle, the
    invariants on all of them."""
    tr = make_config(5)
    B = tr.meta["B"]
    kinds, seeds = make_orderings(B)
    dt = lap.DeviceTrace(tr)
    got = lap.plan_pool(dt, kinds, seeds, fits=[1] * B)
    fps = u64(got["footprints"])
    all_off = got["all_offsets"]
    sample = [0, 3, 4, 700]
    ref = oracle_all_orderings(oracle_mod, tr, kinds, seeds, which=sample, fits=[1] * B)
    for b, (_, off, fp) in ref.items():
        assert np.array_equal(u64(all_off[b]), off), f"ordering {b}"
        assert fps[b] == fp
    _, peak, _ = oracle_mod.load_profile(tr)
    top = (all_off + dt.size[None, :]).max(dim=1).values
    assert np.array_equal(u64(top), fps) and (fps >= peak).all()
    best = int(got["best_ordering"].item())
    for b in (best, 9, B - 1):
        assert _neighbours_disjoint(tr, u64(all_off[b]), range(tr.n_steps)), f"ordering {b}"


def test_full_size_plan_and_replay_of_swaps(lap, oracle_mod):
    """Config 4 (11 000 candidates, 14 000 steps): the swap plan of the WDOA order's prefixes and its
    replay under limits, against the oracle."""
    import torch
    tr = make_config(4)
    link, mb = tr.meta["link_GBps"], tr.meta["min_bytes"]
    dt = lap.DeviceTrace(tr)
    _, peak, _ = oracle_mod.load_profile(tr)
    limits = [peak // 2, peak // 4, peak // 20]
    sel = oracle_mod.select_swaps(tr, link, mb, 2, limits)
    order = sel["order"]
    lst = torch.from_numpy(order.astype(np.uint32).view(np.int32)).cuda()
    k = int(sel["n_selected"][1])
    got = lap.schedule_swaps(dt, link, lst[:k].contiguous())
    ref = oracle_mod.schedule_swaps(tr, link, order[:k])
    for name in ("out_start", "out_end", "in_start", "in_end"):
        assert np.array_equal(got[name].cpu().numpy(), ref[name]), name
    assert np.array_equal(u64(got["load"]), ref["load"]) and int(u64(got["late_ns"])[0]) == ref["late_ns"]
    runs = [(int(sel["n_selected"][q]), limits[q]) for q in range(3)] + [(len(order), 0)]
    sim = lap.simulate_swaps(dt, link, lst, [r[0] for r in runs], [r[1] for r in runs])
    for q, (kq, lim) in enumerate(runs):
        r = oracle_mod.simulate_swaps(tr, link, order[:kq], lim)
        assert int(u64(sim["total_ns"])[q]) == r["total_ns"] and int(u64(sim["peak_resident"])[q]) == r["peak_resident"]
        assert int(sim["forced"].cpu().numpy().view(np.uint32)[q]) == r["forced"]


def test_full_size_load_and_scores(lap, oracle_mod):
    tr = make_config(4)
    dt = lap.DeviceTrace(tr)
    lp = lap.load_profile(dt)
    load, peak, tpk = oracle_mod.load_profile(tr)
    assert np.array_equal(u64(lp["load"]), load) and int(u64(lp["peak"])[0]) == peak and int(lp["t_peak"].item()) == tpk
    got = lap.score_swaps(dt, 64.0, 1 << 20, load=lp["load"])
    ref = oracle_mod.score_swaps(tr, 64.0, 1 << 20)
    assert np.array_equal(got["candidate"].cpu().numpy(), ref["candidate"])
    assert np.array_equal(got["doa_ns"].cpu().numpy(), ref["doa_ns"])
    assert np.array_equal(got["aoa"].cpu().numpy().view(np.uint64), ref["aoa"].view(np.uint64))
    assert np.array_equal(u64(got["wdoa"]), ref["wdoa"])
    assert np.array_equal(u64(got["peak_cut"]), ref["peak_cut"])
