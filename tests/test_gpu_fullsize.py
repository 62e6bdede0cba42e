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


def _all_neighbours_disjoint(tr, all_off, size_dev, steps, rows=None, chunk_elems=1 << 28):
    """Section III-B on the device, for many orderings at once: at every given step, the blocks of the
    variables alive at that step, sorted by offset, do not touch each other's addresses.  Two variables
    whose lifetimes overlap are both alive at the later of their two first steps, so checking every
    step at which something is allocated covers every pair.  Returns the number of violations."""
    import torch
    a, f = tr.alloc.astype(np.int64), tr.free.astype(np.int64)
    order = np.argsort(a, kind="stable")
    bad = 0
    off_all = all_off if rows is None else all_off[rows]
    for t in steps:
        live = np.nonzero((a <= t) & (t < f))[0]
        if len(live) < 2:
            continue
        idx = torch.from_numpy(live).to(all_off.device)
        per = max(1, chunk_elems // len(live))
        for r0 in range(0, off_all.shape[0], per):
            o = off_all[r0:r0 + per].index_select(1, idx)
            so, si = torch.sort(o, dim=1)
            e = so + size_dev[idx][si]
            bad += int((e[:, :-1] > so[:, 1:]).sum().item())
    return bad


def _digests(all_off, rows, chunk=64):
    """SHA-256 prefixes of the given orderings' offsets (rows move to the host in chunks)."""
    from helpers import offsets_digest
    out = {}
    for k in range(0, len(rows), chunk):
        part = rows[k:k + chunk]
        host = u64(all_off[part])
        for i, b in enumerate(part):
            out[b] = offsets_digest(host[i])
    return out


def _full_size(lap, oracle_mod, cfg, best_fit, live_sample, all_steps_rows, step_stride, stored_all=False):
    import torch
    from helpers import fullsize_batch, read_fullsize_golden
    tr = make_config(cfg)
    kinds, seeds = fullsize_batch(cfg)
    B = len(kinds)
    assert B == tr.meta["B"]
    fits = [1] * B if best_fit else None
    dt = lap.DeviceTrace(tr)
    got = lap.plan_pool(dt, kinds, seeds, fits=fits)
    fps = u64(got["footprints"])
    best = int(got["best_ordering"].item())
    all_off = got["all_offsets"]

    # 1. every ordering the oracle has been run on ahead of time (stored footprint and digest of the
    #    offsets, written by tests/golden/make_fullsize_hashes.py from the oracle alone)
    gold = read_fullsize_golden(cfg, best_fit)
    assert len(gold) >= 64, f"stored oracle results for cfg {cfg}: {len(gold)}"
    if stored_all:
        assert sorted(gold) == list(range(B)), f"cfg {cfg}: the oracle's result is stored for every ordering"
    assert {0, 1, 2, 3, 4, 6} <= {g[0] for g in gold.values()}, "every ordering kind is among them"
    rows = sorted(gold)
    for b in rows:
        assert (int(kinds[b]), int(seeds[b])) == gold[b][:2], f"ordering {b} is not the one the oracle ran"
    dig = _digests(all_off, rows)
    wrong = [b for b in rows if dig[b] != gold[b][3] or int(fps[b]) != gold[b][2]]
    assert not wrong, f"cfg {cfg}: {len(wrong)} of {len(rows)} orderings differ from the oracle, first {wrong[:8]}"

    # 1b. the orders themselves, rank by rank, for a spread of orderings with every kind among them
    orders = lap.plan_pool_orders(dt, B)
    for b in sorted(set(range(0, B, max(1, B // 40))) | {0, 1, 2, 3, 63, B - 1}):
        want = oracle_mod.make_perm(tr, int(kinds[b]), int(seeds[b]))
        assert np.array_equal(orders[b].cpu().numpy().view(np.uint32), want), f"cfg {cfg}: order of ordering {b}"
    del orders

    # 2. a live sample recomputed by the oracle now (one ordering per host thread), element by element
    ref = oracle_all_orderings(oracle_mod, tr, kinds, seeds, which=live_sample, fits=fits)
    for b, (_, off, fp) in ref.items():
        assert np.array_equal(u64(all_off[b]), off), f"cfg {cfg} ordering {b}"
        assert fps[b] == fp
        if b in gold:
            from helpers import offsets_digest
            assert offsets_digest(off) == gold[b][3] and fp == gold[b][2]     # the stored line is this oracle's

    # 3. every ordering: footprint = highest block end, never below the peak load (Eq. 2); the best one
    _, peak, _ = oracle_mod.load_profile(tr)
    top = (all_off + dt.size[None, :]).max(dim=1).values        # sums stay far below 2^63
    assert np.array_equal(u64(top), fps)
    assert (fps >= peak).all()
    assert best == int(np.argmin(fps)) and int(u64(got["best_footprint"])[0]) == int(fps.min())
    assert np.array_equal(u64(got["best_offsets"]), u64(all_off[best]))

    # 4. every ordering: no two variables alive together share addresses
    alloc_steps = np.unique(tr.alloc)
    if step_stride == 1:
        assert _all_neighbours_disjoint(tr, all_off, dt.size, alloc_steps) == 0
    else:
        assert _all_neighbours_disjoint(tr, all_off, dt.size, alloc_steps[::step_stride]) == 0
        rws = torch.tensor(sorted(set(all_steps_rows) | {best}), device=all_off.device)
        assert _all_neighbours_disjoint(tr, all_off, dt.size, alloc_steps, rows=rws) == 0
    return len(rows)


def test_full_size_plan_transformer(lap, oracle_mod):
    """Config 5, the benchmark's launch: 1024 orderings of 200 000 variables, every one of them compared
    with the oracle's stored result."""
    _full_size(lap, oracle_mod, 5, False, live_sample=[0, 1, 2, 3, 63, 127, 4, 5, 100, 333, 517, 640, 777, 901, 1000, 1023],
               all_steps_rows=[], step_stride=1, stored_all=True)


def test_full_size_plan_deep_chain(lap, oracle_mod):
    """Config 4: 4096 orderings of 50 000 variables on 14 000 steps (dense interval graph; the segment-list
    kernel), every one of them compared with the oracle's stored result.  The pairwise check runs on every
    61st allocation step for all orderings and on every step for 16 of them.  (Best-fit is not run at this size: on a dense trace it looks at thousands of holes per
    variable and takes minutes per ordering.)"""
    _full_size(lap, oracle_mod, 4, False, live_sample=[0, 1, 2, 3, 63, 127, 4, 9, 800, 1500, 2048, 2600, 3100, 3600, 4000, 4095],
               all_steps_rows=list(range(5, 4096, 273)), step_stride=61, stored_all=True)


def test_full_size_best_fit_transformer(lap, oracle_mod):
    """Config 5 with every ordering planned best-fit, every one of them compared with the oracle's stored result."""
    _full_size(lap, oracle_mod, 5, True, live_sample=[0, 1, 2, 3, 63, 4, 6, 200, 700, 1023], all_steps_rows=[], step_stride=1,
               stored_all=True)


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
