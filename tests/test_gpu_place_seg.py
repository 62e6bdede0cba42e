"""GPU parity of lap_plan_pool on the segment-list path (free lists per time segment, the structure
for traces whose variables live long), forced on small traces through LAP_OPT_SEG_MIN_VARS = 0 so
that the oracle can recompute every ordering: offsets and footprints element by element, first-fit
and best-fit.  At full size the same path places configuration 4 (tests/test_gpu_fullsize.py)."""
import numpy as np
import pytest

from gpu_util import oracle_all_orderings, u64
from traces import make_config, make_orderings, random_trace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lap():
    import paper_1903_06631_amd as lap
    lap.load_library()
    lap.set_option(lap.OPT_SEG_MIN_VARS, 0)
    lap.set_option(lap.OPT_SEG_TRIAL_PERCENT, 0)             # no trial run: the lists place whatever applies
    yield lap
    lap.set_option(lap.OPT_SEG_MIN_VARS, lap.SEG_MIN_VARS_DEFAULT)
    lap.set_option(lap.OPT_SEG_TRIAL_PERCENT, lap.SEG_TRIAL_PERCENT_DEFAULT)


def _check(lap, oracle, tr, kinds, seeds, fits=None, explicit_np=None):
    import torch
    dt = lap.DeviceTrace(tr)
    explicit = None
    if explicit_np:
        explicit = {b: torch.from_numpy(p.astype(np.uint32).view(np.int32)).to(dt.device)
                    for b, p in explicit_np.items()}
    got = lap.plan_pool(dt, kinds, seeds, fits=fits, explicit=explicit)
    ref = oracle_all_orderings(oracle, tr, kinds, seeds, explicit_np, None, fits)
    all_off, fps = u64(got["all_offsets"]), u64(got["footprints"])
    for b, (_, off, fp) in ref.items():
        assert np.array_equal(all_off[b], off), f"ordering {b} kind {kinds[b]}"
        assert fps[b] == fp, f"ordering {b}"
    best = int(got["best_ordering"].item())
    assert best == int(np.argmin(fps)) and np.array_equal(u64(got["best_offsets"]), all_off[best])


def _long_lived(seed, n, T, frac=0.3, max_life=None):
    """lifetimes that sum to far more than 6 n steps: the per-step-list path does not apply"""
    tr = random_trace(4000 + seed, n, T, size_choices=[1, 1, 2, 3, 5, 8, 13, 64], one_step_frac=frac, max_life=max_life)
    return tr


@pytest.mark.parametrize("seed,n,T,max_life", [
    (0, 1, 1, None), (1, 2, 2, None), (2, 64, 3, None),            # one segment, fewer steps than the narrowest segment
    (3, 300, 4, None), (4, 301, 5, None), (5, 700, 17, None),      # ragged last segment
    (6, 1500, 64, None), (7, 2600, 129, None), (8, 5000, 1000, None), (9, 4000, 4097, None),
    (10, 3000, 70001, 3000),                     # more than 65535 steps
    (11, 3000, 70001, None),                     # ... and lifetimes too long for the list pool: the sweep takes over
])
def test_segment_lists_random(lap, oracle_mod, seed, n, T, max_life):
    tr = _long_lived(seed, n, T, max_life=max_life)
    kinds, seeds = make_orderings(20)
    kinds = kinds.copy(); kinds[7::8] = 6
    _check(lap, oracle_mod, tr, kinds, seeds)
    _check(lap, oracle_mod, tr, kinds[:10], seeds[:10], fits=[1] * 10)
    _check(lap, oracle_mod, tr, kinds[:12], seeds[:12], fits=[b % 2 for b in range(12)])    # both policies in one call


def test_segment_lists_whole_time_line_and_mixed_lifetimes(lap, oracle_mod):
    """Variables that live through the whole time line (they ask the one list of everything), variables
    that end exactly on segment boundaries, one-step variables, and everything between."""
    rng = np.random.default_rng(5)
    T, n = 256, 3000
    tr = random_trace(4100, n, T, size_choices=[1, 2, 3, 7, 20, 50])
    a, f = tr.alloc.copy(), tr.free.copy()
    a[:300], f[:300] = 0, T                                      # whole time line
    a[300:600] = (rng.integers(0, 16, 300) * 16).astype(np.uint32)            # aligned starts
    f[300:600] = np.minimum(a[300:600] + 16 * rng.integers(1, 8, 300), T).astype(np.uint32)
    f[600:900] = a[600:900] + 1                                  # one step
    tr.alloc, tr.free = a, f
    tr.gap_lo, tr.gap_hi = a.copy(), (f - 1).astype(np.uint32)
    assert oracle_mod.validate_trace(tr) == 0
    kinds, seeds = make_orderings(24)
    _check(lap, oracle_mod, tr, kinds, seeds)
    _check(lap, oracle_mod, tr, kinds[:8], seeds[:8], fits=[1] * 8)


def test_segment_lists_explicit_permutation_and_more_orderings_than_slots(lap, oracle_mod):
    """An explicit order, and a batch whose orderings outnumber the room in the list pool (the
    workgroups then take several orderings one after the other)."""
    tr = _long_lived(20, 400, 2000, frac=0.05)                   # long lifetimes: every ordering needs many entries
    B = 96
    kinds, seeds = make_orderings(B)
    rng = np.random.default_rng(1)
    explicit = {5: rng.permutation(tr.n_vars).astype(np.uint32)}
    kinds = kinds.copy(); kinds[5] = 5
    _check(lap, oracle_mod, tr, kinds, seeds, explicit_np=explicit)


def _unit_holes_trace(M, fillers=70):
    """Two-step variables A_i (steps 0-1) and one-step variables B_i (step 0) of one unit each, placed in the
    order A_0 B_0 A_1 B_1 ..., land at addresses 0, 1, 2, 3, ...: at step 1 the A's then leave M holes of one
    unit between them.  What follows lives at step 1: a variable of two units has to pass all of those holes,
    variables of one unit fill them one by one (each time a range vanishes from a list of M), variables of
    steps 1-2 ask three lists.  `fillers` long-lived variables elsewhere on the time line keep the sum of the
    lifetimes above what per-step lists take.  Returns the trace and the rank order."""
    from traces.dnn import Trace
    U = 512
    size, alloc, free = [], [], []
    def add(units, a, f):
        size.append(units * U); alloc.append(a); free.append(f)
        return len(size) - 1
    order = []
    for i in range(M):
        order.append(add(1, 0, 2))
        order.append(add(1, 0, 1))
    order.append(add(2, 1, 2))                       # walks over M unit holes to the top
    for j in range(150):
        order.append(add(1, 1, 2))                   # fills the lowest hole exactly
        if j % 10 == 0:
            order.append(add(2, 1, 2))
        if j % 7 == 0:
            order.append(add(1, 1, 3))               # steps 1-2
    order.append(add(3, 0, 2))
    T = 4099
    for k in range(fillers):
        order.insert((k * 977) % len(order), add(5 + k % 3, 3 + (k % 5), T - (k % 7)))
    n = len(size)
    a, f = np.asarray(alloc, np.uint32), np.asarray(free, np.uint32)
    tr = Trace(name="unit-holes", n_steps=T, size=np.asarray(size, np.uint64), alloc=a, free=f,
               gap_lo=a.copy(), gap_hi=(f - 1).astype(np.uint32), meta={"cfg": 0})
    assert sorted(order) == list(range(n))
    return tr, np.asarray(order, np.uint32)


def test_lists_of_many_thousand_ranges(lap, oracle_mod):
    """Lists far longer than what the random traces grow (20 000 ranges in one list): the one-wave path's
    searches take two 64-way sampling levels, its walks pass hundreds of chunks, and a range that vanishes or
    splits low in the list moves a tail of thousands of entries."""
    tr, order = _unit_holes_trace(20000)
    assert oracle_mod.validate_trace(tr) == 0
    assert int((tr.free.astype(np.int64) - tr.alloc).sum()) + tr.n_steps > 6 * tr.n_vars      # no per-step lists
    kinds, seeds = make_orderings(6)
    kinds, seeds = kinds[3:6].copy(), seeds[3:6]                  # two seeded shuffles and the order above
    kinds[2] = 5
    explicit = {2: order}
    _check(lap, oracle_mod, tr, kinds, seeds, explicit_np=explicit)
    # the explicit order really leaves the holes: the first variable of two units sits above all A's
    perm, off, _ = oracle_all_orderings(oracle_mod, tr, kinds, seeds, explicit, which=[2])[2]
    two_units = int(order[np.flatnonzero((tr.size[order] == 1024) & (tr.alloc[order] == 1))[0]])
    assert off[two_units] == (2 * 20000 - 1) * 512


@pytest.mark.parametrize("cfg", [1, 3])
def test_segment_lists_configs(lap, oracle_mod, cfg):
    tr = make_config(cfg)
    B = tr.meta["B"]
    kinds, seeds = make_orderings(B)
    _check(lap, oracle_mod, tr, kinds, seeds)
    _check(lap, oracle_mod, tr, kinds[:32], seeds[:32], fits=[1] * min(32, B))


def test_default_threshold_keeps_small_traces_on_the_sweep(lap, oracle_mod):
    """Same results whichever structure places the trace: the default threshold against the forced path."""
    tr = _long_lived(30, 2000, 300)
    kinds, seeds = make_orderings(16)
    dt = lap.DeviceTrace(tr)
    forced = u64(lap.plan_pool(dt, kinds, seeds)["all_offsets"])
    lap.set_option(lap.OPT_SEG_MIN_VARS, lap.SEG_MIN_VARS_DEFAULT)
    try:
        swept = u64(lap.plan_pool(dt, kinds, seeds)["all_offsets"])
    finally:
        lap.set_option(lap.OPT_SEG_MIN_VARS, 0)
    assert np.array_equal(forced, swept)


def test_trial_run_hands_random_lifetimes_back_to_the_sweep(lap, oracle_mod):
    """With the trial on, a trace with lifetimes at random (searches of many rounds) is placed by the sweep
    and a nested one by the lists; the offsets are the oracle's either way."""
    lap.set_option(lap.OPT_SEG_TRIAL_PERCENT, lap.SEG_TRIAL_PERCENT_DEFAULT)
    try:
        tr = _long_lived(40, 3000, 900)
        kinds, seeds = make_orderings(8)
        _check(lap, oracle_mod, tr, kinds, seeds)
        _check(lap, oracle_mod, make_config(3), kinds, seeds)
    finally:
        lap.set_option(lap.OPT_SEG_TRIAL_PERCENT, 0)
