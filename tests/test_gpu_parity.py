"""HIP path vs the CPU oracle, element by element, through the C ABI.  Integer results are
bit-exact; AOA (one binary64 multiply or divide) is compared bit for bit as well."""
import numpy as np
import pytest

from gpu_util import oracle_all_orderings, u64
from helpers import mk_trace
from traces import make_config, make_orderings, random_trace, tile_in_time

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lap():
    import torch
    assert torch.cuda.is_available()
    import paper_1903_06631_amd as lap
    lap.load_library()
    return lap


def _check_load(lap, oracle, tr):
    dt = lap.DeviceTrace(tr)
    got = lap.load_profile(dt)
    load, peak, tpk = oracle.load_profile(tr)
    assert np.array_equal(u64(got["load"]), load)
    assert int(u64(got["peak"])[0]) == peak
    assert int(got["t_peak"].item()) == tpk
    return dt, got


@pytest.mark.parametrize("seed,n,T", [(0, 1, 1), (1, 7, 3), (2, 1000, 64), (3, 5000, 257), (4, 70001, 4099),
                                      (5, 30000, 9000), (6, 200000, 20000), (7, 63, 8192), (8, 65, 8191)])
def test_load_profile_random(lap, oracle_mod, seed, n, T):
    tr = random_trace(seed, n, T, size_choices=[1, 2, 3, 1000, 77777] if seed % 2 else None)
    _check_load(lap, oracle_mod, tr)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_load_profile_configs(lap, oracle_mod, cfg):
    _check_load(lap, oracle_mod, make_config(cfg))


def test_load_profile_tiled_long_timeline(lap, oracle_mod):
    # many iterations back to back: long time line, time-local chunks (the stress layout)
    tr = tile_in_time(make_config(3), 40)
    _check_load(lap, oracle_mod, tr)


@pytest.mark.parametrize("T", [32767, 32768, 32769, 100003, 4096 * 31 + 1])
def test_load_profile_long_time_lines(lap, oracle_mod, T):
    """time lines of 8 or more scan tiles take the multi-launch scan; equal peaks in different tiles"""
    tr = random_trace(40 + T % 7, 20000, T, max_life=T // 3)
    _check_load(lap, oracle_mod, tr)
    n = 40
    starts = [(k * (T - 2)) // (n - 1) for k in range(n)]                 # the same load at n far-apart steps
    tr = mk_trace([4096] * n, starts, [s + 1 for s in starts], T=T)
    dt, got = _check_load(lap, oracle_mod, tr)
    assert int(got["t_peak"].item()) == 0
    tr = mk_trace([4096] * n + [1], starts + [T - 1], [s + 1 for s in starts] + [T], T=T)
    tr.size[n // 2] += 512                                                # a single higher peak in the middle
    _check_load(lap, oracle_mod, tr)


def test_load_profile_peak_ties_and_extremes(lap, oracle_mod):
    tr = mk_trace([512, 512, 512], [0, 2, 4], [1, 3, 5], T=6)          # three equal peaks -> earliest
    _check_load(lap, oracle_mod, tr)
    tr = mk_trace([(1 << 53) - 1, (1 << 53) - 1, 1], [0, 0, 1], [2, 1, 2], T=2)   # largest legal sizes
    _check_load(lap, oracle_mod, tr)


def _check_plan(lap, oracle, tr, kinds, seeds, explicit_np=None, which=None, fits=None):
    import torch
    dt = lap.DeviceTrace(tr)
    explicit = None
    if explicit_np:
        explicit = {b: torch.from_numpy(p.astype(np.uint32).view(np.int32)).to(dt.device)
                    for b, p in explicit_np.items()}
    got = lap.plan_pool(dt, kinds, seeds, explicit=explicit, fits=fits)
    ref = oracle_all_orderings(oracle, tr, kinds, seeds, explicit_np, which, fits)
    all_off = u64(got["all_offsets"])
    fps = u64(got["footprints"])
    for b, (_, off, fp) in ref.items():
        assert np.array_equal(all_off[b], off), f"ordering {b} kind {kinds[b]}"
        assert fps[b] == fp, f"ordering {b}"
    # properties that hold for every ordering, whatever was sampled
    assert np.array_equal(fps, (all_off + tr.size[None, :]).max(axis=1))
    best = int(got["best_ordering"].item())
    assert best == int(np.argmin(fps)) and int(u64(got["best_footprint"])[0]) == int(fps.min())
    assert np.array_equal(u64(got["best_offsets"]), all_off[best])
    _, peak, _ = oracle.load_profile(tr)
    assert (fps >= peak).all()
    return got


@pytest.mark.parametrize("seed,n,T", [(0, 1, 1), (1, 2, 2), (2, 64, 5), (3, 65, 9), (4, 300, 12), (5, 511, 30),
                                      (6, 512, 30), (7, 513, 7), (8, 1500, 40), (9, 2600, 90)])
def test_plan_pool_random(lap, oracle_mod, seed, n, T):
    # coarse steps and repeated sizes force ties in every key; n spans the 512-entry
    # recent list and several merges
    tr = random_trace(50 + seed, n, T, size_choices=[1, 1, 2, 3, 5, 8, 13, 64])
    kinds, seeds = make_orderings(24)
    _check_plan(lap, oracle_mod, tr, kinds, seeds)


@pytest.mark.parametrize("seed,n,T,frac,max_life", [
    (0, 3000, 40, 0.97, 40),      # per-step lists, tails of a few entries
    (1, 5000, 64, 0.90, 8),       # many short multi-step variables
    (2, 4000, 2, 0.80, 2),        # ~2000 blocks per step: lists too long for registers
    (3, 2000, 7, 1.00, 1),        # one-step variables only
    (4, 6000, 300, 0.99, 300),    # few long-lived among many temporaries (transformer-like)
    (5, 1400, 1, 1.00, 1),        # a single step, 1400 one-step variables
    (6, 5000, 3, 0.45, 3),        # > 1000 multi-step blocks per step: hole lists too long for registers
    (7, 3000, 9, 0.50, 3),        # many splits: multi-step blocks land inside holes
    (8, 30000, 70000, 0.98, 50),  # more than 65535 steps: 64-bit lifetime words with per-step lists
    (9, 30000, 3000, 0.999, 3000),  # lifetimes of thousands of steps: more steps per thread than the kernel keeps notes for
])
def test_plan_pool_per_step_lists(lap, oracle_mod, seed, n, T, frac, max_life):
    """Traces whose lifetimes sum to at most 6N steps take the per-step-list path."""
    tr = random_trace(1000 + seed, n, T, size_choices=[1, 1, 2, 3, 5, 8, 13, 64], one_step_frac=frac,
                      max_life=max_life)
    assert int((tr.free - tr.alloc).sum()) + T <= 6 * n
    kinds, seeds = make_orderings(20 if n < 20000 else 8)
    _check_plan(lap, oracle_mod, tr, kinds, seeds)


@pytest.mark.parametrize("seed,n,T,frac,max_life,sizes", [
    (0, 6000, 40, 0.95, 3, [1]),                       # every hole an exact fit for the next variable: holes used up all the time
    (1, 9000, 12, 0.99, 2, [1, 2]),                    # few steps: long runs of one step's variables in every ordering
    (2, 12000, 60, 0.8, 6, [1, 1, 2, 3, 5, 8, 13, 64]),  # lists of more than 64 holes: fits beyond the first 64
    (3, 4000, 1, 1.0, 2, [1, 3, 7]),                   # one step: one list, one wave
    (4, 8000, 300, 0.9, 10, [7, 9, 100, 1000]),
])
def test_plan_pool_one_step_short_path(lap, oracle_mod, seed, n, T, frac, max_life, sizes):
    """The one-step variables' short path (the first 64 holes of the step's list in registers, one entry
    stored) and what it hands to the full path: holes used up, no fit among the first 64, runs of one step's
    variables (the alloc-ascending order places whole steps from the registers), blocks of multi-step variables
    taken out of the top holes at once or left in the tails."""
    tr = random_trace(1700 + seed, n, T, size_choices=sizes, one_step_frac=frac, max_life=max_life)
    assert int((tr.free.astype(np.int64) - tr.alloc).sum()) + tr.n_steps <= 6 * tr.n_vars     # per-step lists in use
    kinds, seeds = make_orderings(12)
    kinds = kinds.copy(); kinds[6] = 6
    _check_plan(lap, oracle_mod, tr, kinds, seeds)
    _check_plan(lap, oracle_mod, tr, kinds[:6], seeds[:6], fits=[b % 2 for b in range(6)])


def test_plan_pool_64bit_offsets(lap, oracle_mod):
    """Sizes whose sum does not fit 2^32 granules take the 64-bit path."""
    tr = random_trace(31, 900, 25, granule=1)
    tr.size = tr.size * np.uint64(1 << 20) + np.uint64(1)        # odd sizes: granule 1 byte, sum ~ 2^42
    assert int(tr.size.sum()) >= 1 << 32
    kinds, seeds = make_orderings(12)
    _check_plan(lap, oracle_mod, tr, kinds, seeds)


def test_plan_pool_wide_sizes(lap, oracle_mod):
    tr = random_trace(99, 1200, 50, granule=1)          # byte-granular sizes 2^9 .. 2^23
    kinds, seeds = make_orderings(16)
    _check_plan(lap, oracle_mod, tr, kinds, seeds)


def test_plan_pool_explicit_permutations(lap, oracle_mod):
    tr = random_trace(7, 700, 20, size_choices=[1, 2, 3, 4])
    rng = np.random.default_rng(5)
    explicit = {0: rng.permutation(700).astype(np.uint32), 2: np.arange(700, dtype=np.uint32)[::-1].copy()}
    kinds = np.array([5, 0, 5, 4], np.uint32)
    seeds = np.array([0, 0, 0, 99], np.uint64)
    _check_plan(lap, oracle_mod, tr, kinds, seeds, explicit_np=explicit)


def test_plan_pool_malformed_explicit_is_identity(lap, oracle_mod):
    import torch
    tr = random_trace(8, 500, 15, size_choices=[1, 2, 3, 4], one_step_frac=0.9, max_life=4)
    bad1 = np.arange(500, dtype=np.uint32); bad1[7] = 9            # index 9 twice, 7 missing
    bad2 = np.arange(500, dtype=np.uint32)[::-1].copy(); bad2[0] = 1 << 30   # out of range
    dt = lap.DeviceTrace(tr)
    ex = {b: torch.from_numpy(p.view(np.int32)).to(dt.device) for b, p in {0: bad1, 1: bad2}.items()}
    got = lap.plan_pool(dt, [5, 5, 0], [0, 0, 0], explicit=ex)
    ident = oracle_mod.place(tr, np.arange(500, dtype=np.uint32))
    for b in (0, 1):
        assert np.array_equal(u64(got["all_offsets"])[b], ident[0]) and u64(got["footprints"])[b] == ident[1]


@pytest.mark.parametrize("n,T,B", [(64, 9, 1), (128, 3, 3), (9000, 60, 12), (50, 100000, 4)])
def test_plan_pool_shapes(lap, oracle_mod, n, T, B):
    """Window-sized inputs, a single ordering, more than one 4096-entry merge, a very long time line."""
    tr = random_trace(n + T, n, T, size_choices=[1, 2, 3, 5, 8, 300])
    kinds, seeds = make_orderings(max(B, 5))
    _check_plan(lap, oracle_mod, tr, kinds[-B:], seeds[-B:])


def test_plan_pool_seeded_orders_with_equal_leading_key_bits(lap, oracle_mod):
    # 70 000 variables: about 150 pairs of seeded keys agree in their top 24 bits, the part the
    # radix sort looks at; the order inside such runs must come from the full keys
    tr = random_trace(77, 70000, 3000, max_life=3, one_step_frac=0.9)
    seeds = [5, 1 << 40, 631]
    keys = np.array([[oracle_mod.mix64(s, i) >> 40 for i in range(tr.n_vars)] for s in seeds[:1]])
    assert len(np.unique(keys[0])) < tr.n_vars          # there are such runs
    _check_plan(lap, oracle_mod, tr, [4, 4, 4], seeds)


@pytest.mark.parametrize("seed,n,T", [(0, 1, 1), (1, 2, 2), (2, 65, 3), (3, 300, 12), (4, 4097, 9), (5, 20000, 40),
                                      (6, 70000, 3000)])
def test_orders_themselves(lap, oracle_mod, seed, n, T):
    """the orders (not only the offsets they lead to) against the oracle's, rank by rank: every kind, ties in
    the fixed kinds' keys (few steps, few sizes) kept in ascending index order, seeded keys that agree in the
    bits the radix passes look at, an explicit order passed through"""
    import torch
    sizes = [1, 1, 2, 3, 5, 8, 13, 64, 1 << 20, (1 << 33) + 5] if seed % 2 else None
    kw = dict(max_life=3, one_step_frac=0.9) if n > 10000 else {}
    tr = random_trace(4400 + seed, n, T, size_choices=sizes, **kw)
    kinds = [0, 1, 2, 3, 4, 6, 4, 6, 5, 4]
    seeds = [0, 0, 0, 0, 5, 77, 1 << 40, 631, 0, 2 ** 64 - 1]
    rng = np.random.default_rng(seed)
    mine = rng.permutation(n).astype(np.uint32)
    dt = lap.DeviceTrace(tr)
    explicit = {8: torch.from_numpy(mine.view(np.int32)).to(dt.device)}
    lap.plan_pool(dt, kinds, seeds, explicit=explicit, want_all=False)
    got = lap.plan_pool_orders(dt, len(kinds)).cpu().numpy().view(np.uint32)
    for b, (k, s) in enumerate(zip(kinds, seeds)):
        want = mine if k == 5 else oracle_mod.make_perm(tr, k, s)
        assert np.array_equal(got[b], np.asarray(want, dtype=np.uint32)), f"ordering {b} kind {k}"


@pytest.mark.parametrize("n", [2, 63, 64, 65, 127, 253, 257, 4095, 4096, 4097, 8193])
def test_plan_pool_orders_around_wave_and_tile_sizes(lap, oracle_mod, n):
    """every kind of order with the variable count at, just below and just above what a wave (64 ranks;
    63 in the pass over runs of equal sorted bits), a workgroup (256) and a tile of the sort (4096) take;
    few steps and few sizes, so most keys of the fixed kinds tie, and sizes whose keys differ only in
    high bits next to ones that differ only in low bits"""
    kinds = [0, 1, 2, 3, 4, 6, 4, 6]
    seeds = [631 + 7 * b for b in range(len(kinds))]
    for T, sizes in ((3, [1, 2]), (40, [1, 1, 2, 3, 5, 8, 13, 64, 1 << 20, (1 << 33) + 5])):
        tr = random_trace(9000 + n, n, T, size_choices=sizes, one_step_frac=0.3)
        _check_plan(lap, oracle_mod, tr, kinds, seeds)


@pytest.mark.parametrize("seed,n,T", [(0, 1, 1), (1, 300, 12), (2, 5000, 60), (3, 70000, 3000)])
def test_plan_pool_class_seeded_orders(lap, oracle_mod, seed, n, T):
    """shuffles inside size classes (kind 6), both fit policies"""
    kw = dict(max_life=3, one_step_frac=0.9) if n > 10000 else {}
    tr = random_trace(1500 + seed, n, T, **kw)
    B = 3 if n > 10000 else 8
    _check_plan(lap, oracle_mod, tr, [6] * B, [77 + b for b in range(B)], fits=[b % 2 for b in range(B)])


def _mixed(B):
    """first-fit and best-fit orderings side by side, all six kinds of order"""
    kinds = [b % 5 for b in range(B)]
    seeds = [631 + b for b in range(B)]
    fits = [(b // 5 + b) % 2 for b in range(B)]
    return kinds, seeds, fits


def test_best_fit_golden(lap, oracle_mod):
    from helpers import read_golden
    g = read_golden("e4_best_fit.txt")
    tr = mk_trace([int(x) * 512 for x in g["size"][0]], g["alloc"][0], g["free"][0], T=3)
    import torch
    ident = torch.arange(9, dtype=torch.int32, device="cuda")
    dt = lap.DeviceTrace(tr)
    got = lap.plan_pool(dt, [5, 5], [0, 0], explicit={0: ident, 1: ident}, fits=[0, 1])
    off = u64(got["all_offsets"]) // 512
    assert off[0].tolist() == [int(x) for x in g["first_fit"][0]]
    assert off[1].tolist() == [int(x) for x in g["best_fit"][0]]
    assert u64(got["footprints"]).tolist() == [14 * 512, 12 * 512] and int(got["best_ordering"].item()) == 1


@pytest.mark.parametrize("seed,n,T", [(0, 1, 1), (1, 2, 2), (2, 64, 5), (3, 65, 9), (4, 300, 12), (5, 511, 30),
                                      (6, 1000, 64), (7, 2500, 200), (8, 4097, 33)])
def test_best_fit_random(lap, oracle_mod, seed, n, T):
    tr = random_trace(1200 + seed, n, T)
    kinds, seeds, fits = _mixed(20)
    _check_plan(lap, oracle_mod, tr, kinds, seeds, fits=fits)


@pytest.mark.parametrize("seed,n,T,frac,max_life", [
    (0, 3000, 40, 0.9, 6), (1, 8000, 100, 0.95, 30), (2, 20000, 64, 0.98, 64), (3, 6000, 500, 0.8, 4),
    (4, 5000, 12, 0.99, 12), (5, 9000, 70000, 0.9, 3),
    (6, 30000, 3000, 0.999, 3000)])      # lifetimes beyond the steps a thread keeps notes for
def test_best_fit_per_step_lists(lap, oracle_mod, seed, n, T, frac, max_life):
    """mostly one-step variables (hole lists in use), a few long-lived ones that walk the holes"""
    tr = random_trace(1300 + seed, n, T, max_life=max_life, one_step_frac=frac)
    kinds, seeds, fits = _mixed(10)
    _check_plan(lap, oracle_mod, tr, kinds, seeds, fits=fits)


def test_best_fit_64bit_offsets(lap, oracle_mod):
    tr = random_trace(1400, 700, 20, granule=1, max_life=10)
    tr.size = tr.size * np.uint64(1 << 20) + np.uint64(1)        # odd sizes: the 64-bit kernel runs
    assert int(tr.size.sum()) >= 1 << 32
    kinds, seeds, fits = _mixed(10)
    _check_plan(lap, oracle_mod, tr, kinds, seeds, fits=fits)


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_best_fit_configs(lap, oracle_mod, cfg):
    tr = make_config(cfg)
    kinds, seeds = make_orderings(16)
    _check_plan(lap, oracle_mod, tr, kinds, seeds, fits=[1] * 16)
    _check_plan(lap, oracle_mod, tr, kinds, seeds, fits=[b % 2 for b in range(16)])


def test_plan_pool_special_cases(lap, oracle_mod):
    kinds, seeds = make_orderings(8)
    # identical lifetimes: blocks stack, footprint = sum of sizes
    tr = mk_trace([512 * (1 + k % 7) for k in range(600)], [1] * 600, [4] * 600, T=5)
    got = _check_plan(lap, oracle_mod, tr, kinds, seeds)
    assert (u64(got["footprints"]) == int(tr.size.sum())).all()
    # disjoint lifetimes: every offset 0
    tr = mk_trace([512 * (1 + k % 5) for k in range(300)], list(range(300)), list(range(1, 301)))
    got = _check_plan(lap, oracle_mod, tr, kinds, seeds)
    assert not u64(got["all_offsets"]).any()
    # largest legal sizes
    tr = mk_trace([(1 << 53) - 1, 1 << 52, 12345], [0, 0, 0], [1, 1, 1])
    _check_plan(lap, oracle_mod, tr, kinds, seeds)


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_plan_pool_configs(lap, oracle_mod, cfg):
    tr = make_config(cfg)
    kinds, seeds = make_orderings(tr.meta["B"])
    _check_plan(lap, oracle_mod, tr, kinds, seeds)


def _check_scores(lap, oracle, tr, link, min_bytes, use_gaps=True, pass_load=True):
    dt = lap.DeviceTrace(tr, use_gaps=use_gaps)
    load = lap.load_profile(dt)["load"] if pass_load else None
    got = lap.score_swaps(dt, link, min_bytes, load=load)
    ref = oracle.score_swaps(tr, link, min_bytes, use_gaps=use_gaps)
    assert np.array_equal(got["candidate"].cpu().numpy(), ref["candidate"])
    assert np.array_equal(got["doa_ns"].cpu().numpy(), ref["doa_ns"])
    assert np.array_equal(got["aoa"].cpu().numpy().view(np.uint64), ref["aoa"].view(np.uint64))
    assert np.array_equal(u64(got["wdoa"]), ref["wdoa"])
    assert np.array_equal(u64(got["peak_cut"]), ref["peak_cut"])


@pytest.mark.parametrize("seed,n,T,link", [(0, 1, 1, 64.0), (1, 5, 2, 64.0), (2, 300, 17, 64.0), (3, 5000, 300, 0.5),
                                           (4, 20000, 1025, 12.345), (5, 3000, 5000, 900.0), (6, 777, 33, 1e-3)])
def test_score_swaps_random(lap, oracle_mod, seed, n, T, link):
    tr = random_trace(700 + seed, n, T, with_step_ns=(seed % 2 == 0))
    _check_scores(lap, oracle_mod, tr, link, 1 << 14, use_gaps=True, pass_load=(seed % 3 != 0))
    _check_scores(lap, oracle_mod, tr, link, 1 << 14, use_gaps=False)


@pytest.mark.parametrize("cfg", [1, 3, 5])
def test_score_swaps_configs(lap, oracle_mod, cfg):
    tr = make_config(cfg)
    _check_scores(lap, oracle_mod, tr, tr.meta["link_GBps"], tr.meta["min_bytes"])


def test_validate_trace(lap, oracle_mod):
    """Every documented rule with its exact status (the table of helpers.validate_cases, which the
    oracle is pinned to as well)."""
    from helpers import validate_cases
    for name, t, status in validate_cases():
        assert oracle_mod.validate_trace(t) == status, name
        assert lap.validate_trace(lap.DeviceTrace(t)) == status, name


def test_profile_ordering_ms(lap, oracle_mod):
    """The per-ordering durations of the last launch: one positive value per ordering, none longer than the launch."""
    tr = make_config(2)
    kinds, seeds = make_orderings(tr.meta["B"])
    dt = lap.DeviceTrace(tr)
    lap.profile_enable(True)
    lap.plan_pool(dt, kinds, seeds, fits=[b % 2 for b in range(len(kinds))])
    ms = lap.profile_ordering_ms(dt, len(kinds))
    launch = lap.profile_last_ms(lap.K_PLACE)
    lap.profile_enable(False)
    assert ms.shape == (len(kinds),) and (ms > 0).all() and ms.max() <= launch * 1.05 + 0.05
