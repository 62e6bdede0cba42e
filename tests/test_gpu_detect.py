"""GPU parity: lap_detect_iteration against the oracle."""
import numpy as np
import pytest

from traces import make_config
from traces.requests import iteration_tokens, request_stream

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lap():
    import paper_1903_06631_amd as lap
    lap.load_library()
    return lap


def _run(lap, s, min_period):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(s, dtype=np.uint64).view(np.int64)).cuda()
    return int(lap.detect_iteration(t, min_period).item())


def test_detect_tiny(lap, oracle_mod):
    cases = [([7], 1), ([7, 7], 1), ([7, 8], 1), ([1, 2, 3, 1, 2, 3], 1), ([9, 1, 2, 3, 1, 2, 3], 1),
             ([1, 2, 3, 1, 2, 3, 1], 1), ([1, 2, 1, 2, 5, 1, 2, 1, 2, 5], 1), ([5, 1, 2, 1, 2, 5, 1, 2, 1, 2], 1),
             ([5, 1, 2, 1, 2, 5, 1, 2, 1, 2], 3), ([4] * 6, 1), ([4] * 6, 2), ([4] * 6, 4), ([1, 2, 3, 4, 1, 2, 3, 5], 1)]
    for s, mp in cases:
        assert _run(lap, s, mp) == oracle_mod.detect_iteration(s, mp), (s, mp)


@pytest.mark.parametrize("seed", range(6))
def test_detect_random_small_alphabet(lap, oracle_mod, seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(12):
        m = int(rng.integers(1, 5000))
        s = rng.integers(0, 2 + seed % 3, m).astype(np.uint64)
        if rng.random() < 0.6 and m >= 4:
            p = int(rng.integers(1, m // 2 + 1))
            s[m - p:] = s[m - 2 * p:m - p]
        for mp in (1, 3, 50):
            assert _run(lap, s, mp) == oracle_mod.detect_iteration(s, mp)


def test_detect_hash_collisions_do_not_matter(lap, oracle_mod):
    """Thue-Morse words are the classic way to make polynomial hashes mod 2^64 collide: the two
    halves below differ, and whatever the hashes say the answer must come from the tokens."""
    k = 13
    tm = np.array([bin(i).count("1") & 1 for i in range(1 << k)], dtype=np.uint64)
    s = np.concatenate([tm, 1 - tm])                       # no square of half-length 2^k at the end
    for mp in (1, 1 << (k - 1), 1 << k):
        assert _run(lap, s, mp) == oracle_mod.detect_iteration(s, mp)
    s = np.concatenate([tm, 1 - tm, tm, 1 - tm])
    assert _run(lap, s, 1 << k) == oracle_mod.detect_iteration(s, 1 << k) == 1 << (k + 1)


@pytest.mark.parametrize("cfg,iters,warm,tail,mp", [(1, 2, 0, 0, 8), (2, 3, 100, 77, 8), (3, 2, 1000, 0, 64),
                                                    (3, 5, 31, 4001, 64), (5, 2, 12345, 0, 1000)])
def test_detect_streams_from_traces(lap, oracle_mod, cfg, iters, warm, tail, mp):
    it = iteration_tokens(make_config(cfg))
    s = request_stream(it, iters, warm, tail % len(it), seed=cfg)
    p = _run(lap, s, mp)
    assert p == len(it) == oracle_mod.detect_iteration(s, mp)
    assert _run(lap, request_stream(it, 1, warm, 0, seed=cfg), mp) == 0


def test_detect_argument_errors(lap):
    import torch
    t = torch.zeros(8, dtype=torch.int64, device="cuda")
    with pytest.raises(lap.LapError) as e:
        lap.detect_iteration(t, 0)
    assert e.value.status == -2
