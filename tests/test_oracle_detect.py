"""Pins for the oracle's iteration detection (Section V: the request list ends with two equal
consecutive subsequences)."""
import numpy as np
import pytest

from traces import make_config, random_trace
from traces.requests import iteration_tokens, request_stream


def z_function(s):
    """Textbook Z-algorithm: z[i] = length of the longest common prefix of s and s[i:]."""
    n = len(s)
    z = [0] * n
    z[0] = n
    l = r = 0
    for i in range(1, n):
        if i < r:
            z[i] = min(r - i, z[i - l])
        while i + z[i] < n and s[z[i]] == s[i + z[i]]:
            z[i] += 1
        if i + z[i] > r:
            l, r = i, i + z[i]
    return z


def period_by_z(tokens, min_period):
    """The list ends with a square of half-length p  <=>  the reversed list starts with one
    <=>  z_reversed[p] >= p."""
    rev = list(tokens[::-1])
    z = z_function(rev)
    for p in range(min_period, len(rev) // 2 + 1):
        if z[p] >= p:
            return p
    return 0


def test_tiny_cases(oracle_mod):
    d = oracle_mod.detect_iteration
    assert d([7], 1) == 0
    assert d([7, 7], 1) == 1
    assert d([7, 8], 1) == 0
    assert d([1, 2, 3, 1, 2, 3], 1) == 3
    assert d([9, 1, 2, 3, 1, 2, 3], 1) == 3                 # warm-up request in front
    assert d([1, 2, 3, 1, 2, 3, 1], 1) == 3                 # one request into the next iteration
    assert d([1, 2, 1, 2, 5, 1, 2, 1, 2, 5], 1) == 5        # the inner repeat 1 2 1 2 is not at the end
    assert d([5, 1, 2, 1, 2, 5, 1, 2, 1, 2], 1) == 2        # ... here it is: smallest period wins
    assert d([5, 1, 2, 1, 2, 5, 1, 2, 1, 2], 3) == 5        # unless the caller asks for at least 3
    assert d([4, 4, 4, 4, 4, 4], 1) == 1 and d([4, 4, 4, 4, 4, 4], 2) == 2 and d([4, 4, 4, 4, 4, 4], 4) == 0
    assert d([1, 2, 3, 4, 1, 2, 3, 5], 1) == 0              # differs in the last request only


@pytest.mark.parametrize("seed", range(10))
def test_against_z_function(oracle_mod, seed):
    rng = np.random.default_rng(seed)
    alphabet = [2, 3, 5][seed % 3]                         # small alphabets: many accidental squares
    for _ in range(30):
        m = int(rng.integers(1, 200))
        s = rng.integers(0, alphabet, m).astype(np.uint64)
        if rng.random() < 0.5 and m >= 4:                  # plant a square at the end
            p = int(rng.integers(1, m // 2 + 1))
            s[m - p:] = s[m - 2 * p:m - p]
        for mp in (1, 2, 7):
            assert oracle_mod.detect_iteration(s, mp) == period_by_z(s, mp)


@pytest.mark.parametrize("cfg,iters,warm,tail", [(1, 2, 0, 0), (1, 3, 17, 5), (2, 2, 100, 0), (2, 4, 3, 999)])
def test_streams_from_traces(oracle_mod, cfg, iters, warm, tail):
    it = iteration_tokens(make_config(cfg))
    s = request_stream(it, iters, warm, tail % len(it), seed=cfg)
    p = oracle_mod.detect_iteration(s, 8)
    assert p == len(it)
    # the detected subsequence is a rotation of the iteration (exactly it when the tail is empty)
    got = s[len(s) - p:]
    k = tail % len(it)
    assert np.array_equal(np.roll(got, k), it)
    # one iteration alone is not enough
    assert oracle_mod.detect_iteration(request_stream(it, 1, warm, 0, seed=cfg), 8) == 0
