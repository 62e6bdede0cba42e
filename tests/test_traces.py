"""The synthetic trace generator: shapes, determinism, structure."""
import numpy as np
import pytest

from traces import make_config, make_orderings, random_trace, tile_in_time

SHAPES = {1: (120, 22, 16), 2: (600, 42, 256), 3: (3000, 348, 1024)}


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_shapes_and_rules(cfg):
    tr = make_config(cfg)
    n, T, B = SHAPES[cfg]
    assert (tr.n_vars, tr.n_steps, tr.meta["B"]) == (n, T, B)
    assert (tr.size % 512 == 0).all() and (tr.size >= 512).all()
    assert (tr.alloc < tr.free).all() and (tr.free <= T).all()
    assert (tr.alloc <= tr.gap_lo).all() and (tr.gap_lo <= tr.gap_hi).all() and (tr.gap_hi <= tr.free - 1).all()
    one = tr.free - tr.alloc == 1
    assert (tr.gap_lo[one] == tr.gap_hi[one]).all()
    tr2 = make_config(cfg)
    assert all(np.array_equal(getattr(tr, k), getattr(tr2, k)) for k in ("size", "alloc", "free", "gap_lo", "gap_hi"))


def test_big_config_shapes():
    tr = make_config(4)
    assert (tr.n_vars, tr.n_steps) == (50_000, 14_000)


def test_orderings():
    kind, seed = make_orderings(16)
    assert kind.tolist() == [0, 1, 2, 3] + [4] * 12
    assert seed.tolist() == list(range(631, 647))


def test_tile_in_time():
    tr = random_trace(3, 50, 11)
    tt = tile_in_time(tr, 3)
    assert tt.n_vars == 150 and tt.n_steps == 33
    assert np.array_equal(tt.alloc[50:100], tr.alloc + 11)
    assert np.array_equal(tt.size[100:], tr.size)
