"""Pins for the oracle's trace validation: every documented rule with its exact status, both
sides of every threshold.  The expected statuses are written in helpers.validate_cases()."""
import pytest

from helpers import validate_cases

CASES = validate_cases()


@pytest.mark.parametrize("name,tr,status", CASES, ids=[c[0] for c in CASES])
def test_validate_status(oracle_mod, name, tr, status):
    assert oracle_mod.validate_trace(tr) == status


def test_cases_cover_every_rule():
    names = " | ".join(c[0] for c in CASES)
    for rule in ("size 0", "alloc == free", "alloc > free", "free > n_steps", "gap_lo below", "gap_hi above",
                 "gap_lo above gap_hi", "step_ns 0", "size 2^53", "sum of step_ns", "sizes of 2^53 - 1",
                 "size 2^52 over 4096"):
        assert rule in names
    assert {c[2] for c in CASES} == {0, -6, -7}
