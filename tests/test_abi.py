"""Host-only checks of the C ABI: exported symbols, status strings, argument validation.

None of these reaches a HIP call: every error below is detected before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lap():
    import paper_1903_06631_amd as lap
    if not os.path.exists(lap.lib_path()):
        from paper_1903_06631_amd import build
        build.build()
    lap.load_library()
    return lap


def test_every_declared_symbol_is_exported(lap):
    hdr = open(os.path.join(ROOT, "include", "lap.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(lap_[a-z_]+)\s*\(", hdr))
    assert {"lap_load_profile", "lap_plan_pool", "lap_score_swaps", "lap_select_swaps", "lap_detect_iteration", "lap_schedule_swaps", "lap_simulate_swaps", "lap_evaluate_weights",
            "lap_workspace_bytes",
            "lap_validate_trace", "lap_status_string"} <= declared
    lib = lap.load_library()
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lap):
    seen = {lap.status_string(s) for s in range(0, -9, -1)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert lap.status_string(-99) == "unknown status"


def test_workspace_sizes(lap):
    assert lap.workspace_bytes(0, 100, 22) >= 23 * 8
    assert lap.workspace_bytes(1, 120, 22, 16) >= 16 * 120 * (4 + 8)
    assert lap.workspace_bytes(2, 120, 22) >= 6 * 23 * 8
    assert lap.workspace_bytes(3, 1, 1) > 0
    assert lap.workspace_bytes(4, 120, 22, 2) > lap.workspace_bytes(4, 120, 22, 1) > lap.workspace_bytes(2, 120, 22)
    assert lap.workspace_bytes(42, 1, 1) == 0
    assert lap.workspace_bytes(1, 120, 22, 32) > lap.workspace_bytes(1, 120, 22, 16)


def test_argument_errors(lap):
    from paper_1903_06631_amd.binding import _Ordering, _Trace
    lib = lap.load_library()
    fake = 0x1000   # never dereferenced: all of these fail in the host-side checks
    good = _Trace(4, 3, fake, fake, fake, None, None, None)
    ords = (_Ordering * 2)()
    ords[0].kind, ords[1].kind = 0, 4

    # NULL pointers
    assert lib.lap_load_profile(None, fake, fake, fake, fake, 1 << 20, None) == -1
    assert lib.lap_load_profile(C.byref(good), None, fake, fake, fake, 1 << 20, None) == -1
    assert lib.lap_load_profile(C.byref(_Trace(4, 3, None, fake, fake, None, None, None)),
                                fake, fake, fake, fake, 1 << 20, None) == -1
    assert lib.lap_load_profile(C.byref(_Trace(4, 3, fake, fake, fake, fake, None, None)),
                                fake, fake, fake, fake, 1 << 20, None) == -1   # only one of the gap arrays
    assert lib.lap_plan_pool(C.byref(good), None, 2, fake, fake, fake, None, None, fake, 1 << 30, None) == -1
    assert lib.lap_plan_pool(C.byref(good), ords, 2, None, fake, fake, None, None, fake, 1 << 30, None) == -1
    assert lib.lap_score_swaps(C.byref(good), 64.0, 1, None, None, fake, fake, fake, fake, fake, 1 << 20, None) == -1
    # sizes
    assert lib.lap_load_profile(C.byref(_Trace(0, 3, fake, fake, fake, None, None, None)),
                                fake, fake, fake, fake, 1 << 20, None) == -2
    assert lib.lap_load_profile(C.byref(_Trace(4, 0, fake, fake, fake, None, None, None)),
                                fake, fake, fake, fake, 1 << 20, None) == -2
    assert lib.lap_plan_pool(C.byref(good), ords, 0, fake, fake, fake, None, None, fake, 1 << 30, None) == -2
    # workspace: NULL, misaligned, too small
    assert lib.lap_load_profile(C.byref(good), fake, fake, fake, None, 1 << 20, None) == -3
    assert lib.lap_load_profile(C.byref(good), fake, fake, fake, fake + 8, 1 << 20, None) == -3
    assert lib.lap_load_profile(C.byref(good), fake, fake, fake, fake, 8, None) == -3
    need = lap.workspace_bytes(1, 4, 3, 2)
    assert lib.lap_plan_pool(C.byref(good), ords, 2, fake, fake, fake, None, None, fake, need - 1, None) == -3
    # orderings
    ords[1].kind = 7
    assert lib.lap_plan_pool(C.byref(good), ords, 2, fake, fake, fake, None, None, fake, 1 << 30, None) == -4
    ords[1].kind, ords[1].seed = 5, 0
    assert lib.lap_plan_pool(C.byref(good), ords, 2, fake, fake, fake, None, None, fake, 1 << 30, None) == -4
    ords[1].kind, ords[1].fit = 4, 2        # unknown fit policy
    assert lib.lap_plan_pool(C.byref(good), ords, 2, fake, fake, fake, None, None, fake, 1 << 30, None) == -4
    ords[1].fit = 0
    # link
    for link in (0.0, -3.0, float("nan"), float("inf"), 1e-9):
        assert lib.lap_score_swaps(C.byref(good), link, 1, None, fake, fake, fake, fake, fake,
                                   fake, 1 << 20, None) == -5

    # selection: NULL outputs, sizes, score kinds, link, workspace
    kinds = (C.c_uint32 * 2)(3, 0)
    lims = (C.c_uint64 * 1)(5)
    sel = lambda **kw: lib.lap_select_swaps(
        C.byref(good), kw.get("link", 64.0), 1, None, kw.get("kinds", kinds), kw.get("K", 2), kw.get("lims", lims),
        kw.get("L", 1), kw.get("order", fake), None, fake, fake, kw.get("nsel", fake), fake, fake, fake,
        kw.get("ws", 1 << 30), None)
    assert sel(order=None) == -1 and sel(kinds=None) == -1 and sel(lims=None) == -1 and sel(nsel=None) == -1
    assert sel(K=0) == -2 and sel(K=65) == -2 and sel(L=1025) == -2
    assert sel(kinds=(C.c_uint32 * 2)(3, 5)) == -4
    assert sel(link=0.0) == -5
    assert sel(ws=lap.workspace_bytes(4, 4, 3, 2) - 1) == -3

    # swap schedule
    sch = lambda **kw: lib.lap_schedule_swaps(C.byref(good), kw.get("link", 1.0), None, kw.get("lst", fake), kw.get("k", 2),
                                              fake, fake, fake, fake, kw.get("load", fake), fake, fake, fake,
                                              kw.get("ws", 1 << 30), None)
    assert sch(lst=None) == -1 and sch(load=None) == -1 and sch(k=5) == -2 and sch(link=-1.0) == -5
    assert sch(ws=lap.workspace_bytes(6, 4, 3) - 1) == -3
    # schedule under a limit
    pl = (C.c_uint32 * 2)(1, 2)
    lm = (C.c_uint64 * 2)(10, 20)
    sim = lambda **kw: lib.lap_simulate_swaps(C.byref(good), kw.get("link", 1.0), fake, kw.get("k", 2), kw.get("pl", pl),
                                              lm, kw.get("Q", 2), kw.get("out", fake), fake, fake, fake, fake,
                                              kw.get("ws", 1 << 30), None)
    assert sim(pl=None) == -1 and sim(out=None) == -1 and sim(Q=0) == -2 and sim(Q=5000) == -2 and sim(k=1) == -2
    assert sim(link=0.0) == -5 and sim(ws=lap.workspace_bytes(7, 4, 3, 2) - 1) == -3
    # weight vectors
    wv = (C.c_double * 8)(1, 0, 0, 0, 0, 1, 0, 0)
    ew = lambda **kw: lib.lap_evaluate_weights(C.byref(good), kw.get("link", 1.0), 1, None, kw.get("wv", wv), kw.get("W", 2),
                                               5, kw.get("order", fake), fake, fake, fake, fake, fake, fake, fake, fake,
                                               kw.get("ws", 1 << 30), None)
    assert ew(wv=None) == -1 and ew(order=None) == -1 and ew(W=0) == -2 and ew(W=65) == -2 and ew(link=0.0) == -5
    assert ew(wv=(C.c_double * 8)(1, 0, 0, float("inf"), 0, 1, 0, 0)) == -4
    assert ew(ws=lap.workspace_bytes(8, 4, 3, 2) - 1) == -3
    # iteration detection
    assert lib.lap_detect_iteration(None, 8, 1, fake, fake, 1 << 20, None) == -1
    assert lib.lap_detect_iteration(fake, 0, 1, fake, fake, 1 << 20, None) == -2
    assert lib.lap_detect_iteration(fake, 8, 0, fake, fake, 1 << 20, None) == -2
    assert lib.lap_detect_iteration(fake, 8, 1, fake, fake, 8, None) == -3


def test_no_cpu_fallback(lap, monkeypatch, tmp_path):
    """A missing library is an import-time error, never a silent CPU path."""
    from paper_1903_06631_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.load_library()


def test_product_never_imports_oracle():
    pkg = os.path.join(ROOT, "paper_1903_06631_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt.lower() or f == "__init__.py" and "oracle" not in txt, (dirpath, f)


def test_static_entry_point_rejects_on_the_host(lap):
    """lap_load_profile_static: NULL arguments and time lines beyond its fixed scratch are refused
    before any HIP call."""
    from paper_1903_06631_amd.binding import STATIC_MAX_STEPS, _Trace
    lib = lap.load_library()
    fake = 0x1000
    hdr = open(os.path.join(ROOT, "include", "lap.h")).read()
    assert int(re.search(r"#define LAP_STATIC_MAX_STEPS \(1u << (\d+)\)", hdr).group(1)) == STATIC_MAX_STEPS.bit_length() - 1
    assert lib.lap_load_profile_static(None, fake, fake, fake, None) == -1
    ok = _Trace(4, 3, fake, fake, fake, None, None, None)
    assert lib.lap_load_profile_static(C.byref(ok), None, fake, fake, None) == -1
    long_ = _Trace(4, STATIC_MAX_STEPS + 1, fake, fake, fake, None, None, None)
    assert lib.lap_load_profile_static(C.byref(long_), fake, fake, fake, None) == -2
    assert lib.lap_load_profile_static(C.byref(_Trace(0, 3, fake, fake, fake, None, None, None)), fake, fake, fake, None) == -2


def test_options_and_ordering_durations_reject_on_the_host(lap):
    """lap_set_option refuses unknown options and values; lap_profile_ordering_ms checks its arguments before
    it touches the device."""
    import numpy as np
    lib = lap.load_library()
    assert lib.lap_set_option(99, 1) == -4
    assert lib.lap_set_option(1, 1 << 40) == -4                       # rounds, times 100: 32 bits
    assert lib.lap_set_option(0, lap.SEG_MIN_VARS_DEFAULT) == 0 and lib.lap_set_option(1, lap.SEG_TRIAL_PERCENT_DEFAULT) == 0
    out = np.zeros(4, np.float32)
    p = out.ctypes.data_as(C.c_void_p)
    fake = 0x1000
    assert lib.lap_profile_ordering_ms(10, 5, 4, fake, 1 << 30, None, None) == -1
    assert lib.lap_profile_ordering_ms(0, 5, 4, fake, 1 << 30, None, p) == -2
    assert lib.lap_profile_ordering_ms(10, 5, 4, None, 1 << 30, None, p) == -3
    assert lib.lap_profile_ordering_ms(10, 5, 4, fake, 16, None, p) == -3             # workspace too small
    assert lib.lap_profile_ordering_ms(10, 5, 4, fake + 8, 1 << 30, None, p) == -3    # misaligned
    # lap_plan_pool_orders: the same workspace checks, before anything is enqueued
    assert lib.lap_plan_pool_orders(10, 5, 4, fake, 1 << 30, None, None) == -1
    assert lib.lap_plan_pool_orders(10, 0, 4, fake, 1 << 30, None, fake) == -2
    assert lib.lap_plan_pool_orders(10, 5, 0, fake, 1 << 30, None, fake) == -2
    assert lib.lap_plan_pool_orders(10, 5, 4, None, 1 << 30, None, fake) == -3
    assert lib.lap_plan_pool_orders(10, 5, 4, fake, 16, None, fake) == -3
    assert lib.lap_plan_pool_orders(10, 5, 4, fake + 8, 1 << 30, None, fake) == -3
