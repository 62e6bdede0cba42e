"""ctypes access to the plain CPU oracle (oracle/lap_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg.  The product package never imports this.
All arguments and results are numpy arrays in host memory.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lap_oracle.c")
_LIB = os.path.join(_HERE, "liblap_oracle.so")
_lib = None

u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
u64p = np.ctypeslib.ndpointer(np.uint64, flags="C_CONTIGUOUS")
i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.lapo_count_edges.restype = C.c_uint64
        _lib.lapo_mix64.restype = C.c_uint64
        _lib.lapo_mix64.argtypes = [C.c_uint64, C.c_uint32]
    return _lib


def _opt(arr, dtype):
    if arr is None:
        return None
    a = np.ascontiguousarray(arr, dtype=dtype)
    return a.ctypes.data_as(C.c_void_p)


def _c(arr, dtype):
    return np.ascontiguousarray(arr, dtype=dtype)


def load_profile(tr):
    lib = _load()
    T = tr.n_steps
    load = np.zeros(T, np.uint64)
    peak = C.c_uint64(0)
    tpk = C.c_uint32(0)
    rc = lib.lapo_load_profile(C.c_uint32(tr.n_vars), C.c_uint32(T),
                               _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32), _opt(tr.free, np.uint32),
                               load.ctypes.data_as(C.c_void_p), C.byref(peak), C.byref(tpk))
    if rc:
        raise RuntimeError(f"lapo_load_profile rc={rc}")
    return load, int(peak.value), int(tpk.value)


def count_edges(tr) -> int:
    lib = _load()
    return int(lib.lapo_count_edges(C.c_uint32(tr.n_vars), _opt(tr.alloc, np.uint32), _opt(tr.free, np.uint32)))


def validate_trace(tr, use_gaps=True) -> int:
    lib = _load()
    return int(lib.lapo_validate_trace(
        C.c_uint32(tr.n_vars), C.c_uint32(tr.n_steps),
        _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32), _opt(tr.free, np.uint32),
        _opt(tr.gap_lo if use_gaps else None, np.uint32), _opt(tr.gap_hi if use_gaps else None, np.uint32),
        _opt(tr.step_ns, np.uint64)))


def mix64(seed: int, i: int) -> int:
    return int(_load().lapo_mix64(C.c_uint64(seed & (2**64 - 1)), C.c_uint32(i)))


def make_perm(tr, kind: int, seed: int = 0, explicit=None):
    lib = _load()
    perm = np.zeros(tr.n_vars, np.uint32)
    ex = None if explicit is None else _c(explicit, np.uint32)
    rc = lib.lapo_make_perm(C.c_uint32(tr.n_vars), _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32),
                            _opt(tr.free, np.uint32), C.c_uint32(kind), C.c_uint64(seed),
                            None if ex is None else ex.ctypes.data_as(C.c_void_p),
                            perm.ctypes.data_as(C.c_void_p))
    if rc:
        raise RuntimeError(f"lapo_make_perm rc={rc}")
    return perm


def place(tr, perm, best_fit: bool = False):
    lib = _load()
    perm = _c(perm, np.uint32)
    off = np.zeros(tr.n_vars, np.uint64)
    fp = C.c_uint64(0)
    fn = lib.lapo_place_best if best_fit else lib.lapo_place
    rc = fn(C.c_uint32(tr.n_vars), _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32),
                        _opt(tr.free, np.uint32), perm.ctypes.data_as(C.c_void_p),
                        off.ctypes.data_as(C.c_void_p), C.byref(fp))
    if rc:
        raise RuntimeError(f"lapo_place rc={rc}")
    return off, int(fp.value)


def plan_pool(tr, kinds, seeds, explicit=None, want_all=True):
    """explicit: dict ordering index -> u32 permutation (for kind 5)."""
    lib = _load()
    kinds = _c(kinds, np.uint32)
    seeds = _c(seeds, np.uint64).copy()
    keep = []
    if explicit:
        for b, p in explicit.items():
            p = _c(p, np.uint32)
            keep.append(p)
            seeds[b] = p.ctypes.data
    B, n = len(kinds), tr.n_vars
    best_off = np.zeros(n, np.uint64)
    fps = np.zeros(B, np.uint64)
    all_off = np.zeros((B, n), np.uint64) if want_all else None
    bfp = C.c_uint64(0)
    bidx = C.c_uint32(0)
    rc = lib.lapo_plan_pool(C.c_uint32(n), _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32),
                            _opt(tr.free, np.uint32), C.c_uint32(B),
                            kinds.ctypes.data_as(C.c_void_p), seeds.ctypes.data_as(C.c_void_p),
                            best_off.ctypes.data_as(C.c_void_p), C.byref(bfp), C.byref(bidx),
                            fps.ctypes.data_as(C.c_void_p),
                            None if all_off is None else all_off.ctypes.data_as(C.c_void_p))
    if rc:
        raise RuntimeError(f"lapo_plan_pool rc={rc}")
    return dict(best_offsets=best_off, best_footprint=int(bfp.value), best_ordering=int(bidx.value),
                footprints=fps, all_offsets=all_off)


def score_swaps(tr, link_GBps: float, min_bytes: int, use_gaps=True, check=True):
    lib = _load()
    n = tr.n_vars
    cand = np.zeros(n, np.uint8)
    doa = np.zeros(n, np.int64)
    aoa = np.zeros(n, np.float64)
    wdoa = np.zeros(n, np.uint64)
    cut = np.zeros(n, np.uint64)
    rc = lib.lapo_score_swaps(
        C.c_uint32(n), C.c_uint32(tr.n_steps),
        _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32), _opt(tr.free, np.uint32),
        _opt(tr.gap_lo if use_gaps else None, np.uint32), _opt(tr.gap_hi if use_gaps else None, np.uint32),
        _opt(tr.step_ns, np.uint64), C.c_double(link_GBps), C.c_uint64(min_bytes),
        cand.ctypes.data_as(C.c_void_p), doa.ctypes.data_as(C.c_void_p), aoa.ctypes.data_as(C.c_void_p),
        wdoa.ctypes.data_as(C.c_void_p), cut.ctypes.data_as(C.c_void_p))
    if rc and check:
        raise RuntimeError(f"lapo_score_swaps rc={rc}")
    if rc:
        return rc
    return dict(candidate=cand, doa_ns=doa, aoa=aoa, wdoa=wdoa, peak_cut=cut)


def select_swaps(tr, link_GBps: float, min_bytes: int, score_kind: int, limits, use_gaps=True):
    lib = _load()
    n = tr.n_vars
    limits = _c(limits, np.uint64)
    L = len(limits)
    order = np.zeros(n, np.uint32)
    rank = np.zeros(n, np.uint32)
    peaks = np.zeros(n + 1, np.uint64)
    n_sel = np.zeros(max(L, 1), np.uint32)
    peak_after = np.zeros(max(L, 1), np.uint64)
    n_cand = C.c_uint32(0)
    load_min = C.c_uint64(0)
    rc = lib.lapo_select_swaps(
        C.c_uint32(n), C.c_uint32(tr.n_steps),
        _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32), _opt(tr.free, np.uint32),
        _opt(tr.gap_lo if use_gaps else None, np.uint32), _opt(tr.gap_hi if use_gaps else None, np.uint32),
        _opt(tr.step_ns, np.uint64), C.c_double(link_GBps), C.c_uint64(min_bytes), C.c_uint32(score_kind),
        limits.ctypes.data_as(C.c_void_p), C.c_uint32(L),
        order.ctypes.data_as(C.c_void_p), rank.ctypes.data_as(C.c_void_p), C.byref(n_cand),
        peaks.ctypes.data_as(C.c_void_p), n_sel.ctypes.data_as(C.c_void_p), peak_after.ctypes.data_as(C.c_void_p),
        C.byref(load_min))
    if rc:
        raise RuntimeError(f"lapo_select_swaps rc={rc}")
    nc = int(n_cand.value)
    return dict(order=order[:nc], rank=rank, n_cand=nc, peaks=peaks[:nc + 1], n_selected=n_sel[:L],
                peak_after=peak_after[:L], load_min=int(load_min.value))


def detect_iteration(tokens, min_period: int = 1) -> int:
    lib = _load()
    tokens = _c(tokens, np.uint64)
    period = C.c_uint32(0)
    rc = lib.lapo_detect_iteration(tokens.ctypes.data_as(C.c_void_p), C.c_uint32(len(tokens)),
                                   C.c_uint32(min_period), C.byref(period))
    if rc:
        raise RuntimeError(f"lapo_detect_iteration rc={rc}")
    return int(period.value)


def schedule_swaps(tr, link_GBps: float, swap_list, use_gaps=True):
    lib = _load()
    sl = _c(swap_list, np.uint32)
    k, T = len(sl), tr.n_steps
    o = [np.zeros(max(k, 1), np.int64) for _ in range(4)]
    load = np.zeros(T, np.uint64)
    peak = C.c_uint64(0)
    late = C.c_uint64(0)
    rc = lib.lapo_schedule_swaps(
        C.c_uint32(tr.n_vars), C.c_uint32(T), _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32),
        _opt(tr.free, np.uint32), _opt(tr.gap_lo if use_gaps else None, np.uint32),
        _opt(tr.gap_hi if use_gaps else None, np.uint32), _opt(tr.step_ns, np.uint64), C.c_double(link_GBps),
        sl.ctypes.data_as(C.c_void_p), C.c_uint32(k), *[a.ctypes.data_as(C.c_void_p) for a in o],
        load.ctypes.data_as(C.c_void_p), C.byref(peak), C.byref(late))
    if rc:
        raise RuntimeError(f"lapo_schedule_swaps rc={rc}")
    return dict(out_start=o[0][:k], out_end=o[1][:k], in_start=o[2][:k], in_end=o[3][:k], load=load,
                peak=int(peak.value), late_ns=int(late.value))


def simulate_swaps(tr, link_GBps: float, swap_list, limit: int, use_gaps=True):
    lib = _load()
    sl = _c(swap_list, np.uint32)
    total, over, peak = C.c_uint64(0), C.c_uint64(0), C.c_uint64(0)
    forced = C.c_uint32(0)
    rc = lib.lapo_simulate_swaps(
        C.c_uint32(tr.n_vars), C.c_uint32(tr.n_steps), _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32),
        _opt(tr.free, np.uint32), _opt(tr.gap_lo if use_gaps else None, np.uint32),
        _opt(tr.gap_hi if use_gaps else None, np.uint32), _opt(tr.step_ns, np.uint64), C.c_double(link_GBps),
        sl.ctypes.data_as(C.c_void_p), C.c_uint32(len(sl)), C.c_uint64(limit), C.byref(total), C.byref(over),
        C.byref(peak), C.byref(forced))
    if rc:
        raise RuntimeError(f"lapo_simulate_swaps rc={rc}")
    return dict(total_ns=int(total.value), overhead_ns=int(over.value), peak_resident=int(peak.value),
                forced=int(forced.value))


def evaluate_weights(tr, link_GBps: float, min_bytes: int, weights, limit: int, use_gaps=True):
    lib = _load()
    w = _c(weights, np.float64).reshape(-1, 4)
    W, n = len(w), tr.n_vars
    order = np.zeros((W, n), np.uint32)
    n_sel = np.zeros(W, np.uint32)
    peak_after = np.zeros(W, np.uint64)
    overhead = np.zeros(W, np.uint64)
    forced = np.zeros(W, np.uint32)
    swdoa = np.zeros(n, np.uint64)
    n_cand, best = C.c_uint32(0), C.c_uint32(0)
    rc = lib.lapo_evaluate_weights(
        C.c_uint32(n), C.c_uint32(tr.n_steps), _opt(tr.size, np.uint64), _opt(tr.alloc, np.uint32),
        _opt(tr.free, np.uint32), _opt(tr.gap_lo if use_gaps else None, np.uint32),
        _opt(tr.gap_hi if use_gaps else None, np.uint32), _opt(tr.step_ns, np.uint64), C.c_double(link_GBps),
        C.c_uint64(min_bytes), w.ctypes.data_as(C.c_void_p), C.c_uint32(W), C.c_uint64(limit),
        order.ctypes.data_as(C.c_void_p), C.byref(n_cand), n_sel.ctypes.data_as(C.c_void_p),
        peak_after.ctypes.data_as(C.c_void_p), overhead.ctypes.data_as(C.c_void_p),
        forced.ctypes.data_as(C.c_void_p), C.byref(best), swdoa.ctypes.data_as(C.c_void_p))
    if rc:
        raise RuntimeError(f"lapo_evaluate_weights rc={rc}")
    nc = int(n_cand.value)
    return dict(order=order[:, :nc], n_cand=nc, n_selected=n_sel, peak_after=peak_after, overhead_ns=overhead,
                forced=forced, best=int(best.value), swdoa=swdoa)
