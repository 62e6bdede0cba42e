"""ctypes binding of liblap.so: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblap.so")
_lib = None

EXPORTS = [
    "lap_workspace_bytes", "lap_load_profile", "lap_load_profile_static", "lap_plan_pool", "lap_score_swaps", "lap_select_swaps",
    "lap_detect_iteration", "lap_schedule_swaps", "lap_simulate_swaps", "lap_evaluate_weights",
    "lap_validate_trace", "lap_status_string", "lap_profile_enable", "lap_profile_last_ms", "lap_profile_ordering_ms", "lap_plan_pool_orders", "lap_set_option",
]


class LapError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


class _Trace(C.Structure):
    _fields_ = [("n_vars", C.c_uint32), ("n_steps", C.c_uint32),
                ("size", C.c_void_p), ("alloc", C.c_void_p), ("free_", C.c_void_p),
                ("gap_lo", C.c_void_p), ("gap_hi", C.c_void_p), ("step_ns", C.c_void_p)]


class _Ordering(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("fit", C.c_uint32), ("seed", C.c_uint64)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load liblap.so (built in-tree by paper_1903_06631_amd/build.py).  Fails loudly."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    # torch brings its own HIP runtime: load it first so that liblap binds to the same one
    # (two runtimes in one process do not both see the GPU)
    import torch  # noqa: F401
    lib = C.CDLL(_LIB_PATH)
    lib.lap_workspace_bytes.restype = C.c_size_t
    lib.lap_workspace_bytes.argtypes = [C.c_int, C.c_uint32, C.c_uint32, C.c_uint32]
    lib.lap_status_string.restype = C.c_char_p
    lib.lap_status_string.argtypes = [C.c_int]
    lib.lap_load_profile.restype = C.c_int
    lib.lap_load_profile.argtypes = [C.POINTER(_Trace), C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lap_load_profile_static.restype = C.c_int
    lib.lap_load_profile_static.argtypes = [C.POINTER(_Trace), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.lap_plan_pool.restype = C.c_int
    lib.lap_plan_pool.argtypes = [C.POINTER(_Trace), C.POINTER(_Ordering), C.c_uint32,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lap_score_swaps.restype = C.c_int
    lib.lap_score_swaps.argtypes = [C.POINTER(_Trace), C.c_double, C.c_uint64, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lap_select_swaps.restype = C.c_int
    lib.lap_select_swaps.argtypes = [C.POINTER(_Trace), C.c_double, C.c_uint64, C.c_void_p,
                                     C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lap_schedule_swaps.restype = C.c_int
    lib.lap_schedule_swaps.argtypes = [C.POINTER(_Trace), C.c_double, C.c_void_p, C.c_void_p, C.c_uint32,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lap_simulate_swaps.restype = C.c_int
    lib.lap_simulate_swaps.argtypes = [C.POINTER(_Trace), C.c_double, C.c_void_p, C.c_uint32, C.c_void_p,
                                       C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lap_evaluate_weights.restype = C.c_int
    lib.lap_evaluate_weights.argtypes = [C.POINTER(_Trace), C.c_double, C.c_uint64, C.c_void_p, C.c_void_p, C.c_uint32,
                                         C.c_uint64] + [C.c_void_p] * 9 + [C.c_size_t, C.c_void_p]
    lib.lap_detect_iteration.restype = C.c_int
    lib.lap_detect_iteration.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_size_t,
                                         C.c_void_p]
    lib.lap_validate_trace.restype = C.c_int
    lib.lap_validate_trace.argtypes = [C.POINTER(_Trace), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.lap_set_option.restype = C.c_int
    lib.lap_set_option.argtypes = [C.c_int, C.c_uint64]
    lib.lap_profile_enable.restype = C.c_int
    lib.lap_profile_enable.argtypes = [C.c_int]
    lib.lap_profile_ordering_ms.restype = C.c_int
    lib.lap_profile_ordering_ms.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p,
                                            C.c_void_p]
    lib.lap_profile_last_ms.restype = C.c_float
    lib.lap_plan_pool_orders.restype = C.c_int
    lib.lap_plan_pool_orders.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.lap_profile_last_ms.argtypes = [C.c_int]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().lap_status_string(int(status)).decode()


def workspace_bytes(which: int, n_vars: int, n_steps: int, B: int = 0) -> int:
    return int(load_library().lap_workspace_bytes(which, n_vars, n_steps, B))


OPT_SEG_MIN_VARS = 0
OPT_SEG_TRIAL_PERCENT = 1
SEG_MIN_VARS_DEFAULT = 32768
SEG_TRIAL_PERCENT_DEFAULT = 250


def set_option(option: int, value: int) -> None:
    rc = load_library().lap_set_option(int(option), int(value))
    if rc:
        raise LapError(rc, "lap_set_option")


def profile_enable(on: bool) -> None:
    load_library().lap_profile_enable(1 if on else 0)


def profile_last_ms(kernel_id: int) -> float:
    return float(load_library().lap_profile_last_ms(kernel_id))


def profile_ordering_ms(dt, B: int) -> np.ndarray:
    """lap_profile_ordering_ms: per-ordering duration (ms) of the last plan_pool call on this trace with B orderings."""
    ws, need = dt.workspace(1, B)
    out = np.zeros(B, np.float32)
    rc = load_library().lap_profile_ordering_ms(dt.n_vars, dt.n_steps, B, ws.data_ptr(), need, _stream_ptr(dt.device),
                                                out.ctypes.data_as(C.c_void_p))
    if rc:
        raise LapError(rc, "lap_profile_ordering_ms")
    return out


def plan_pool_orders(dt, B: int):
    """lap_plan_pool_orders: the placement orders of the last plan_pool call on this trace with B orderings,
    int32 device tensor [B, N] (the bits of the uint32 variable indices)."""
    torch = _torch()
    ws, need = dt.workspace(1, B)
    out = torch.empty((B, dt.n_vars), dtype=torch.int32, device=dt.device)
    rc = load_library().lap_plan_pool_orders(dt.n_vars, dt.n_steps, B, ws.data_ptr(), need, _stream_ptr(dt.device),
                                             out.data_ptr())
    if rc:
        raise LapError(rc, "lap_plan_pool_orders")
    return out


def _torch():
    import torch
    return torch


def _as_signed(a: np.ndarray) -> np.ndarray:
    """torch has no full uint32/uint64 support: move the bits through the signed twin."""
    return a.view({np.dtype(np.uint64): np.int64, np.dtype(np.uint32): np.int32}.get(a.dtype, a.dtype))


class DeviceTrace:
    """A trace resident in HBM: structure of arrays, one torch tensor per field."""

    def __init__(self, trace, device="cuda:0", use_gaps: bool = True):
        torch = _torch()
        self.device = torch.device(device)
        self.n_vars = int(trace.n_vars)
        self.n_steps = int(trace.n_steps)
        put = lambda a, dt: torch.from_numpy(_as_signed(np.ascontiguousarray(a, dtype=dt))).to(self.device)
        self.size = put(trace.size, np.uint64)
        self.alloc = put(trace.alloc, np.uint32)
        self.free = put(trace.free, np.uint32)
        self.gap_lo = put(trace.gap_lo, np.uint32) if use_gaps and trace.gap_lo is not None else None
        self.gap_hi = put(trace.gap_hi, np.uint32) if use_gaps and trace.gap_hi is not None else None
        self.step_ns = put(trace.step_ns, np.uint64) if trace.step_ns is not None else None
        self._ws = {}

    def nbytes(self) -> int:
        ts = [self.size, self.alloc, self.free, self.gap_lo, self.gap_hi, self.step_ns]
        return sum(t.numel() * t.element_size() for t in ts if t is not None)

    def c_struct(self) -> _Trace:
        p = lambda t: None if t is None else t.data_ptr()
        return _Trace(self.n_vars, self.n_steps, p(self.size), p(self.alloc), p(self.free),
                      p(self.gap_lo), p(self.gap_hi), p(self.step_ns))

    def workspace(self, which: int, B: int = 0):
        """Grow-only scratch tensor for one kind of call (caller-owned device memory)."""
        torch = _torch()
        need = workspace_bytes(which, self.n_vars, self.n_steps, B)
        ws = self._ws.get(which)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device=self.device)
            self._ws[which] = ws
        return ws, need


def _stream_ptr(device) -> int:
    torch = _torch()
    return int(torch.cuda.current_stream(device).cuda_stream)


def _u64(t):
    """int64 tensor -> numpy uint64 (host copy)."""
    return t.cpu().numpy().view(np.uint64)


def load_profile(dt: DeviceTrace, sync: bool = True):
    """lap_load_profile: returns dict(load[T], peak, t_peak) as device tensors (int64/int32 bit patterns)."""
    torch = _torch()
    lib = load_library()
    load = torch.empty(dt.n_steps, dtype=torch.int64, device=dt.device)
    peak = torch.empty(1, dtype=torch.int64, device=dt.device)
    t_peak = torch.empty(1, dtype=torch.int32, device=dt.device)
    ws, need = dt.workspace(0)
    tr = dt.c_struct()
    rc = lib.lap_load_profile(C.byref(tr), load.data_ptr(), peak.data_ptr(), t_peak.data_ptr(),
                              ws.data_ptr(), need, _stream_ptr(dt.device))
    if rc:
        raise LapError(rc, "lap_load_profile")
    if sync:
        torch.cuda.current_stream(dt.device).synchronize()
    return dict(load=load, peak=peak, t_peak=t_peak)


STATIC_MAX_STEPS = 1 << 20


def load_profile_static(dt: DeviceTrace, sync: bool = True):
    """lap_load_profile_static: as load_profile, with the library's own fixed scratch array (no workspace)."""
    torch = _torch()
    lib = load_library()
    load = torch.empty(dt.n_steps, dtype=torch.int64, device=dt.device)
    peak = torch.empty(1, dtype=torch.int64, device=dt.device)
    t_peak = torch.empty(1, dtype=torch.int32, device=dt.device)
    tr = dt.c_struct()
    rc = lib.lap_load_profile_static(C.byref(tr), load.data_ptr(), peak.data_ptr(), t_peak.data_ptr(),
                                     _stream_ptr(dt.device))
    if rc:
        raise LapError(rc, "lap_load_profile_static")
    if sync:
        torch.cuda.current_stream(dt.device).synchronize()
    return dict(load=load, peak=peak, t_peak=t_peak)


def make_orderings(kinds: Sequence[int], seeds: Sequence[int], fits: Optional[Sequence[int]] = None):
    arr = (_Ordering * len(kinds))()
    for b, (k, s) in enumerate(zip(kinds, seeds)):
        arr[b].kind = int(k)
        arr[b].fit = 0 if fits is None else int(fits[b])
        arr[b].seed = int(s)
    return arr


def plan_pool(dt: DeviceTrace, kinds: Sequence[int], seeds: Sequence[int], *, explicit: Optional[dict] = None,
              fits: Optional[Sequence[int]] = None, want_all: bool = True, want_footprints: bool = True, sync: bool = True, out: Optional[dict] = None):
    """lap_plan_pool.  explicit: {ordering index: int32 device tensor with a permutation} for kind 5.

    Returns device tensors: best_offsets[N], best_footprint[1], best_ordering[1],
    footprints[B] (optional), all_offsets[B,N] (optional)."""
    torch = _torch()
    lib = load_library()
    B, n = len(kinds), dt.n_vars
    seeds = [int(s) for s in seeds]
    if explicit:
        for b, t in explicit.items():
            assert t.dtype == torch.int32 and t.is_contiguous() and t.numel() == n
            seeds[b] = t.data_ptr()
    ords = make_orderings(kinds, seeds, fits)
    if out is None:
        out = dict(
            best_offsets=torch.empty(n, dtype=torch.int64, device=dt.device),
            best_footprint=torch.empty(1, dtype=torch.int64, device=dt.device),
            best_ordering=torch.empty(1, dtype=torch.int32, device=dt.device),
            footprints=torch.empty(B, dtype=torch.int64, device=dt.device) if want_footprints else None,
            all_offsets=torch.empty((B, n), dtype=torch.int64, device=dt.device) if want_all else None,
        )
    ws, need = dt.workspace(1, B)
    tr = dt.c_struct()
    p = lambda t: None if t is None else t.data_ptr()
    rc = lib.lap_plan_pool(C.byref(tr), ords, B, p(out["best_offsets"]), p(out["best_footprint"]),
                           p(out["best_ordering"]), p(out.get("footprints")), p(out.get("all_offsets")),
                           ws.data_ptr(), need, _stream_ptr(dt.device))
    if rc:
        raise LapError(rc, "lap_plan_pool")
    if sync:
        torch.cuda.current_stream(dt.device).synchronize()
    return out


def score_swaps(dt: DeviceTrace, link_GBps: float, min_bytes: int, load=None, sync: bool = True):
    """lap_score_swaps: returns dict of device tensors candidate(u8), doa_ns(i64), aoa(f64), wdoa, peak_cut."""
    torch = _torch()
    lib = load_library()
    n = dt.n_vars
    out = dict(
        candidate=torch.empty(n, dtype=torch.uint8, device=dt.device),
        doa_ns=torch.empty(n, dtype=torch.int64, device=dt.device),
        aoa=torch.empty(n, dtype=torch.float64, device=dt.device),
        wdoa=torch.empty(n, dtype=torch.int64, device=dt.device),
        peak_cut=torch.empty(n, dtype=torch.int64, device=dt.device),
    )
    ws, need = dt.workspace(2)
    tr = dt.c_struct()
    rc = lib.lap_score_swaps(C.byref(tr), float(link_GBps), int(min_bytes),
                             None if load is None else load.data_ptr(),
                             out["candidate"].data_ptr(), out["doa_ns"].data_ptr(), out["aoa"].data_ptr(),
                             out["wdoa"].data_ptr(), out["peak_cut"].data_ptr(),
                             ws.data_ptr(), need, _stream_ptr(dt.device))
    if rc:
        raise LapError(rc, "lap_score_swaps")
    if sync:
        torch.cuda.current_stream(dt.device).synchronize()
    return out


def select_swaps(dt: DeviceTrace, link_GBps: float, min_bytes: int, score_kinds: Sequence[int],
                 limits: Sequence[int] = (), load=None, want_rank: bool = True, sync: bool = True):
    """lap_select_swaps: returns device tensors order[K,N], rank[K,N] (optional), peaks[K,N+1], n_cand[1],
    n_selected[K,L], peak_after[K,L], load_min[1] (rows are valid up to n_cand; see include/lap.h)."""
    torch = _torch()
    lib = load_library()
    n, K, L = dt.n_vars, len(score_kinds), len(limits)
    kinds = (C.c_uint32 * max(K, 1))(*[int(k) for k in score_kinds])
    lims = (C.c_uint64 * max(L, 1))(*[int(x) for x in limits])
    out = dict(
        order=torch.empty((K, n), dtype=torch.int32, device=dt.device),
        rank=torch.empty((K, n), dtype=torch.int32, device=dt.device) if want_rank else None,
        peaks=torch.empty((K, n + 1), dtype=torch.int64, device=dt.device),
        n_cand=torch.empty(1, dtype=torch.int32, device=dt.device),
        n_selected=torch.empty((K, L), dtype=torch.int32, device=dt.device),
        peak_after=torch.empty((K, L), dtype=torch.int64, device=dt.device),
        load_min=torch.empty(1, dtype=torch.int64, device=dt.device),
    )
    ws, need = dt.workspace(4, K)
    tr = dt.c_struct()
    p = lambda t: None if t is None else t.data_ptr()
    rc = lib.lap_select_swaps(C.byref(tr), float(link_GBps), int(min_bytes), p(load),
                              kinds, K, lims if L else None, L,
                              p(out["order"]), p(out["rank"]), p(out["peaks"]), p(out["n_cand"]),
                              p(out["n_selected"]) if L else None, p(out["peak_after"]) if L else None,
                              p(out["load_min"]), ws.data_ptr(), need, _stream_ptr(dt.device))
    if rc:
        raise LapError(rc, "lap_select_swaps")
    if sync:
        torch.cuda.current_stream(dt.device).synchronize()
    return out


def schedule_swaps(dt: DeviceTrace, link_GBps: float, swap_list, load=None, sync: bool = True):
    """lap_schedule_swaps: swap_list is an int32 device tensor of variable indices.  Returns device tensors
    out_start, out_end, in_start, in_end [k] (int64 ns), load[T], peak[1], late_ns[1]."""
    torch = _torch()
    lib = load_library()
    assert swap_list.dtype == torch.int32 and swap_list.is_contiguous()
    k = swap_list.numel()
    mk = lambda m, dtp=torch.int64: torch.empty(m, dtype=dtp, device=dt.device)
    out = dict(out_start=mk(k), out_end=mk(k), in_start=mk(k), in_end=mk(k), load=mk(dt.n_steps), peak=mk(1),
               late_ns=mk(1))
    ws, need = dt.workspace(6)
    tr = dt.c_struct()
    p = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
    rc = lib.lap_schedule_swaps(C.byref(tr), float(link_GBps), p(load), p(swap_list), k, p(out["out_start"]),
                                p(out["out_end"]), p(out["in_start"]), p(out["in_end"]), p(out["load"]),
                                p(out["peak"]), p(out["late_ns"]), ws.data_ptr(), need, _stream_ptr(dt.device))
    if rc:
        raise LapError(rc, "lap_schedule_swaps")
    if sync:
        torch.cuda.current_stream(dt.device).synchronize()
    return out


def simulate_swaps(dt: DeviceTrace, link_GBps: float, swap_list, prefix_len: Sequence[int],
                   limits: Sequence[int], sync: bool = True):
    """lap_simulate_swaps: Q = len(limits) runs; returns device tensors total_ns, overhead_ns, peak_resident
    (int64 bit patterns) and forced (int32), one entry per run."""
    torch = _torch()
    lib = load_library()
    assert swap_list.dtype == torch.int32 and swap_list.is_contiguous()
    Q = len(limits)
    assert len(prefix_len) == Q
    pl = (C.c_uint32 * max(Q, 1))(*[int(x) for x in prefix_len])
    lm = (C.c_uint64 * max(Q, 1))(*[int(x) for x in limits])
    out = dict(total_ns=torch.empty(Q, dtype=torch.int64, device=dt.device),
               overhead_ns=torch.empty(Q, dtype=torch.int64, device=dt.device),
               peak_resident=torch.empty(Q, dtype=torch.int64, device=dt.device),
               forced=torch.empty(Q, dtype=torch.int32, device=dt.device))
    ws, need = dt.workspace(7, Q)
    tr = dt.c_struct()
    k = swap_list.numel()
    rc = lib.lap_simulate_swaps(C.byref(tr), float(link_GBps), swap_list.data_ptr() if k else None, k, pl, lm, Q,
                                out["total_ns"].data_ptr(), out["overhead_ns"].data_ptr(),
                                out["peak_resident"].data_ptr(), out["forced"].data_ptr(), ws.data_ptr(), need,
                                _stream_ptr(dt.device))
    if rc:
        raise LapError(rc, "lap_simulate_swaps")
    if sync:
        torch.cuda.current_stream(dt.device).synchronize()
    return out


def evaluate_weights(dt: DeviceTrace, link_GBps: float, min_bytes: int, weights, limit: int, load=None,
                     sync: bool = True):
    """lap_evaluate_weights: weights is a (W, 4) array-like of (a, b, c, d).  Returns device tensors order[W,N],
    n_cand[1], n_selected[W], peak_after[W], overhead_ns[W], forced[W], best[1], swdoa[N]."""
    torch = _torch()
    lib = load_library()
    w = np.ascontiguousarray(weights, dtype=np.float64).reshape(-1, 4)
    W, n = len(w), dt.n_vars
    i32 = lambda m: torch.empty(m, dtype=torch.int32, device=dt.device)
    i64 = lambda m: torch.empty(m, dtype=torch.int64, device=dt.device)
    out = dict(order=torch.empty((W, n), dtype=torch.int32, device=dt.device), n_cand=i32(1), n_selected=i32(W),
               peak_after=i64(W), overhead_ns=i64(W), forced=i32(W), best=i32(1), swdoa=i64(n))
    ws, need = dt.workspace(8, W)
    tr = dt.c_struct()
    rc = lib.lap_evaluate_weights(C.byref(tr), float(link_GBps), int(min_bytes),
                                  None if load is None else load.data_ptr(), w.ctypes.data_as(C.c_void_p), W,
                                  int(limit), out["order"].data_ptr(), out["n_cand"].data_ptr(),
                                  out["n_selected"].data_ptr(), out["peak_after"].data_ptr(),
                                  out["overhead_ns"].data_ptr(), out["forced"].data_ptr(), out["best"].data_ptr(),
                                  out["swdoa"].data_ptr(), ws.data_ptr(), need, _stream_ptr(dt.device))
    if rc:
        raise LapError(rc, "lap_evaluate_weights")
    if sync:
        torch.cuda.current_stream(dt.device).synchronize()
    return out


def detect_iteration(tokens, min_period: int = 1, sync: bool = True):
    """lap_detect_iteration: tokens is an int64 device tensor (bit patterns of the 64-bit request tokens);
    returns a 1-element int32 device tensor with the period (0 = none)."""
    torch = _torch()
    lib = load_library()
    assert tokens.dtype == torch.int64 and tokens.is_contiguous() and tokens.is_cuda
    m = tokens.numel()
    need = workspace_bytes(5, m, 0, 0)
    ws = torch.empty(need, dtype=torch.uint8, device=tokens.device)
    period = torch.empty(1, dtype=torch.int32, device=tokens.device)
    rc = lib.lap_detect_iteration(tokens.data_ptr(), m, int(min_period), period.data_ptr(), ws.data_ptr(), need,
                                  _stream_ptr(tokens.device))
    if rc:
        raise LapError(rc, "lap_detect_iteration")
    if sync:
        torch.cuda.current_stream(tokens.device).synchronize()
    return period


def validate_trace(dt: DeviceTrace) -> int:
    """lap_validate_trace: returns the status code (0 = valid); waits for the stream."""
    lib = load_library()
    ws, need = dt.workspace(3)
    tr = dt.c_struct()
    return int(lib.lap_validate_trace(C.byref(tr), ws.data_ptr(), need, _stream_ptr(dt.device)))
