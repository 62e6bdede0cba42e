"""Deterministic, seeded synthetic variable traces shaped like DNN training.

A trace describes one training iteration as the planner sees it (Section
III-A of the paper: every variable has a size and a fixed logical time at which
it is allocated and freed; Section IV: the accesses that bound its idle gap).
Real traces of the paper's networks are not available, so these stand in for
them and keep the structure Section II-D describes: weights live for the whole
iteration, feature maps are created in the forward pass and released in the
backward pass (load ramps up, peaks at the end of forward, ramps down), sizes
spread over many orders of magnitude.

Only input generation lives here.  Random draws come from a counter-based
integer generator (a 64-bit finaliser applied to seed and counter), so a trace
is a pure function of (config, seed) on any machine.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

TRACE_SEED_BASE = 190306631
ORDER_SEED = 631
GRANULE = 512

CONFIG_NAMES = {
    1: "tiny-conv-chain",
    2: "vgg16",
    3: "resnet50",
    4: "deep-residual-chain",
    5: "transformer",
}

# ordering kinds of the boundary (same numbering as include/lap.h)
ORD_SIZE_DESC, ORD_LIFE_DESC, ORD_AREA_DESC, ORD_ALLOC_ASC, ORD_SEEDED, ORD_EXPLICIT, ORD_CLASS_SEEDED = range(7)

_M64 = (1 << 64) - 1


def _fmix(x: int) -> int:
    """64-bit avalanche finaliser (generator-only; unrelated to ordering keys)."""
    x &= _M64
    x ^= x >> 33
    x = (x * 0xFF51AFD7ED558CCD) & _M64
    x ^= x >> 33
    x = (x * 0xC4CEB9FE1A85EC53) & _M64
    x ^= x >> 33
    return x


class CounterRng:
    """draw(i) = fmix(fmix(seed) + i * odd): stateless apart from the counter."""

    def __init__(self, seed: int):
        self.key = _fmix(seed * 0x9E3779B97F4A7C15 + 0x1234567)
        self.ctr = 0

    def u64(self) -> int:
        self.ctr += 1
        return _fmix(self.key + self.ctr * 0xD6E8FEB86659FD93)

    def below(self, n: int) -> int:
        """integer uniform on [0, n) (modulo reduction; bias is irrelevant here)."""
        return self.u64() % n

    def uniform(self, lo: int, hi: int) -> int:
        """integer uniform on [lo, hi] inclusive."""
        return lo + self.below(hi - lo + 1)

    def log_uniform(self, lo_exp: int, hi_exp: int) -> int:
        """exponent e uniform in [lo_exp, hi_exp], value uniform in [2^e, 2^(e+1))."""
        e = self.uniform(lo_exp, hi_exp)
        return (1 << e) + self.below(1 << e)


def _round_up(nbytes: int) -> int:
    return max(GRANULE, (int(nbytes) + GRANULE - 1) // GRANULE * GRANULE)


@dataclass
class Trace:
    name: str
    n_steps: int
    size: np.ndarray      # u64 [N] bytes
    alloc: np.ndarray     # u32 [N] first live step
    free: np.ndarray      # u32 [N] one past the last live step
    gap_lo: np.ndarray    # u32 [N] access that opens the longest idle gap
    gap_hi: np.ndarray    # u32 [N] access that closes it
    step_ns: Optional[np.ndarray] = None   # u64 [T] or None (= 1 ms per step)
    meta: dict = field(default_factory=dict)

    @property
    def n_vars(self) -> int:
        return int(self.size.shape[0])


class _Builder:
    def __init__(self):
        self.size: List[int] = []
        self.alloc: List[int] = []
        self.free: List[int] = []
        self.glo: List[int] = []
        self.ghi: List[int] = []

    def add(self, nbytes, a, f, glo=None, ghi=None):
        assert 0 <= a < f
        glo = a if glo is None else glo
        ghi = f - 1 if ghi is None else ghi
        assert a <= glo <= ghi <= f - 1, (a, f, glo, ghi)
        self.size.append(_round_up(nbytes))
        self.alloc.append(a)
        self.free.append(f)
        self.glo.append(glo)
        self.ghi.append(ghi)

    def __len__(self):
        return len(self.size)

    def finish(self, name, T, step_ns=None, meta=None) -> Trace:
        return Trace(
            name=name,
            n_steps=T,
            size=np.asarray(self.size, dtype=np.uint64),
            alloc=np.asarray(self.alloc, dtype=np.uint32),
            free=np.asarray(self.free, dtype=np.uint32),
            gap_lo=np.asarray(self.glo, dtype=np.uint32),
            gap_hi=np.asarray(self.ghi, dtype=np.uint32),
            step_ns=step_ns,
            meta=meta or {},
        )


@dataclass
class _Op:
    out: int                      # bytes of the output tensor
    weight: int = 0               # bytes of the parameter tensor (0 = none)
    workspace: bool = False       # has forward and backward scratch
    extra_acts: tuple = ()        # more saved tensors that also get a gradient
    extra_stats: tuple = ()       # saved tensors without a gradient


def _emit(ops: List[_Op], rng: CounterRng, draw_ws, n_total: int, draw_tmp) -> _Builder:
    """Lay the ops out on the time line and pad with 1-step temporaries.

    Forward op k runs at step k, its backward at step 2F-1-k, T = 2F.
    """
    F = len(ops)
    T = 2 * F
    b = _Builder()
    # forward tensors, op order
    for k, op in enumerate(ops):
        bk = 2 * F - 1 - k
        if op.weight:
            b.add(op.weight, 0, T, k, bk)                      # read in fwd, again in bwd
        if k < F - 1:
            glo, ghi = k + 1, 2 * F - 2 - k
        else:
            glo, ghi = F - 1, F
        for nbytes in (op.out,) + tuple(op.extra_acts) + tuple(op.extra_stats):
            b.add(nbytes, k, 2 * F - k, glo, ghi)
        if op.workspace:
            b.add(draw_ws(rng), k, k + 1)
    # backward tensors, backward order
    for k in range(F - 1, -1, -1):
        op = ops[k]
        bk = 2 * F - 1 - k
        if op.workspace:
            b.add(draw_ws(rng), bk, bk + 1)
        for nbytes in (op.out,) + tuple(op.extra_acts):
            b.add(nbytes, bk, min(bk + 2, T))                  # gradient lives 2 steps
        if op.weight:
            b.add(op.weight, 0, T, bk, T - 1)                  # weight gradient
    assert len(b) <= n_total, (len(b), n_total)
    while len(b) < n_total:
        t = rng.below(T)
        b.add(draw_tmp(rng), t, t + 1)
    return b


def _ops_tiny() -> List[_Op]:
    chans = [16, 16, 16, 32, 32, 32, 64, 64, 64, 64]
    spatial = [32, 32, 32, 16, 16, 16, 8, 8, 8, 8]
    ops, cin = [], 3
    for c, h in zip(chans, spatial):
        ops.append(_Op(out=8 * c * h * h * 4, weight=cin * c * 9 * 4, workspace=True))
        cin = c
    ops.append(_Op(out=8 * 10 * 4, weight=64 * 8 * 8 * 10 * 4, workspace=True))
    return ops


def _ops_vgg16() -> List[_Op]:
    cfg = [(64, 2, 224), (128, 2, 112), (256, 3, 56), (512, 3, 28), (512, 3, 14)]
    ops, cin, batch = [], 3, 64
    for c, reps, h in cfg:
        for _ in range(reps):
            ops.append(_Op(out=batch * c * h * h * 4, weight=cin * c * 9 * 4, workspace=True))
            cin = c
        pooled = batch * c * (h // 2) * (h // 2)
        ops.append(_Op(out=pooled * 4, extra_stats=(pooled * 4,)))     # int32 argmax mask
    feat = 512 * 7 * 7
    for width in (4096, 4096, 1000):
        ops.append(_Op(out=batch * width * 4, weight=feat * width * 4, workspace=True))
        feat = width
    return ops


def _conv_bn_relu(ops, batch, cin, cout, h, k, relu=True):
    act = batch * cout * h * h * 4
    ops.append(_Op(out=act, weight=cin * cout * k * k * 4, workspace=True))
    ops.append(_Op(out=act, weight=2 * cout * 4, extra_stats=(2 * cout * 4,)))   # BN + saved mean/var
    if relu:
        ops.append(_Op(out=act))


def _ops_resnet50() -> List[_Op]:
    batch, ops = 128, []
    _conv_bn_relu(ops, batch, 3, 64, 112, 7)
    ops.append(_Op(out=batch * 64 * 56 * 56 * 4))                      # max pool
    cin, h = 64, 56
    for stage, (blocks, width) in enumerate(zip([3, 4, 6, 3], [256, 512, 1024, 2048])):
        mid = width // 4
        for blk in range(blocks):
            if blk == 0 and stage > 0:
                h //= 2
            if blk == 0:
                _conv_bn_relu(ops, batch, cin, width, h, 1, relu=False)   # projection shortcut
            _conv_bn_relu(ops, batch, cin, mid, h, 1)
            _conv_bn_relu(ops, batch, mid, mid, h, 3)
            _conv_bn_relu(ops, batch, mid, width, h, 1, relu=False)
            act = batch * width * h * h * 4
            ops.append(_Op(out=act))                                   # residual add
            ops.append(_Op(out=act))                                   # ReLU
            cin = width
    ops.append(_Op(out=batch * 2048 * 4))                              # global average pool
    ops.append(_Op(out=batch * 1000 * 4, weight=2048 * 1000 * 4, workspace=True))
    return ops


def _ops_deep_chain() -> List[_Op]:
    batch, c, h = 32, 256, 56
    act = batch * c * h * h * 4
    ops = []
    for _ in range(1000):
        for _half in range(2):
            ops.append(_Op(out=act, weight=c * c * 9 * 4, workspace=True))
            ops.append(_Op(out=act, weight=2 * c * 4, extra_stats=(2 * c * 4,)))
            if _half == 0:
                ops.append(_Op(out=act))                               # ReLU
        ops.append(_Op(out=act))                                       # add
        ops.append(_Op(out=act))                                       # ReLU
    return ops


def _ops_transformer() -> List[_Op]:
    batch, seq, hid, heads, ffn, e = 8, 2048, 2048, 16, 8192, 2
    tok = batch * seq
    x = tok * hid * e
    stat = batch * seq * 4
    scores = batch * heads * seq * seq * e
    ops = [_Op(out=x, weight=32000 * hid * e)]                          # embedding
    for _ in range(24):
        ops.append(_Op(out=x, weight=2 * hid * e, extra_stats=(stat, stat)))          # LN
        ops.append(_Op(out=x, weight=hid * 3 * hid * e, workspace=True, extra_acts=(x, x)))  # Q,K,V
        ops.append(_Op(out=scores, workspace=True))                                   # QK^T
        ops.append(_Op(out=scores))                                                   # softmax
        ops.append(_Op(out=x, workspace=True))                                        # PV
        ops.append(_Op(out=x, weight=hid * hid * e, workspace=True))                  # out proj
        ops.append(_Op(out=x))                                                        # residual
        ops.append(_Op(out=x, weight=2 * hid * e, extra_stats=(stat, stat)))          # LN
        ops.append(_Op(out=tok * ffn * e, weight=hid * ffn * e, workspace=True))      # MLP up
        ops.append(_Op(out=tok * ffn * e))                                            # activation
        ops.append(_Op(out=x, weight=ffn * hid * e, workspace=True))                  # MLP down
        ops.append(_Op(out=x))                                                        # residual
    ops.append(_Op(out=x, weight=2 * hid * e, extra_stats=(stat, stat)))              # final LN
    return ops


_SPECS = {
    # cfg: (ops, N, B, workspace draw, temporary draw, swap scoring?, step_ns range or None)
    1: (_ops_tiny, 120, 16, lambda r: r.uniform(0, 1 << 20), lambda r: r.uniform(0, 1 << 20), True, None),
    2: (_ops_vgg16, 600, 256, lambda r: r.uniform(0, 64 << 20), lambda r: r.uniform(0, 64 << 20), False, None),
    3: (_ops_resnet50, 3000, 1024, lambda r: r.uniform(0, 64 << 20), lambda r: r.uniform(0, 64 << 20), True,
        (200_000, 2_000_000)),
    4: (_ops_deep_chain, 50_000, 4096, lambda r: r.log_uniform(12, 24), lambda r: r.log_uniform(12, 24), False, None),
    5: (_ops_transformer, 200_000, 1024, lambda r: r.uniform(0, 16 << 20), lambda r: r.uniform(0, 16 << 20), True, None),
}


def make_config(cfg: int) -> Trace:
    """Trace of benchmark configuration `cfg` (1..5).  Deterministic."""
    ops_fn, n_total, n_orderings, draw_ws, draw_tmp, score, ns_range = _SPECS[cfg]
    rng = CounterRng(TRACE_SEED_BASE + cfg)
    ops = ops_fn()
    b = _emit(ops, rng, draw_ws, n_total, draw_tmp)
    T = 2 * len(ops)
    step_ns = None
    if ns_range is not None:
        srng = CounterRng(TRACE_SEED_BASE + cfg + 1000)
        step_ns = np.asarray([srng.uniform(*ns_range) for _ in range(T)], dtype=np.uint64)
    meta = dict(cfg=cfg, B=n_orderings, link_GBps=64.0, min_bytes=1 << 20, score_swaps=score)
    return b.finish(CONFIG_NAMES[cfg], T, step_ns, meta)


def make_orderings(B: int):
    """The harness's ordering batch: the 4 fixed heuristics, then seeded shuffles.

    Returns (kind u32[B], seed u64[B]); seed of ordering b is ORDER_SEED + b.
    """
    kind = np.full(B, ORD_SEEDED, dtype=np.uint32)
    nfix = min(B, 4)
    kind[:nfix] = np.arange(nfix, dtype=np.uint32)
    seed = (ORDER_SEED + np.arange(B)).astype(np.uint64)
    return kind, seed


def random_trace(seed: int, n: int, T: int, *, size_choices=None, max_life=None,
                 one_step_frac: float = 0.3, with_step_ns: bool = False,
                 granule: int = GRANULE) -> Trace:
    """Small random trace for property tests: coarse steps and repeated sizes
    force ties in every ordering key; a mix of 1-step and long lifetimes."""
    rng = CounterRng(0xABCDEF ^ seed)
    b = _Builder()
    max_life = max_life or T
    thresh = int(one_step_frac * 1000)
    for _ in range(n):
        if size_choices is not None:
            s = size_choices[rng.below(len(size_choices))] * granule
        else:
            s = rng.log_uniform(9, 22)
        if rng.below(1000) < thresh:
            a = rng.below(T)
            f = a + 1
        else:
            a = rng.below(T)
            f = a + 1 + rng.below(min(max_life, T - a))
        if rng.below(2):
            glo, ghi = a, f - 1                       # touched when created and when last used
        else:
            glo = rng.uniform(a, f - 1)
            ghi = rng.uniform(glo, f - 1)
        b.size.append(max(granule, (s + granule - 1) // granule * granule) if granule > 1 else max(1, s))
        b.alloc.append(a)
        b.free.append(f)
        b.glo.append(glo)
        b.ghi.append(ghi)
    step_ns = None
    if with_step_ns:
        step_ns = np.asarray([rng.uniform(1_000, 3_000_000) for _ in range(T)], dtype=np.uint64)
    return b.finish(f"random-{seed}", T, step_ns, dict(cfg=0))


def tile_in_time(tr: Trace, reps: int) -> Trace:
    """Repeat a trace `reps` times along the time axis (iteration after
    iteration, as in the multi-iteration load curve of Section II-D)."""
    T = tr.n_steps
    shift = (np.arange(reps, dtype=np.uint32) * np.uint32(T))[:, None]
    rep = lambda a: (a[None, :] + shift).reshape(-1).astype(np.uint32)
    return Trace(
        name=f"{tr.name}-x{reps}",
        n_steps=T * reps,
        size=np.tile(tr.size, reps),
        alloc=rep(tr.alloc), free=rep(tr.free), gap_lo=rep(tr.gap_lo), gap_hi=rep(tr.gap_hi),
        step_ns=None if tr.step_ns is None else np.tile(tr.step_ns, reps),
        meta=dict(tr.meta, reps=reps),
    )
