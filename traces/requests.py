"""Seeded synthetic request streams (what a runtime would record in its first iterations): one
64-bit token per request = operation kind in the top byte, size below.  Generator only."""
from __future__ import annotations

import numpy as np

from .dnn import CounterRng

OP_MALLOC, OP_FREE, OP_READ, OP_WRITE = 1, 2, 3, 4


def iteration_tokens(tr) -> np.ndarray:
    """One iteration of a trace as a request list: per step the mallocs, one write and one read
    per live variable that is accessed there (gap_lo / gap_hi), then the frees."""
    ev = []
    for i in range(tr.n_vars):
        s = int(tr.size[i])
        ev.append((int(tr.alloc[i]), 0, i, (OP_MALLOC << 56) | s))
        ev.append((int(tr.gap_lo[i]), 1, i, (OP_WRITE << 56) | s))
        if tr.gap_hi[i] != tr.gap_lo[i]:
            ev.append((int(tr.gap_hi[i]), 2, i, (OP_READ << 56) | s))
        ev.append((int(tr.free[i]) - 1, 3, i, (OP_FREE << 56) | s))
    ev.sort()
    return np.array([e[3] for e in ev], dtype=np.uint64)


def request_stream(iteration: np.ndarray, n_iters: int, warmup: int, tail: int, seed: int) -> np.ndarray:
    """warm-up requests that belong to no iteration, n_iters copies of the iteration, and the first
    `tail` requests of one more."""
    rng = CounterRng(seed)
    pre = np.array([(OP_MALLOC << 56) | (512 * (1 + rng.below(4096))) for _ in range(warmup)], dtype=np.uint64)
    return np.concatenate([pre] + [iteration] * n_iters + [iteration[:tail]]).astype(np.uint64)
