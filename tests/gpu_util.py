"""Helpers for the GPU parity tests: oracle runs spread over host threads."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

# one oracle run per host thread; a GPU machine gives a job 16 CPUs whatever os.cpu_count() says
WORKERS = max(1, min(16, (os.cpu_count() or 8)))


def u64(t):
    return t.cpu().numpy().view(np.uint64)


def oracle_all_orderings(oracle, tr, kinds, seeds, explicit=None, which=None, fits=None):
    """Oracle offsets/footprints for the given orderings (ctypes releases the GIL)."""
    idx = list(range(len(kinds))) if which is None else list(which)

    def one(b):
        ex = None if not explicit or b not in explicit else explicit[b]
        perm = oracle.make_perm(tr, int(kinds[b]), int(seeds[b]), explicit=ex)
        off, fp = oracle.place(tr, perm, best_fit=bool(fits[b]) if fits is not None else False)
        return b, perm, off, fp

    with ThreadPoolExecutor(WORKERS) as ex:
        res = list(ex.map(one, idx))
    return {b: (perm, off, fp) for b, perm, off, fp in res}
