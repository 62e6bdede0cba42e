#!/usr/bin/env python3
"""Writes the stored oracle results for the full-size placement tests.

For configurations 4 and 5 the oracle (oracle/lap_oracle.c, single-threaded, about a minute per
ordering) places one ordering per worker process; every finished ordering appends one line

    <ordering index> <kind> <seed> <footprint in bytes> <16 hex digits of SHA-256 of the u64 offsets>

to tests/golden/fullsize_cfg<c>_<first|best>_fit.txt.  Only the oracle and the seeded input
generators are called; nothing here touches the GPU library.  The run is resumable: orderings
already in a file are skipped.  The order of work puts a spread of 64 orderings per file first
(the fixed orders, every kind-6 position, a seeded sample), then the rest in ascending order.

    python tests/golden/make_fullsize_hashes.py --workers 6 [--jobs 5:first 4:first 5:best 4:best]
                                                [--limit 5:first=1024 4:first=512 ...]
                                                [--count 160] [--from-the-end]

--count bounds the orderings of one run; --from-the-end takes the orderings after the first 64 in
descending order, so that a second run on another machine does not repeat what the first one does.
"""
import argparse
import os
import sys
from concurrent.futures import ProcessPoolExecutor, as_completed

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np  # noqa: E402

HEADER = """# Oracle results at full size, written by tests/golden/make_fullsize_hashes.py (oracle only):
# configuration {cfg}, {fit}-fit placement (Section III-C) of the batch helpers.fullsize_batch({cfg}).
# columns: ordering index, kind, seed, footprint in bytes, first 16 hex digits of SHA-256 over the
# little-endian u64 offsets of all variables.  Lines are in order of completion.
"""


def work_order(B, kinds):
    rng = np.random.default_rng(19030663)
    first = [0, 1, 2, 3] + [int(b) for b in np.nonzero(kinds == 6)[0][:12]]
    pool = [int(b) for b in rng.permutation(B) if int(b) not in first]
    first += pool[: 64 - len(first)]
    rest = [b for b in range(B) if b not in set(first)]
    return first, rest


def one(cfg, best, b, kind, seed):
    import oracle
    from helpers import offsets_digest
    from traces import make_config
    tr = one.cache.get(cfg)
    if tr is None:
        tr = one.cache[cfg] = make_config(cfg)
    perm = oracle.make_perm(tr, kind, seed)
    off, fp = oracle.place(tr, perm, best_fit=best)
    return cfg, best, b, kind, seed, fp, offsets_digest(off)


one.cache = {}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workers", type=int, default=4)
    ap.add_argument("--jobs", nargs="*", default=["5:first", "4:first", "5:best", "4:best"])
    ap.add_argument("--limit", nargs="*", default=[], help="job=count: at most this many orderings in that file")
    ap.add_argument("--count", type=int, default=0, help="at most this many orderings in this run (0: no bound)")
    ap.add_argument("--from-the-end", action="store_true")
    args = ap.parse_args()
    import oracle
    from helpers import fullsize_batch, fullsize_golden_path, read_fullsize_golden
    oracle.build()
    limits = dict((kv.split("=")[0], int(kv.split("=")[1])) for kv in args.limit)
    phases = [[], []]
    for job in args.jobs:
        cfg, fit = int(job.split(":")[0]), job.split(":")[1]
        best = fit == "best"
        kinds, seeds = fullsize_batch(cfg)
        path = fullsize_golden_path(cfg, best)
        if not os.path.exists(path):
            with open(path, "w") as fh:
                fh.write(HEADER.format(cfg=cfg, fit=fit))
        done = read_fullsize_golden(cfg, best)
        first, rest = work_order(len(kinds), kinds)
        if args.from_the_end:
            rest = rest[::-1]
        room = limits.get(job, len(kinds)) - len(done)
        for ph, lst in enumerate((first, rest)):
            for b in lst:
                if b not in done and room > 0:
                    phases[ph].append((cfg, best, b, int(kinds[b]), int(seeds[b])))
                    room -= 1
    tasks = phases[0] + phases[1]
    if args.count:
        tasks = tasks[: args.count]
    print(f"{len(tasks)} orderings to do", flush=True)
    with ProcessPoolExecutor(args.workers) as ex:
        futs = [ex.submit(one, *t) for t in tasks]
        for k, f in enumerate(as_completed(futs)):
            cfg, best, b, kind, seed, fp, dig = f.result()
            with open(fullsize_golden_path(cfg, best), "a") as fh:
                fh.write(f"{b} {kind} {seed} {fp} {dig}\n")
            if k % 10 == 0 or args.count:
                print(f"{k + 1}/{len(tasks)} done", flush=True)


if __name__ == "__main__":
    main()
