#!/usr/bin/env python3
"""Benchmark of the lifetime-aware pool planner's hot path on one MI355X.

One step = one pass of the whole path over one synthetic trace resident in HBM:
lap_load_profile, lap_plan_pool over B orderings, lap_score_swaps.  The headline
value is variable placements per second (B*N / step time).  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBPS = 8000.0     # MI355X HBM3E, published peak


def count_edges(tr) -> int:
    """|E| of the interval graph (pairs of variables alive together): all pairs minus the pairs
    where one is freed no later than the other is allocated.  A work measure of the input."""
    n = tr.n_vars
    fs = np.sort(tr.free.astype(np.int64))
    disjoint = int(np.searchsorted(fs, tr.alloc.astype(np.int64), side="right").sum())
    return n * (n - 1) // 2 - disjoint


def source_stamp(*names) -> str:
    """16 hex digits of SHA-256 over the code of the named kernel sources (comments and blank space
    left out): a counter summary under profiles/ is only used while the kernel it was measured on is
    the one in the tree."""
    import hashlib
    import re
    h = hashlib.sha256()
    for nm in names:
        with open(os.path.join(ROOT, "paper_1903_06631_amd", "csrc", nm)) as fh:
            text = re.sub(r"/\*.*?\*/", "", fh.read(), flags=re.S)
        for ln in text.split("\n"):
            ln = " ".join(ln.split("//")[0].split())
            if ln:
                h.update(ln.encode() + b"\n")
    return h.hexdigest()[:16]


def read_profile_values(path):
    """'key: value' lines of a text summary under profiles/ (comments and tables are skipped)."""
    import re
    vals = {}
    if os.path.exists(path):
        for ln in open(path):
            m = re.match(r"^([A-Za-z_0-9]+):\s*(\S+)\s*$", ln)
            if m:
                vals[m.group(1)] = m.group(2)
    return vals


# dominant placement kernel of every benchmark configuration: its name, the sources it is built
# from, and the stem of its counter summaries under profiles/
PLACE_KERNEL = {
    5: ("k_place_fast<u32,false>", ("place_fast.hip", "lap_dev.h"), "k_place_fast_transformer_B1024"),
    4: ("k_place_seg", ("place_seg.hip", "seg_core.h", "lap_dev.h"), "k_place_seg_deepchain_B4096"),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5 (5 = transformer-shaped, the largest trace)")
    ap.add_argument("--orderings", type=int, default=0, help="override B (0 = the config's own)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stress", action="store_true",
                    help="skip the load-profile run on the 2 GiB time-tiled trace")
    ap.add_argument("--no-extras", action="store_true", help="skip the best-fit and selection legs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build plans on ONE GPU (the orderings are what would shard across GPUs); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_1903_06631_amd as lap
    from traces import CONFIG_NAMES, make_config, make_orderings

    lap.load_library()
    dev = torch.device("cuda:0")
    tr = make_config(args.config)
    B = args.orderings or tr.meta["B"]
    kinds, seeds = make_orderings(B)
    n, T = tr.n_vars, tr.n_steps
    n_edges = count_edges(tr)

    t0 = time.perf_counter()
    dt = lap.DeviceTrace(tr, dev)
    torch.cuda.synchronize()
    upload_s = time.perf_counter() - t0
    assert lap.validate_trace(dt) == 0

    # a plain device-to-device copy of 1 GiB, timed in this run: what this GPU's memory system gives
    # a kernel that does nothing but stream (and the kernel rocprofv3's FETCH_SIZE / WRITE_SIZE
    # readings are scaled by)
    src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    copy_ms = []
    for _ in range(5):
        ev0.record()
        dst.copy_(src)
        ev1.record()
        torch.cuda.synchronize()
        copy_ms.append(ev0.elapsed_time(ev1))
    copy_GBps = 2 * src.numel() * 4 / (float(np.median(copy_ms)) * 1e-3) / 1e9      # bytes read + bytes written
    del src, dst

    out = None
    lap.profile_enable(True)

    def step():
        nonlocal out
        lp = lap.load_profile(dt, sync=False)
        out = lap.plan_pool(dt, kinds, seeds, want_all=False, sync=False, out=out)
        sc = lap.score_swaps(dt, tr.meta["link_GBps"], tr.meta["min_bytes"], load=lp["load"], sync=False)
        return lp, sc

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    place_ms, sort_ms = [], []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        lp, sc = step()
        # the kernel's own duration, from HIP events recorded on the launch stream
        torch.cuda.synchronize()
        place_ms.append(lap.profile_last_ms(lap.K_PLACE))
        sort_ms.append(lap.profile_last_ms(lap.K_SORT))
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    ord_ms = lap.profile_ordering_ms(dt, B)          # how long the last launch worked on each ordering
    ms_per_step = 1e3 * total_s / args.steps
    value = B * n * args.steps / total_s

    u64 = lambda t: t.cpu().numpy().view(np.uint64)
    peak = int(u64(lp["peak"])[0])
    best_fp = int(u64(out["best_footprint"])[0])
    fps = u64(out["footprints"])

    # Dominant kernel: placement.  Its duration is measured here (HIP events on the launch stream);
    # the HBM bytes it moves per launch come from rocprofv3 FETCH_SIZE + WRITE_SIZE runs of this same
    # command, kept under profiles/ with a stamp of the kernel source: if the source has changed
    # since, the bytes are not used and achieved / frac are null.
    k_ms = float(np.mean(place_ms))
    k_name, k_src, k_stem = PLACE_KERNEL.get(args.config, ("k_place_*", ("place_fast.hip", "lap_dev.h"), None))
    traffic, counters = None, {}
    if k_stem and B == tr.meta["B"]:
        tv = read_profile_values(os.path.join(ROOT, "profiles", k_stem + "_hbm_traffic.txt"))
        if tv.get("source_sha256_16") == source_stamp(*k_src) and "traffic_bytes_per_launch" in tv:
            traffic = int(tv["traffic_bytes_per_launch"])
            cv = read_profile_values(os.path.join(ROOT, "profiles", k_stem + "_sq_counters.txt"))
            if cv.get("source_sha256_16") == source_stamp(*k_src):
                counters = {k: float(v) for k, v in cv.items() if k not in ("source_sha256_16",)}
    achieved = traffic / (k_ms * 1e-3) / 1e9 if traffic else None
    # the pair-by-pair model: every time-overlapping pair examined once per ordering (16 B: the earlier
    # block's offset and end) plus 24 B per variable.  Not a bound for this kernel: per-step hole lists
    # summarise the one-step neighbours, so it moves fewer bytes than that.
    pair_bytes = B * (16 * n_edges + 24 * n)
    roofline = dict(bound="hbm", kernel=k_name, achieved=achieved, peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBPS if achieved else None, traffic=traffic, kernel_ms=k_ms,
                    limited_by="the dependent memory accesses of one placement (latency and number of scattered "
                               "requests, see counters), not HBM bandwidth",
                    counters=counters or None, copy_GBps=copy_GBps,
                    # the launch ends with its slowest ordering
                    ordering_ms=dict(min=float(ord_ms.min()), median=float(np.median(ord_ms)), mean=float(ord_ms.mean()),
                                     p90=float(np.percentile(ord_ms, 90)), max=float(ord_ms.max()),
                                     slowest=int(ord_ms.argmax()), fixed_orders=[float(x) for x in ord_ms[:4]]),
                    frac_of_copy=achieved / copy_GBps if achieved else None,
                    sort_kernel_ms=float(np.mean(sort_ms)),
                    pairwise_model=dict(bytes=pair_bytes, GBps=pair_bytes / (k_ms * 1e-3) / 1e9,
                                        over_hbm_peak=pair_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                        note="not a bound and not a roofline fraction: bytes a kernel that reads "
                                             "every overlapping pair would move, over this kernel's time"),
                    note="achieved = HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (profiles/, "
                         "stamped with the kernel source) / kernel duration measured in this run")

    # The oracle (plain single-threaded C, as it stands) on this machine's host cores, after the timed region.
    # Leg 1, one thread: the ordering the timed run found best, all N variables -- the paper's planner is
    # a single-threaded host program that runs one ordering (Section III-C, VI-A).  Leg 2, every hardware
    # thread this process may use: one ordering per thread.  Both are compared with the TIMED outputs.
    cpu = None
    if not args.no_cpu_baseline:
        print("bench.py: timed region done; oracle legs on the host cores ...", file=sys.stderr, flush=True)
        import oracle
        from concurrent.futures import ThreadPoolExecutor
        oracle.build()
        best_b = int(out["best_ordering"].item())
        perm = oracle.make_perm(tr, int(kinds[best_b]), int(seeds[best_b]))
        c0 = time.perf_counter()
        o_off, o_fp = oracle.place(tr, perm)
        c_s = time.perf_counter() - c0
        assert np.array_equal(u64(out["best_offsets"]), o_off), "timed GPU offsets differ from the oracle"
        assert int(fps[best_b]) == o_fp == best_fp
        cores = max(1, min(16, len(os.sched_getaffinity(0))))
        nb = B if c_s * B / cores < 20.0 else cores          # all orderings when that takes seconds, else one per thread
        which = list(range(B)) if nb == B else [4 + i for i in range(cores)] if B >= 4 + cores else list(range(nb))

        def one(b):
            pm = oracle.make_perm(tr, int(kinds[b]), int(seeds[b]))
            return b, oracle.place(tr, pm)                   # ctypes releases the GIL during the call

        c0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            res = list(ex.map(one, which))
        m_s = time.perf_counter() - c0
        chk = lap.plan_pool(dt, [kinds[b] for b in which], [seeds[b] for b in which], want_all=True)
        chk_off = u64(chk["all_offsets"])
        for i, (b, (off_b, fp_b)) in enumerate(res):
            assert int(fps[b]) == fp_b, f"timed footprint of ordering {b} differs from the oracle"
            assert np.array_equal(chk_off[i], off_b), f"GPU offsets of ordering {b} differ from the oracle"
        cpu = dict(value=len(which) * n / m_s, unit="placements/s", cores=cores, kind="oracle",
                   sample=f"first-fit placement of {len(which)} of the {B} orderings "
                          f"({'all' if nb == B else 'the seeded orderings ' + str(which[0]) + '..' + str(which[-1])}), "
                          f"all {n} variables each, one ordering per thread on {cores} threads, {m_s:.1f} s",
                   full_batch_s_extrapolated=B * n / (len(which) * n / m_s),
                   extrapolation="linear in the number of orderings (they are independent)",
                   pair_tests_per_s=len(which) * n_edges / m_s,
                   single_thread=dict(value=n / c_s, unit="placements/s", cores=1,
                                      sample=f"first-fit placement of ordering {best_b} (the best of the timed run: "
                                             f"kind {int(kinds[best_b])}), all {n} variables, {c_s:.1f} s",
                                      pair_tests_per_s=n_edges / c_s))

    # The same step captured in a HIP graph and replayed (no per-kernel events inside a graph, so this leg
    # has no kernel times): what the launch overhead of the ~25 small kernels of a step costs.  Not `value`.
    graph_ms = None
    if not args.no_extras:
        print("bench.py: graph replay, then the rows beyond the timed path ...", file=sys.stderr, flush=True)
        lap.profile_enable(False)
        lap.load_profile(dt); lap.plan_pool(dt, kinds, seeds, want_all=False); torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                glp = lap.load_profile(dt, sync=False)
                gpp = lap.plan_pool(dt, kinds, seeds, want_all=False, sync=False)
                lap.score_swaps(dt, tr.meta["link_GBps"], tr.meta["min_bytes"], load=glp["load"], sync=False)
        torch.cuda.current_stream().wait_stream(side)
        g.replay(); torch.cuda.synchronize()
        reps = max(2, min(args.steps, 5))
        c0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = 1e3 * (time.perf_counter() - c0) / reps
        assert torch.equal(gpp["best_offsets"], out["best_offsets"]) and torch.equal(gpp["footprints"], out["footprints"])
        del g, glp, gpp
        lap.profile_enable(True)

    # The rows built beyond the timed path (never part of `value`): the same orderings planned
    # best-fit, and the selection walk for all five priority scores down to a sweep of limits.
    extra = None
    if not args.no_extras:
        # best-fit looks at every hole that fits: on the dense residual-chain trace that is thousands per
        # variable and minutes per ordering, so that configuration leaves this leg out
        dense = int((tr.free.astype(np.int64) - tr.alloc).sum()) > 64 * n
        bf = None
        if not dense:
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            bf = lap.plan_pool(dt, kinds, seeds, want_all=False, fits=[1] * B)
            bf_s = time.perf_counter() - c0
            bf_ms = lap.profile_last_ms(lap.K_PLACE)
            bfps = u64(bf["footprints"])
        limits = [peak * q // 20 for q in range(21)]
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        sel = lap.select_swaps(dt, tr.meta["link_GBps"], tr.meta["min_bytes"], [0, 1, 2, 3, 4], limits,
                               load=lp["load"])
        sel_s = time.perf_counter() - c0
        extra = dict(best_fit=None if bf is None else dict(
                         call_ms=1e3 * bf_s, kernel_ms=bf_ms, placements_per_s=B * n / bf_s,
                         footprint_over_peak=int(u64(bf["best_footprint"])[0]) / peak,
                         footprint_over_peak_fixed_orders=[float(x) / peak for x in bfps[:4]],
                         mean_footprint_over_first_fit=float(np.mean(bfps.astype(np.float64) / fps.astype(np.float64)))),
                     select_swaps=dict(call_ms=1e3 * sel_s, kernel_ms=lap.profile_last_ms(lap.K_SELECT),
                                       score_kinds=5, limits=len(limits), candidates=int(sel["n_cand"].item()),
                                       load_min_over_peak=int(u64(sel["load_min"])[0]) / peak,
                                       lowest_peak_over_peak=int(u64(sel["peak_after"])[3, 0]) / peak))
        # the swap plan for what the selection picked at 60 % of the peak, and that plan replayed
        # under every limit of the sweep (SWDOA order)
        row = 3
        nsel = sel["n_selected"].cpu().numpy().view(np.uint32)[row]
        order = sel["order"][row].contiguous()
        k60 = int(nsel[12])
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        plan = lap.schedule_swaps(dt, tr.meta["link_GBps"], order[:k60].contiguous(), load=lp["load"])
        plan_s = time.perf_counter() - c0
        c0 = time.perf_counter()
        sim = lap.simulate_swaps(dt, tr.meta["link_GBps"], order[:int(nsel.max())].contiguous(),
                                 [int(x) for x in nsel], limits)
        sim_s = time.perf_counter() - c0
        ovh = u64(sim["overhead_ns"]).astype(np.float64) / float(u64(sim["total_ns"])[-1])
        extra["schedule_swaps"] = dict(call_ms=1e3 * plan_s, swapped=k60, limit_over_peak=0.6,
                                       peak_under_plan_over_peak=int(u64(plan["peak"])[0]) / peak,
                                       late_ns=int(u64(plan["late_ns"])[0]))
        extra["simulate_swaps"] = dict(call_ms=1e3 * sim_s, runs=len(limits),
                                       overhead_over_iteration_by_limit={f"{q * 5}%": round(float(ovh[q]), 4)
                                                                         for q in range(6, 21, 2)},
                                       forced_at_60pct=int(sim["forced"].cpu().numpy().view(np.uint32)[12]))
        # iteration detection on a request stream of two iterations of this trace after a warm-up
        from traces.requests import iteration_tokens, request_stream
        it = iteration_tokens(tr)
        stream = request_stream(it, 2, 1000, 0, seed=1)
        tok = torch.from_numpy(stream.view(np.int64)).to(dev)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        per = lap.detect_iteration(tok, 64)
        det_s = time.perf_counter() - c0
        assert int(per.item()) == len(it)
        extra["detect_iteration"] = dict(call_ms=1e3 * det_s, requests=len(stream), period=len(it))
        lap.plan_pool(dt, kinds[:1], seeds[:1], want_all=False)      # leave the profile slots on first-fit

    # The load-profile kernel on the largest benchmark trace moves 3.2 MB (launch-latency bound), so
    # its HBM fraction is also measured on the same trace repeated along time until the SoA is ~2 GiB.
    lp_small_ms = lap.profile_last_ms(lap.K_LOAD_SCATTER)
    stress = None
    if not args.no_stress:
        print("bench.py: load profile on the time-tiled stress trace ...", file=sys.stderr, flush=True)
        from traces import tile_in_time
        big = tile_in_time(tr, 670)
        bdt = lap.DeviceTrace(big, dev, use_gaps=False)
        ms_k, ms_call = [], []
        for it in range(6):
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            blp = lap.load_profile(bdt)
            ms_call.append(1e3 * (time.perf_counter() - c0))
            ms_k.append(lap.profile_last_ms(lap.K_LOAD_SCATTER))
        nbytes = 16 * big.n_vars + 8 * big.n_steps
        k_ms, call_ms = float(np.median(ms_k[1:])), float(np.median(ms_call[1:]))
        # same curve every iteration: the tiled profile repeats the single-iteration one
        assert np.array_equal(u64(blp["load"])[:T], u64(lp["load"])) and int(u64(blp["peak"])[0]) == peak
        stress = dict(workload="configs[4] repeated 670x along time (not one of the benchmark configurations)", n_vars=big.n_vars,
                      n_steps=big.n_steps, algorithmic_bytes=nbytes, kernel="k_delta_window", kernel_ms=k_ms,
                      kernel_GBps=nbytes / k_ms / 1e6, kernel_frac=nbytes / k_ms / 1e6 / HBM_PEAK_GBPS,
                      call_ms=call_ms, call_GBps=nbytes / call_ms / 1e6, call_frac=nbytes / call_ms / 1e6 / HBM_PEAK_GBPS)
        del bdt, blp

    line = {
        "metric": "variable placements/sec across B orderings; footprint / peak-live-bytes ratio",
        "value": value, "unit": "placements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32/u64 integer (AOA: f64)", "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}] {CONFIG_NAMES[args.config]}-shaped trace",
                   "n_vars": n, "n_steps": T, "orderings": B, "edges": n_edges,
                   "link_GBps": tr.meta["link_GBps"], "trace_bytes": dt.nbytes(), "upload_ms": 1e3 * upload_s},
        "pair_tests_per_s": B * n_edges * args.steps / total_s,
        "footprint_over_peak": best_fp / peak, "best_ordering": int(out["best_ordering"].item()),
        "footprint_over_peak_fixed_orders": [float(x) / peak for x in fps[:4]],
        "roofline": roofline, "cpu_baseline": cpu, "graph_replay_ms_per_step": graph_ms,
        "beyond_the_timed_path": extra,
        "load_profile": {"kernel_ms_on_workload": lp_small_ms, "stress": stress},
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
