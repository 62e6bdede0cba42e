"""The counter summaries bench.py reads from profiles/ belong to the kernel sources in the tree: a
summary measured on an older kernel must not reach a benchmark record unnoticed."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_traffic_summaries_match_the_kernel_sources():
    bench = _bench()
    for cfg, (kernel, sources, stem) in bench.PLACE_KERNEL.items():
        tv = bench.read_profile_values(os.path.join(ROOT, "profiles", stem + "_hbm_traffic.txt"))
        assert tv, f"no traffic summary for configuration {cfg} ({stem})"
        assert tv.get("source_sha256_16") == bench.source_stamp(*sources), \
            f"profiles/{stem}_hbm_traffic.txt was measured on other sources than {sources}: measure again"
        assert int(tv["traffic_bytes_per_launch"]) > 0
        cv = bench.read_profile_values(os.path.join(ROOT, "profiles", stem + "_sq_counters.txt"))
        assert cv.get("source_sha256_16") == tv["source_sha256_16"]
        assert 0.0 <= float(cv["valu_busy_pct"]) <= 100.0


def test_every_stamped_summary_matches_the_kernel_sources():
    """also the summaries bench.py does not read (the best-fit kernel's): a stamp names the sources of the
    kernel family the file is named for"""
    bench = _bench()
    families = {"k_place_fast": ("place_fast.hip", "lap_dev.h"), "k_place_seg": ("place_seg.hip", "seg_core.h", "lap_dev.h")}
    seen = 0
    for name in sorted(os.listdir(os.path.join(ROOT, "profiles"))):
        tv = bench.read_profile_values(os.path.join(ROOT, "profiles", name))
        if "source_sha256_16" not in tv:
            continue
        fam = [f for f in families if name.startswith(f)]
        assert fam, f"profiles/{name} carries a stamp but no known kernel family"
        assert tv["source_sha256_16"] == bench.source_stamp(*families[fam[0]]), f"profiles/{name}: measure again"
        seen += 1
    assert seen >= 6


def test_profiles_hold_text_summaries_only():
    for name in os.listdir(os.path.join(ROOT, "profiles")):
        assert name.endswith((".txt", ".md")), name
        assert os.path.getsize(os.path.join(ROOT, "profiles", name)) < 64 * 1024
