"""Builds liblap.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "liblap.so")
OBJ_DIR = os.path.join(_HERE, "_build")
SOURCES = ["api.hip", "load_profile.hip", "orderings.hip", "place_fast.hip", "place_wide.hip", "place_seg.hip",
           "swap_scores.hip", "select_swaps.hip", "detect_iteration.hip",
           "schedule_swaps.hip", "simulate_swaps.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Wall", "-Wno-unused-function",
    "-ffp-contract=off",                                        # AOA is one IEEE binary64 operation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(verbose: bool = False) -> str:
    """Every source is compiled (each time: no up-to-date check), up to 8 at once, then linked."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    sources = list(SOURCES)

    def one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, "-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        text = "\n".join(ln for ln in r.stdout.splitlines() if "packed-fp32-ops" not in ln)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{text}")
        if text.strip() and verbose:
            print(text)
        return obj

    with ThreadPoolExecutor(min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(one, sources))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
