"""Host logic of the segment-list placement (csrc/seg_core.h: list search, carving, the geometry of
segments and list ids): the header is compiled with g++ and its address / undefined-behaviour
sanitizers and driven sequentially, against a bitmap brute force and against the oracle's first fit.
The HIP kernel calls the same functions, one list per thread."""
import ctypes as C
import os
import subprocess
import sys

import numpy as np
import pytest

from traces import make_config, make_orderings, random_trace

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def host(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("seg") / "libseg_host.so")
    # the sanitizer runtimes are linked statically so that the library loads into an unsanitized python
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-shared", "-fPIC", "-fsanitize=undefined", "-fno-sanitize-recover=all",
           "-static-libubsan", "-D_GLIBCXX_ASSERTIONS", "-o", out, os.path.join(ROOT, "tests", "seg_core_host.cpp")]
    subprocess.check_call(cmd)
    lib = C.CDLL(out)
    lib.seg_host_unit.restype = C.c_int
    lib.seg_host_unit.argtypes = [C.c_uint32] * 4
    lib.seg_host_place.restype = C.c_int
    lib.seg_host_place.argtypes = [C.c_uint32, C.c_uint32] + [C.c_void_p] * 4 + [C.c_uint32] + [C.c_void_p] * 3
    return lib


def test_list_primitives_against_a_bitmap(host):
    assert host.seg_host_unit(1, 4000, 12, 200) == 0           # short lists, every case of carving
    assert host.seg_host_unit(2, 300, 400, 5000) == 0          # hundreds of holes: the doubling searches
    assert host.seg_host_unit(3, 2000, 3, 9) == 0              # tiny address space: ranges that touch


def _place(host, tr, perm, shift):
    orv = int(np.bitwise_or.reduce(tr.size))
    gsh = (orv & -orv).bit_length() - 1
    size = (tr.size >> np.uint64(gsh)).astype(np.uint32)
    alloc, free_ = tr.alloc.astype(np.uint32), tr.free.astype(np.uint32)
    perm = np.ascontiguousarray(perm, np.uint32)
    off = np.zeros(tr.n_vars, np.uint32)
    pool, rounds = C.c_uint64(0), C.c_uint64(0)
    rc = host.seg_host_place(tr.n_vars, tr.n_steps, size.ctypes.data, alloc.ctypes.data, free_.ctypes.data,
                             perm.ctypes.data, shift, off.ctypes.data, C.addressof(pool), C.addressof(rounds))
    assert rc == 0, rc
    return off.astype(np.uint64) << np.uint64(gsh), pool.value, rounds.value / tr.n_vars


@pytest.mark.parametrize("seed,n,T", [(0, 1, 1), (1, 40, 3), (2, 300, 4), (3, 301, 5), (4, 700, 17), (5, 900, 64),
                                      (6, 1200, 129), (7, 1500, 1000), (8, 600, 4097)])
def test_placement_with_segment_lists_equals_the_oracle(host, oracle_mod, seed, n, T):
    """Every segment width from 4 steps up, ragged last segments, fewer steps than a segment, whole-time-line
    variables: the offsets are the oracle's first fit."""
    tr = random_trace(7000 + seed, n, T, size_choices=[1, 1, 2, 3, 5, 8, 13, 64], one_step_frac=0.3)
    if n > 10:
        tr.alloc[:n // 10], tr.free[:n // 10] = 0, T               # some live through the whole time line
        tr.gap_lo, tr.gap_hi = tr.alloc.copy(), (tr.free - 1).astype(np.uint32)
    kinds, seeds = make_orderings(6)
    for b in (0, 1, 3, 4, 5):
        perm = oracle_mod.make_perm(tr, int(kinds[b]), int(seeds[b]))
        want, _ = oracle_mod.place(tr, perm)
        for shift in (2, 3, 5, 7, 10):
            got, _, _ = _place(host, tr, perm, shift)
            assert np.array_equal(got, want), (b, shift)


def test_configuration_3_and_the_room_of_the_lists(host, oracle_mod):
    """The lists need the number of entries the library's width choice counts (blocks entered + one per
    list), and a training-shaped trace converges in about three rounds per variable."""
    tr = make_config(3)
    kinds, seeds = make_orderings(8)
    perm = oracle_mod.make_perm(tr, int(kinds[4]), int(seeds[4]))
    want, _ = oracle_mod.place(tr, perm)
    a, f, T = tr.alloc.astype(np.int64), tr.free.astype(np.int64), tr.n_steps
    for shift in (3, 4, 5, 6):
        got, pool, rounds = _place(host, tr, perm, shift)
        assert np.array_equal(got, want)
        w = 1 << shift
        K = (T + w - 1) >> shift
        k0, k1 = a >> shift, (f - 1) >> shift
        kf0, kf1 = (a + w - 1) >> shift, np.where(f == T, K, f >> shift)
        nf = np.maximum(kf1 - kf0, 0)
        steps = (f - a) - np.where(nf > 0, np.minimum(kf1 << shift, T) - (kf0 << shift), 0)
        assert pool == int((1 + (k1 - k0 + 1) + nf + steps).sum()) + 2 * K + T + 1     # the formula of k_plan_prep1 / k_plan_prep2
        assert rounds < 4.0
