"""lap_load_profile_static (the entry point that allocates nothing: its scratch is a fixed array
inside the library) against lap_load_profile, through the C ABI, bit for bit; two calls in a row on
the same GPU array, the second with a smaller input, so stale scratch contents would show."""
import ctypes as C

import numpy as np
import pytest

from gpu_util import u64
from traces import make_config, random_trace, tile_in_time

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lap():
    import paper_1903_06631_amd as lap
    lap.load_library()
    return lap


def _same(lap, tr):
    import torch
    dt = lap.DeviceTrace(tr)
    ref = lap.load_profile(dt)
    before = torch.cuda.memory_allocated()
    # raw C ABI: outputs preallocated, no workspace argument at all
    load = torch.full((tr.n_steps,), -1, dtype=torch.int64, device=dt.device)
    peak = torch.full((1,), -1, dtype=torch.int64, device=dt.device)
    tpk = torch.full((1,), -1, dtype=torch.int32, device=dt.device)
    held = torch.cuda.memory_allocated()
    lib = lap.load_library()
    c = dt.c_struct()
    rc = lib.lap_load_profile_static(C.byref(c), load.data_ptr(), peak.data_ptr(), tpk.data_ptr(),
                                     int(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == held and held >= before      # torch's allocator was not touched
    assert np.array_equal(u64(load), u64(ref["load"]))
    assert int(u64(peak)[0]) == int(u64(ref["peak"])[0]) and int(tpk.item()) == int(ref["t_peak"].item())
    # and through the binding
    got = lap.load_profile_static(dt)
    assert np.array_equal(u64(got["load"]), u64(ref["load"]))
    return u64(ref["load"])


def test_static_scratch_two_calls_in_a_row_second_smaller(lap, oracle_mod):
    big = tile_in_time(make_config(5), 70)             # 40 600 steps: the tiled scan, 14 M variables
    small = random_trace(77, 5000, 333)                # single-workgroup scan, LDS bins
    tiny = random_trace(78, 3, 2)
    l_big = _same(lap, big)
    l_small = _same(lap, small)                        # smaller than the call before: stale bins must not leak
    l_tiny = _same(lap, tiny)
    _same(lap, big)                                    # and larger again
    # the reference itself is the oracle's
    assert np.array_equal(l_small, oracle_mod.load_profile(small)[0])
    assert np.array_equal(l_tiny, oracle_mod.load_profile(tiny)[0])
    assert np.array_equal(l_big[:580], oracle_mod.load_profile(make_config(5))[0])


def test_static_scratch_limits(lap):
    import torch
    from paper_1903_06631_amd.binding import STATIC_MAX_STEPS, _Trace
    lib = lap.load_library()
    out = torch.zeros(4, dtype=torch.int64, device="cuda")
    fake = out.data_ptr()
    too_long = _Trace(4, STATIC_MAX_STEPS + 1, fake, fake, fake, None, None, None)
    assert lib.lap_load_profile_static(C.byref(too_long), fake, fake, fake, None) == -2       # rejected, nothing enqueued
    assert lib.lap_load_profile_static(None, fake, fake, fake, None) == -1
    # the largest supported time line works
    tr = random_trace(5, 2000, 1000)
    tr.n_steps = STATIC_MAX_STEPS
    dt = lap.DeviceTrace(tr)
    a, b = lap.load_profile_static(dt), lap.load_profile(dt)
    assert np.array_equal(u64(a["load"]), u64(b["load"])) and int(a["t_peak"].item()) == int(b["t_peak"].item())
