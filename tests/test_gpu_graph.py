"""The calls enqueue kernels only (small host arrays travel in kernel arguments, scratch is cleared by fill
kernels, nothing waits), so a whole planning pass can be captured in a HIP graph.  The graph is replayed
several times, with the program's own eager work and synchronisations between the replays, and every replay
is compared with the eager result and with the oracle."""
import numpy as np
import pytest

from gpu_util import u64
from traces import make_config, make_orderings

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lap():
    import paper_1903_06631_amd as lap
    lap.load_library()
    return lap


@pytest.mark.parametrize("cfg", [1, 2])
def test_planning_pass_in_a_graph(lap, oracle_mod, cfg):
    import torch
    tr = make_config(cfg)
    kinds, seeds = make_orderings(tr.meta["B"])
    fits = [b % 2 for b in range(len(kinds))]                    # both placement policies in the pass
    dt = lap.DeviceTrace(tr)
    link, mb = tr.meta["link_GBps"], tr.meta["min_bytes"]
    lap.profile_enable(False)                                    # (event records do not belong in a graph)

    eager_lp = lap.load_profile(dt)
    eager_pp = lap.plan_pool(dt, kinds, seeds, fits=fits)
    eager_sc = lap.score_swaps(dt, link, mb, load=eager_lp["load"])
    lap.load_profile_static(dt)                                  # its address look-up happens outside the capture
    want = {k: v.clone() for k, v in {**eager_lp, **{"pp_" + k: v for k, v in eager_pp.items()},
                                      **{"sc_" + k: v for k, v in eager_sc.items()}}.items()}

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            g_lp = lap.load_profile(dt, sync=False)
            g_ls = lap.load_profile_static(dt, sync=False)
            g_pp = lap.plan_pool(dt, kinds, seeds, fits=fits, sync=False)
            g_sc = lap.score_swaps(dt, link, mb, load=g_lp["load"], sync=False)
    torch.cuda.current_stream().wait_stream(side)
    got = {**g_lp, **{"pp_" + k: v for k, v in g_pp.items()}, **{"sc_" + k: v for k, v in g_sc.items()}}

    for replay in range(4):
        for v in got.values():
            v.zero_()                                            # a replay has to write everything again
        g_ls["load"].zero_()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in want.items():
            assert torch.equal(got[k].view(torch.uint8), v.view(torch.uint8)), (replay, k)
        assert torch.equal(g_ls["load"], want["load"])
        # eager work of the program itself between the replays, on the same workspaces
        again = lap.plan_pool(dt, kinds[::-1].copy(), seeds[::-1].copy())
        assert int(u64(again["best_footprint"])[0]) > 0
        torch.cuda.synchronize()

    ref = oracle_mod.plan_pool(tr, kinds[::2], seeds[::2])       # the first-fit half, against the oracle
    assert np.array_equal(u64(got["pp_all_offsets"])[::2], ref["all_offsets"])
