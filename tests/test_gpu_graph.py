"""gp_propagate enqueues only kernels on the caller's stream once a plan has been
used (no allocation, no memset, no synchronisation), so a caller can capture it
in a HIP graph.  Replays are checked against eager runs, with other work and
synchronisations in between and fresh input contents each time."""
import numpy as np
import pytest

import gp_synth
import paper_2207_12000_amd as gp

pytestmark = pytest.mark.gpu


def test_capture_and_replay(gpu_or_skip):
    import torch
    w = gp_synth.make_workload(1, scale=0.3)
    n, d, K = w.n, w.d, w.K
    with gp.gp_plan_blocks(w.src, w.dst, n, 5000, w.flags) as lp:
        assert lp.num_partial_rows > 0
        x = torch.from_numpy(w.X).cuda()
        out = torch.zeros((K + 1, n, d), device="cuda:0")
        ref = torch.zeros_like(out)
        # first call outside the capture: uploads the plan and sizes the scratch
        gp.propagate_tensors(lp, x, w.agg, K, out=ref)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(g, stream=side):
            gp.gp_propagate(lp, x.data_ptr(), d, d, gp.GP_F32, w.agg, K, out.data_ptr(), d,
                            torch.cuda.current_stream().cuda_stream)
        for rep in range(4):
            x.copy_(torch.from_numpy(gp_synth.features(n, d, "normal", gp_synth.rng_for(99, rep))))
            out.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            gp.propagate_tensors(lp, x, w.agg, K, out=ref)       # eager, same inputs
            torch.cuda.synchronize()
            assert torch.equal(out, ref), f"replay {rep} differs from the eager result"


@pytest.mark.parametrize("kind", ["clusters", "hubs"])
def test_capture_and_replay_with_the_lds_pass(gpu_or_skip, kind):
    """The same with the LDS pass in the hop (its schedule, planes and the kernel's LDS clearance are set up by
    the first call; the captured call launches kernels only)."""
    import torch
    try:
        if kind == "clusters":
            w = gp_synth.make_workload(4, scale=0.01, d=52)
            gp.gp_set_option("lds_pass", 1)
        else:
            w = gp_synth.make_workload(2, scale=0.2, d=36)
            gp.gp_set_option("hub_pass", 1)
        n, d, K = w.n, w.d, 2
        with gp.gp_plan_blocks(w.src, w.dst, n, max(20_000, w.m // 3), w.flags) as lp:
            x = torch.from_numpy(w.X).cuda()
            out = torch.zeros((K + 1, n, d), device="cuda:0")
            ref = torch.zeros_like(out)
            gp.gp_profile_enable(True)
            gp.propagate_tensors(lp, x, w.agg, K, out=ref)
            torch.cuda.synchronize()
            launches, _ = gp.gp_profile_read("gp_hop_cluster_lds")
            gp.gp_profile_enable(False)
            assert launches == K
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.graph(g, stream=side):
                gp.gp_propagate(lp, x.data_ptr(), d, d, gp.GP_F32, w.agg, K, out.data_ptr(), d,
                                torch.cuda.current_stream().cuda_stream)
            for rep in range(3):
                x.copy_(torch.from_numpy(gp_synth.features(n, d, "normal", gp_synth.rng_for(98, rep))))
                out.fill_(float("nan"))
                g.replay()
                torch.cuda.synchronize()
                gp.propagate_tensors(lp, x, w.agg, K, out=ref)
                torch.cuda.synchronize()
                assert torch.equal(out, ref), f"replay {rep} differs from the eager result"
    finally:
        gp.gp_set_option("lds_pass", 0)
        gp.gp_set_option("hub_pass", 0)
