"""gp_propagate_noalloc (the entry point for callers that cannot allocate) against
gp_propagate: the same bits, on two calls in a row, the second on a smaller input; the
size limit and the not-yet-uploaded plan are errors."""
import numpy as np
import pytest

import gp_synth
import paper_2207_12000_amd as gp

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu(gpu_or_skip):
    # the allocating call is kept to whole records: its split schedule (which needs buffers the
    # allocation-free call cannot have) would group a row's partial sums differently
    gp.gp_set_option("split_records", 2)
    yield
    gp.gp_set_option("split_records", 0)
    gp.gp_set_option("segment_edges", 0)


def tensors(w, dtype, ld_pad=0):
    import torch
    X = torch.from_numpy(w.X).cuda()
    if dtype == gp.GP_BF16:
        X = X.to(torch.bfloat16)
    return X


def both_ways(w, dtype, agg, K, budget, first_agg=None):
    """Returns (allocating result, allocation-free result) as torch tensors."""
    import torch
    X = tensors(w, dtype)
    n, d = X.shape
    with gp.gp_plan_blocks(w.src, w.dst, w.n, budget, w.flags) as plan:
        want = torch.full((K + 1, n, d), float("nan"), dtype=X.dtype, device="cuda")
        # the first allocating call uploads the plan; with another operator first, the
        # per-edge weights of the sym operator have not been built when the second call comes
        if first_agg is not None:
            gp.gp_propagate(plan, X.data_ptr(), d, d, dtype, first_agg, 1, want.data_ptr(), d, None)
            got = torch.full_like(want, float("nan"))
            gp.gp_propagate_noalloc(plan, X.data_ptr(), d, d, dtype, agg, K, got.data_ptr(), d, None)
            gp.gp_propagate(plan, X.data_ptr(), d, d, dtype, agg, K, want.data_ptr(), d, None)
        else:
            gp.gp_propagate(plan, X.data_ptr(), d, d, dtype, agg, K, want.data_ptr(), d, None)
            got = torch.full_like(want, float("nan"))
            gp.gp_propagate_noalloc(plan, X.data_ptr(), d, d, dtype, agg, K, got.data_ptr(), d, None)
        torch.cuda.synchronize()
        assert plan.num_partial_rows > 0          # the scratch is really used
    return want, got


def test_two_calls_in_a_row_second_one_smaller():
    import torch
    gp.gp_set_option("segment_edges", 16)          # many cut rows: the partial-row scratch is well filled
    big = gp_synth.make_workload(3, scale=0.01)    # 24,500 nodes, hubs cut into many partial rows, 8 blocks
    want, got = both_ways(big, gp.GP_F32, gp.GP_AGG_MEAN, 3, big.block_budget_edges // 4)
    assert torch.equal(want.view(torch.int32), got.view(torch.int32))
    small = gp_synth.make_workload(2, scale=0.02, d=36)
    want, got = both_ways(small, gp.GP_BF16, gp.GP_AGG_SYM, 2, 10_000)
    assert torch.equal(want.view(torch.int16), got.view(torch.int16))
    # sym before any allocating sym call: weights gathered by column id instead of read per edge
    want, got = both_ways(small, gp.GP_F32, gp.GP_AGG_SYM, 2, 10_000, first_agg=gp.GP_AGG_SUM)
    assert torch.equal(want.view(torch.int32), got.view(torch.int32))


def test_limit_and_unprepared_plan_are_errors():
    import torch
    w = gp_synth.make_workload(3, scale=0.01, d=512)
    X = torch.from_numpy(w.X).cuda()
    out = torch.empty((2, w.n, 512), device="cuda")
    gp.gp_set_option("segment_edges", 8)
    with gp.gp_plan_blocks(w.src, w.dst, w.n, w.block_budget_edges, w.flags) as plan:
        with pytest.raises(gp.GpError) as e:      # not on the device yet
            gp.gp_propagate_noalloc(plan, X.data_ptr(), 512, 512, gp.GP_F32, w.agg, 1, out.data_ptr(), 512, None)
        assert e.value.status == gp.GP_ERR_INVALID_ARG
        gp.gp_propagate(plan, X.data_ptr(), 512, 512, gp.GP_F32, w.agg, 1, out.data_ptr(), 512, None)
        assert plan.num_partial_rows * 512 * 4 > gp.gp_noalloc_partial_row_bytes()
        with pytest.raises(gp.GpError) as e:      # beyond the fixed scratch
            gp.gp_propagate_noalloc(plan, X.data_ptr(), 512, 512, gp.GP_F32, w.agg, 1, out.data_ptr(), 512, None)
        assert e.value.status == gp.GP_ERR_UNSUPPORTED and "bytes" in str(e.value)
        # a narrower matrix fits the same plan
        Xn = X[:, :32].contiguous()
        a = torch.empty((2, w.n, 32), device="cuda")
        b = torch.empty((2, w.n, 32), device="cuda")
        gp.gp_propagate(plan, Xn.data_ptr(), 32, 32, gp.GP_F32, w.agg, 1, a.data_ptr(), 32, None)
        gp.gp_propagate_noalloc(plan, Xn.data_ptr(), 32, 32, gp.GP_F32, w.agg, 1, b.data_ptr(), 32, None)
        torch.cuda.synchronize()
        assert torch.equal(a, b)


def test_the_lds_pass_is_taken_over_from_an_allocating_call():
    """What an allocating call has built for the LDS pass (schedule, planes) serves the allocation-free call too:
    the same launches, the same bits."""
    import torch
    gp.gp_set_option("split_records", 0)
    gp.gp_set_option("lds_pass", 1)
    try:
        w = gp_synth.make_workload(4, scale=0.01, d=52)
        gp.gp_set_option("segment_edges", 16)
        gp.gp_profile_enable(True)
        want, got = both_ways(w, gp.GP_F32, gp.GP_AGG_SYM, 2, max(20_000, w.m // 3))
        launches, _ = gp.gp_profile_read("gp_hop_cluster_lds")
        assert launches == 4, f"{launches} LDS launches, expected two per call"
        assert torch.equal(want.view(torch.int32), got.view(torch.int32))
    finally:
        gp.gp_profile_enable(False)
        gp.gp_set_option("lds_pass", 0)
        gp.gp_set_option("split_records", 2)
