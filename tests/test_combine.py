"""Polynomial graph filter sum_k coeff[k] A^^k X (Appendix A, Eq. 13 with constant
coefficients; K-step Personalized-PageRank diffusion as a special case): pins for
the oracle's combination on the CPU, parity of gp_propagate_combine on the GPU."""
import numpy as np
import pytest

import gp_synth
import oracle
import paper_2207_12000_amd as gp
from oracle import AGG_MEAN, AGG_SUM, AGG_SYM

BOTH = 3


def test_oracle_ppr_coefficients_equal_the_iteration():
    """The polynomial form against the defining recursion Z <- (1-a) A^ Z + a X."""
    w = gp_synth.make_workload(2, scale=0.01, d=5)
    plan = oracle.plan_blocks(w.src, w.dst, w.n, 10**9, w.flags)
    X = w.X.astype(np.float64)
    alpha, K = 0.15, 6
    Z = X.copy()
    for _ in range(K):
        Z = (1 - alpha) * oracle.hop(plan, Z, AGG_SYM) + alpha * X
    val, bnd = oracle.combine(plan, X, AGG_SYM, oracle.ppr_coefficients(alpha, K))
    assert np.all(np.abs(val - Z) <= 1e-13 * bnd + 1e-300)
    assert abs(sum(oracle.ppr_coefficients(alpha, K)) - 1.0) < 1e-15


def test_oracle_combine_closed_form_on_complete_graph():
    n = 8
    src = [i for i in range(n) for j in range(i)]
    dst = [j for i in range(n) for j in range(i)]
    plan = oracle.plan_blocks(src, dst, n, 100, BOTH)
    X = np.random.default_rng(2).standard_normal((n, 3))
    coeff = [0.5, -2.0, 0.25, 3.0]
    val, _ = oracle.combine(plan, X, AGG_SYM, coeff)
    want = coeff[0] * X + sum(coeff[1:]) * X.mean(axis=0)       # A^^k X = column means for every k >= 1
    assert np.allclose(val, want, rtol=1e-13, atol=1e-14)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [gp.GP_F32, gp.GP_BF16])
@pytest.mark.parametrize("agg,K,d,ld_pad", [(AGG_SYM, 3, 128, 0), (AGG_MEAN, 2, 100, 4), (AGG_SUM, 1, 36, 1),
                                            (AGG_SYM, 0, 7, 0), (AGG_SYM, 5, 602, 2)])
def test_gpu_combine_matches_oracle(gpu_or_skip, dtype, agg, K, d, ld_pad):
    import torch
    w = gp_synth.make_workload(2, scale=0.03, d=d)
    X = w.X if dtype == gp.GP_F32 else gp_synth.f32_to_bf16_bits(w.X)
    Xw = (w.X if dtype == gp.GP_F32 else gp_synth.bf16_bits_to_f32(X)).astype(np.float64)
    rng = np.random.default_rng(K + d)
    coeff = oracle.ppr_coefficients(0.2, K) if agg == AGG_SYM and K == 3 else rng.uniform(-1, 1, K + 1).tolist()
    tdt = torch.float32 if dtype == gp.GP_F32 else torch.bfloat16
    xt = torch.from_numpy(X) if dtype == gp.GP_F32 else torch.from_numpy(X.view(np.int16)).view(torch.bfloat16)
    xd = xt.cuda()
    ldo = d + ld_pad
    out = torch.full((w.n, ldo), float("nan"), dtype=tdt, device="cuda:0")
    op = oracle.plan_blocks(w.src, w.dst, w.n, 4000, w.flags)
    gp.gp_set_option("segment_edges", 16)                      # cut rows too: the fix-up path adds terms as well
    try:
        with gp.gp_plan_blocks(w.src, w.dst, w.n, 4000, w.flags) as lp:
            assert lp.num_partial_rows > 0
            stream = torch.cuda.current_stream().cuda_stream
            for _ in range(2):                                    # second call reuses the scratch slabs
                gp.gp_propagate_combine(lp, xd.data_ptr(), d, d, dtype, agg, K, coeff, out.data_ptr(), ldo, stream)
            torch.cuda.synchronize()
    finally:
        gp.gp_set_option("segment_edges", 0)
    got = out[:, :d].float().cpu().numpy().astype(np.float64)
    if ld_pad:
        assert torch.isnan(out[:, d:].float()).all()
    c32 = np.asarray(coeff, dtype=np.float32).astype(np.float64)  # the library takes fp32 coefficients
    want, bound = oracle.combine(op, Xw, agg, c32, threads=4)
    tol = 1e-5 if dtype == gp.GP_F32 else 1e-2
    err = np.abs(got - want)
    assert np.all(err <= tol * bound + 1e-30), f"worst ratio {np.max(err / (bound + 1e-300)):.3g}"


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,d,agg,hubs", [(gp.GP_F32, 52, AGG_SYM, False), (gp.GP_BF16, 36, AGG_SYM, False), (gp.GP_F32, 37, 1, True)])
def test_gpu_combine_with_the_lds_pass(gpu_or_skip, dtype, d, agg, hubs):
    """The filter sum where the hops take their hot non-zeros from LDS (a community graph's clusters, a
    power-law graph's hubs; forced on these small graphs): the epilogue that adds gamma_k times the hop's rows
    sits in the segment kernel, after the plane entries have joined the sums."""
    import torch
    K = 3
    w = gp_synth.make_workload(2, scale=0.2, d=d) if hubs else gp_synth.make_workload(4, scale=0.01, d=d)
    X = w.X if dtype == gp.GP_F32 else gp_synth.f32_to_bf16_bits(w.X)
    Xw = (w.X if dtype == gp.GP_F32 else gp_synth.bf16_bits_to_f32(X)).astype(np.float64)
    coeff = np.random.default_rng(d).uniform(-1, 1, K + 1).tolist()
    tdt = torch.float32 if dtype == gp.GP_F32 else torch.bfloat16
    xt = torch.from_numpy(X) if dtype == gp.GP_F32 else torch.from_numpy(X.view(np.int16)).view(torch.bfloat16)
    xd = xt.cuda()
    out = torch.full((w.n, d), float("nan"), dtype=tdt, device="cuda:0")
    budget = max(20_000, w.m // 3)
    op = oracle.plan_blocks(w.src, w.dst, w.n, budget, w.flags)
    gp.gp_set_option("segment_edges", 16)
    gp.gp_set_option("hub_pass" if hubs else "lds_pass", 1)
    gp.gp_profile_enable(True)
    try:
        with gp.gp_plan_blocks(w.src, w.dst, w.n, budget, w.flags) as lp:
            stream = torch.cuda.current_stream().cuda_stream
            gp.gp_propagate_combine(lp, xd.data_ptr(), d, d, dtype, agg, K, coeff, out.data_ptr(), d, stream)
            torch.cuda.synchronize()
        launches, _ = gp.gp_profile_read("gp_hop_cluster_lds")
    finally:
        gp.gp_profile_enable(False)
        gp.gp_set_option("segment_edges", 0)
        gp.gp_set_option("lds_pass", 0)
        gp.gp_set_option("hub_pass", 0)
    assert launches == K
    got = out.float().cpu().numpy().astype(np.float64)
    c32 = np.asarray(coeff, dtype=np.float32).astype(np.float64)
    want, bound = oracle.combine(op, Xw, agg, c32, threads=4)
    tol = 1e-5 if dtype == gp.GP_F32 else 1e-2
    err = np.abs(got - want)
    assert np.all(err <= tol * bound + 1e-30), f"worst ratio {np.max(err / (bound + 1e-300)):.3g}"


@pytest.mark.gpu
def test_gpu_combine_rejects_bad_arguments(gpu_or_skip):
    import torch
    x = torch.zeros((8, 4), device="cuda:0")
    out = torch.zeros((8, 4), device="cuda:0")
    with gp.gp_plan_blocks([0], [1], 8, 4, 3) as lp:
        with pytest.raises(gp.GpError) as e:
            gp.gp_propagate_combine(lp, x.data_ptr(), 4, 4, gp.GP_F32, 0, 1, [1.0, 1.0], x.data_ptr(), 4)
        assert e.value.status == gp.GP_ERR_INVALID_ARG           # out overlaps X
        xh = torch.zeros((8, 4)).pin_memory()
        with pytest.raises(gp.GpError) as e:
            gp.gp_propagate_combine(lp, xh.data_ptr(), 4, 4, gp.GP_F32, 0, 1, [1.0, 1.0], out.data_ptr(), 4)
        assert e.value.status == gp.GP_ERR_UNSUPPORTED
