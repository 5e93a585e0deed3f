"""Parity of the HIP path (through the C ABI) with the fp64 oracle on the same
seeded inputs.  fp32: |gpu - oracle| <= 1e-5 * (A^^k |X|) elementwise at every
hop; bf16 storage: <= 1e-2 * (A^^k |X|), oracle fed the bf16-rounded X and never
re-rounding between hops."""
import numpy as np
import pytest

import gp_synth
import oracle
import paper_2207_12000_amd as gp

DEFAULT_SEGMENT_EDGES = 0   # automatic

pytestmark = pytest.mark.gpu

TOL = {gp.GP_F32: 1e-5, gp.GP_BF16: 1e-2}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu(gpu_or_skip):
    yield


def torch_dev():
    import torch
    return torch, torch.device("cuda:0")


def run_library(plan, X_np, dtype, agg, K, ld_pad=0, alias=False):
    """X_np: float32 (n,d) or uint16 bf16 bits.  Returns float64 (K+1, n, d)
    of what the library stored, exactly widened."""
    torch, dev = torch_dev()
    n, d = X_np.shape
    tdt = torch.float32 if dtype == gp.GP_F32 else torch.bfloat16
    if dtype == gp.GP_F32:
        xt = torch.from_numpy(np.ascontiguousarray(X_np))
    else:
        xt = torch.from_numpy(np.ascontiguousarray(X_np).view(np.int16)).view(torch.bfloat16)
    ldo = d + ld_pad
    out = torch.full((K + 1, n, ldo), float("nan"), dtype=tdt, device=dev)
    if alias:
        out[0, :, :d] = xt.to(dev)
        xdev, ldx = out, ldo
    else:
        ldx = d + (ld_pad and ld_pad + 1)
        xdev = torch.zeros((n, ldx), dtype=tdt, device=dev)
        xdev[:, :d] = xt.to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    gp.gp_propagate(plan, xdev.data_ptr(), ldx, d, dtype, agg, K, out.data_ptr(), ldo, stream)
    torch.cuda.synchronize()
    if ld_pad:
        assert torch.isnan(out[:, :, d:].float()).all(), "library wrote into the row padding"
    return out[:, :, :d].float().cpu().numpy().astype(np.float64)


def widen(X_np, dtype):
    return (X_np if dtype == gp.GP_F32 else gp_synth.bf16_bits_to_f32(X_np)).astype(np.float64)


def check(got, want, bound, tol, what=""):
    for k in range(len(want)):
        err = np.abs(got[k] - want[k])
        lim = tol * bound[k]
        zero = bound[k] == 0
        assert np.all(got[k][zero] == 0), f"{what} hop {k}: non-zero where the bound is zero"
        bad = err > lim + 1e-30
        assert not bad.any(), (f"{what} hop {k}: {bad.sum()} elements over tolerance, worst ratio "
                               f"{np.max(err[~zero] / lim[~zero]):.3g}")


def plan_pair(src, dst, n, budget, flags):
    return gp.gp_plan_blocks(src, dst, n, budget, flags), oracle.plan_blocks(src, dst, n, budget, flags)


def parity_case(w, K=None, d=None, dtype=None, agg=None, ld_pad=0, alias=False, budget=None, threads=4):
    K = w.K if K is None else K
    dtype = w.dtype if dtype is None else dtype
    agg = w.agg if agg is None else agg
    X = w.X if d is None else w.X[:, :d]
    if dtype == gp.GP_BF16 and X.dtype != np.uint16:
        X = gp_synth.f32_to_bf16_bits(X)
    if dtype == gp.GP_F32 and X.dtype == np.uint16:
        X = gp_synth.bf16_bits_to_f32(X)
    budget = budget or w.block_budget_edges or 10**9
    lp, op = plan_pair(w.src, w.dst, w.n, budget, w.flags)
    with lp:
        got = run_library(lp, X, dtype, agg, K, ld_pad, alias)
    Xw = widen(X, dtype)
    want = oracle.propagate(op, Xw, agg, K, threads)
    bound = oracle.bound_stack(op, Xw, agg, K, threads)
    assert np.array_equal(got[0], Xw), "slot 0 must be X exactly"
    check(got, want, bound, TOL[dtype], w.name)
    return got


# ---- the five workloads at sizes the oracle finishes in seconds ------------------

def test_config1_tiny_full_size_four_blocks():
    w = gp_synth.make_workload(1)
    nnz = 2 * w.m + w.n
    parity_case(w, budget=-(-nnz // 4))


def test_config2_quarter_scale():
    parity_case(gp_synth.make_workload(2, scale=0.25))


def test_config3_mean_d100():
    parity_case(gp_synth.make_workload(3, scale=0.01))


def test_config4_sum_d602():
    parity_case(gp_synth.make_workload(4, scale=0.002))


def test_config5_bf16_resident():
    parity_case(gp_synth.make_workload(5, scale=0.0005))


# ---- shapes: ragged d, padded leading dimensions, aliasing, column tiles ---------

@pytest.mark.parametrize("d", [1, 2, 3, 7, 8, 33, 64, 100, 128, 130, 257, 600, 1030])
@pytest.mark.parametrize("dtype", [gp.GP_F32, gp.GP_BF16])
def test_feature_widths(d, dtype):
    w = gp_synth.make_workload(2, scale=0.01, d=d)
    parity_case(w, K=2, dtype=dtype)


@pytest.mark.parametrize("dtype", [gp.GP_F32, gp.GP_BF16])
@pytest.mark.parametrize("agg", [gp.GP_AGG_SYM, gp.GP_AGG_MEAN, gp.GP_AGG_SUM])
@pytest.mark.parametrize("ld_pad,alias", [(0, True), (3, False), (4, True), (1, False)])
def test_leading_dimension_and_alias(dtype, agg, ld_pad, alias):
    w = gp_synth.make_workload(3, scale=0.002, d=36)
    parity_case(w, K=2, dtype=dtype, agg=agg, ld_pad=ld_pad, alias=alias)


def test_column_tile_option_changes_nothing():
    w = gp_synth.make_workload(2, scale=0.02, d=200)
    gp.gp_set_option("split_records", 2)     # whole records on both sides (cut records group the sums differently)
    try:
        a = parity_case(w, K=2)
        gp.gp_set_option("column_tile", 64)
        b = parity_case(w, K=2)
    finally:
        gp.gp_set_option("column_tile", 0)
        gp.gp_set_option("split_records", 0)
    assert np.array_equal(a, b)          # per-row summation order does not depend on the tile


# ---- schedule independence, hubs, block cuts, determinism ---------------------

def test_hub_rows_and_block_cuts_small_segments():
    w = gp_synth.make_workload(3, scale=0.005, d=20)
    gp.gp_set_option("segment_edges", 8)
    try:
        for budget in (10**9, 1000, 37):
            parity_case(w, K=2, budget=budget, agg=gp.GP_AGG_SYM)
    finally:
        gp.gp_set_option("segment_edges", DEFAULT_SEGMENT_EDGES)


def test_star_graph_one_row_spans_every_block():
    n = 5000
    src = np.arange(1, n, dtype=np.int32)
    dst = np.zeros(n - 1, dtype=np.int32)
    X = gp_synth.features(n, 24, "normal", gp_synth.rng_for(7, 7))
    for agg in (gp.GP_AGG_SYM, gp.GP_AGG_MEAN, gp.GP_AGG_SUM):
        lp, op = plan_pair(src, dst, n, 600, 3)
        with lp:
            got = run_library(lp, X, gp.GP_F32, agg, 2)
        Xw = X.astype(np.float64)
        check(got, oracle.propagate(op, Xw, agg, 2), oracle.bound_stack(op, Xw, agg, 2), 1e-5, "star")


def test_deterministic_and_block_count_independent():
    w = gp_synth.make_workload(2, scale=0.05, d=32)
    a = parity_case(w, K=2, budget=10**9)
    b = parity_case(w, K=2, budget=10**9)
    assert np.array_equal(a, b)
    c = parity_case(w, K=2, budget=5000)
    # cutting rows at block boundaries may change rounding, not more
    assert np.allclose(a, c, rtol=1e-4, atol=1e-5)


# ---- degenerate cases --------------------------------------------------------

def test_k_zero_and_no_edges():
    X = gp_synth.features(17, 5, "normal", gp_synth.rng_for(1, 2))
    lp, op = plan_pair([], [], 17, 4, 0)
    with lp:
        got = run_library(lp, X, gp.GP_F32, gp.GP_AGG_SUM, 2)
    assert np.array_equal(got[0], X.astype(np.float64)) and np.all(got[1:] == 0)
    lp, op = plan_pair([], [], 17, 4, gp.GP_ADD_SELF_LOOPS)
    for agg in (gp.GP_AGG_SYM, gp.GP_AGG_MEAN, gp.GP_AGG_SUM):   # A^ = I
        with gp.gp_plan_blocks([], [], 17, 4, gp.GP_ADD_SELF_LOOPS) as p2:
            got = run_library(p2, X, gp.GP_F32, agg, 2)
        assert all(np.array_equal(got[k], X.astype(np.float64)) for k in range(3))
    with gp.gp_plan_blocks([0], [1], 17, 4, 3) as p3:
        got = run_library(p3, X, gp.GP_F32, gp.GP_AGG_SYM, 0)
    assert got.shape[0] == 1 and np.array_equal(got[0], X.astype(np.float64))
    lp.close()


def test_mean_without_loops_zero_rows_and_constants():
    rng = np.random.default_rng(4)
    n = 400
    src, dst = rng.integers(0, n, 300), rng.integers(0, n, 300)
    lp, op = plan_pair(src, dst, n, 64, gp.GP_SYMMETRISE)
    X = np.full((n, 12), 1.5, dtype=np.float32)
    with lp:
        got = run_library(lp, X, gp.GP_F32, gp.GP_AGG_MEAN, 1)
    has = op.deg > 0
    assert (~has).any()
    assert np.all(got[1][~has] == 0) and np.allclose(got[1][has], 1.5, rtol=1e-6)


def test_sum_of_ones_is_exactly_the_degree():
    w = gp_synth.make_workload(2, scale=0.05, d=4)
    lp, op = plan_pair(w.src, w.dst, w.n, 4096, w.flags)
    ones = np.ones((w.n, 4), dtype=np.float32)
    with lp:
        got = run_library(lp, ones, gp.GP_F32, gp.GP_AGG_SUM, 1)
    assert np.array_equal(got[1][:, 0], op.deg.astype(np.float64))


def test_untouched_rows_do_not_leak_nonfinite_values():
    """A NaN in a row nobody aggregates from must not reach any output row."""
    n = 64
    src = np.arange(1, 33, dtype=np.int32)
    dst = np.zeros(32, dtype=np.int32)          # rows 33.. are isolated, row 40 holds NaN
    X = np.ones((n, 8), dtype=np.float32)
    X[40] = np.nan
    with gp.gp_plan_blocks(src, dst, n, 10, gp.GP_SYMMETRISE) as lp:
        got = run_library(lp, X, gp.GP_F32, gp.GP_AGG_SUM, 1)
    assert np.isfinite(got[1]).all()


def test_bad_arguments_return_status():
    torch, dev = torch_dev()
    x = torch.zeros((8, 4), device=dev)
    out = torch.zeros((2, 8, 4), device=dev)
    host = np.zeros((8, 4), dtype=np.float32)
    with gp.gp_plan_blocks([0], [1], 8, 4, 3) as lp:
        for args in [
            (0, 4, 4, 0, 0, 1, out.data_ptr(), 4),                       # X NULL
            (x.data_ptr(), 3, 4, 0, 0, 1, out.data_ptr(), 4),            # ldx < d
            (x.data_ptr(), 4, 0, 0, 0, 1, out.data_ptr(), 4),            # d = 0
            (x.data_ptr(), 4, 4, 0, 0, -1, out.data_ptr(), 4),           # K < 0
            (x.data_ptr(), 4, 4, 5, 0, 1, out.data_ptr(), 4),            # dtype
            (x.data_ptr(), 4, 4, 0, 9, 1, out.data_ptr(), 4),            # agg
            (host.ctypes.data, 4, 4, 0, 0, 1, out.data_ptr(), 4),        # pageable host X
        ]:
            with pytest.raises(gp.GpError) as e:
                gp.gp_propagate(lp, *args)
            assert e.value.status == gp.GP_ERR_INVALID_ARG


def test_many_hops_and_repeated_calls_on_one_plan():
    """K = 6 (error grows at most linearly with K against the bound), then the same
    plan reused with another width, dtype and operator: the scratch is resized."""
    w = gp_synth.make_workload(2, scale=0.02, d=48)
    lp, op = plan_pair(w.src, w.dst, w.n, 3000, w.flags)
    with lp:
        for d, dtype, agg, K in [(48, gp.GP_F32, gp.GP_AGG_SYM, 6), (16, gp.GP_BF16, gp.GP_AGG_MEAN, 2),
                                 (48, gp.GP_F32, gp.GP_AGG_SUM, 1), (40, gp.GP_BF16, gp.GP_AGG_SYM, 3)]:
            X = w.X[:, :d]
            if dtype == gp.GP_BF16:
                X = gp_synth.f32_to_bf16_bits(X)
            got = run_library(lp, X, dtype, agg, K)
            Xw = widen(X, dtype)
            check(got, oracle.propagate(op, Xw, agg, K, 4), oracle.bound_stack(op, Xw, agg, K, 4), TOL[dtype],
                  f"d={d} dtype={dtype} agg={agg} K={K}")


# ---- work mapping: column slices, workgroup count, explicit per-XCD lists ----------------

@pytest.fixture
def _mapping_defaults():
    yield
    for k in ("column_slices", "persistent_blocks", "cache_schedule", "segment_edges", "split_records", "lds_pass", "hub_pass", "plane_strips"):
        gp.gp_set_option(k, 0)


@pytest.mark.parametrize("dtype,d", [(gp.GP_F32, 136), (gp.GP_BF16, 264), (gp.GP_F32, 602)])
@pytest.mark.parametrize("slices", [1, 2, 4, 8])
def test_implicit_lists_any_slice_count_and_grid(dtype, d, slices, _mapping_defaults):
    """Column slices and the number of workgroups change which lane group computes what,
    not what is computed: every (slices, grid) gives the bits of the default mapping."""
    w = gp_synth.make_workload(3, scale=0.004, d=d)
    gp.gp_set_option("cache_schedule", 2)
    ref = parity_case(w, K=2, dtype=dtype, agg=gp.GP_AGG_SYM)
    gp.gp_set_option("column_slices", slices)
    gp.gp_set_option("persistent_blocks", 40)          # fewer workgroups than stay resident: every group walks far
    got = parity_case(w, K=2, dtype=dtype, agg=gp.GP_AGG_SYM)
    assert np.array_equal(ref, got)


@pytest.mark.parametrize("dtype,d,agg", [(gp.GP_F32, 602, gp.GP_AGG_SUM), (gp.GP_F32, 100, gp.GP_AGG_MEAN),
                                         (gp.GP_BF16, 128, gp.GP_AGG_SYM), (gp.GP_F32, 37, gp.GP_AGG_SYM)])
@pytest.mark.parametrize("slices", [0, 1, 3, 5, 16])
def test_explicit_lists_match_the_oracle_and_the_implicit_bits(dtype, d, agg, slices, _mapping_defaults):
    """The cache schedule (explicit per-XCD work lists handed out from cursors) forced on a
    community graph and on a graph without communities: the oracle's bound holds and the
    bits are those of the implicit lists (a record's sum does not depend on who adds it up);
    with every record cut into a piece that gathers inside the row's cluster and one that
    gathers outside it, in phases of their own, the sums are grouped differently and are
    checked against the oracle."""
    for cfg, scale in ((4, 0.004), (2, 0.03)):
        w = gp_synth.make_workload(cfg, scale=scale, d=d)
        gp.gp_set_option("segment_edges", 16)          # cut rows too
        gp.gp_set_option("cache_schedule", 2)
        gp.gp_set_option("column_slices", 0)
        ref = parity_case(w, K=2, dtype=dtype, agg=agg, budget=20_000)
        gp.gp_set_option("cache_schedule", 1)
        gp.gp_set_option("column_slices", slices)
        gp.gp_set_option("split_records", 2)           # whole records: the very same sums
        got = parity_case(w, K=2, dtype=dtype, agg=agg, budget=20_000)
        assert np.array_equal(ref, got), f"config {cfg}"
        gp.gp_set_option("split_records", 1)           # hot and cold pieces: other partial sums, the oracle's bound holds
        parity_case(w, K=2, dtype=dtype, agg=agg, budget=20_000)


def community_workload(n_comm, comm, pairs, d, seed):
    """A small stochastic block model of the config-4 kind with communities of a chosen size."""
    g = gp_synth.rng_for(seed, 0)
    src, dst = gp_synth.sbm_pairs(n_comm, comm, pairs, 0.9, g)
    X = gp_synth.features(n_comm * comm, d, "uniform", gp_synth.rng_for(seed, 1))
    return gp_synth.Workload("sbm_test", n_comm * comm, d, 2, gp.GP_AGG_SUM, gp.GP_F32,
                             gp_synth.SYMMETRISE | gp_synth.ADD_SELF_LOOPS, None, 4, src, dst, X)


@pytest.mark.parametrize("dtype,d,agg", [(gp.GP_F32, 602, gp.GP_AGG_SUM), (gp.GP_F32, 100, gp.GP_AGG_MEAN), (gp.GP_F32, 37, gp.GP_AGG_SYM),
                                         (gp.GP_F32, 4, gp.GP_AGG_SYM), (gp.GP_F32, 7, gp.GP_AGG_SUM),
                                         (gp.GP_BF16, 128, gp.GP_AGG_SYM), (gp.GP_BF16, 36, gp.GP_AGG_SUM), (gp.GP_BF16, 100, gp.GP_AGG_MEAN)])
@pytest.mark.parametrize("segment_edges,order", [(0, 1), (16, 1), (0, 3)])
def test_lds_pass_matches_the_oracle(dtype, d, agg, segment_edges, order, _mapping_defaults):
    """The hot pieces gathered from LDS, reads in conflict-free order (1) and in the column
    list's (3), forced (with rows cut into short segments the automatic choice would decline
    the padding): community graphs whose clusters take one
    strip in half of a compute unit's LDS and more than half of it, column counts that
    end in a partial strip, rows with and without partial-row slots, every operator, fp32
    storage and bf16 storage (rows of a multiple of four columns: vectors of eight columns
    that span two strips, the last one moved back).
    A second call on the same plan's twin repeats the first bit for bit."""
    cases = [gp_synth.make_workload(4, scale=0.004, d=d), gp_synth.make_workload(4, scale=0.04, d=d)]
    if d <= 37:
        cases.append(community_workload(3, 6000, 400_000, d, 77))    # clusters beyond half the LDS: one workgroup per unit
    for w in cases:
        gp.gp_set_option("segment_edges", segment_edges)
        gp.gp_set_option("cache_schedule", 1)
        gp.gp_set_option("split_records", 1)
        gp.gp_set_option("lds_pass", order)
        budget = max(20_000, w.m // 3)
        gp.gp_profile_enable(True)
        try:
            a = parity_case(w, K=2, dtype=dtype, agg=agg, budget=budget)
            b = parity_case(w, K=2, dtype=dtype, agg=agg, budget=budget)
            launches, _ = gp.gp_profile_read("gp_hop_cluster_lds")
        finally:
            gp.gp_profile_enable(False)
        assert launches == 4, f"{w.name} n {w.n}: the LDS pass ran {launches} times, expected once per hop"
        assert np.array_equal(a, b)


@pytest.mark.parametrize("cfg,scale,d,agg", [(2, 0.2, 128, gp.GP_AGG_SYM), (3, 0.02, 100, gp.GP_AGG_MEAN), (2, 0.2, 37, gp.GP_AGG_SUM),
                                             (3, 0.02, 6, gp.GP_AGG_SYM)])
@pytest.mark.parametrize("segment_edges,order", [(0, 1), (16, 1), (0, 3)])
def test_hub_pass_matches_the_oracle(cfg, scale, d, agg, segment_edges, order, _mapping_defaults):
    """Power-law graphs (no row clusters): the non-zeros whose source is one of the most popular
    rows are served from LDS, the others gathered from memory, forced on graphs smaller than
    the automatic choice would take.  Checked against the oracle, with the LDS launch
    counted; bf16 storage goes the same way where the rows are whole strips, and whole
    records (hub_pass = 2) keep working on the same graph."""
    w = gp_synth.make_workload(cfg, scale=scale, d=d)
    gp.gp_set_option("segment_edges", segment_edges)
    gp.gp_set_option("hub_pass", 1)
    gp.gp_set_option("lds_pass", order)
    budget = max(20_000, w.m // 3)
    gp.gp_profile_enable(True)
    try:
        a = parity_case(w, K=2, dtype=gp.GP_F32, agg=agg, budget=budget)
        launches, _ = gp.gp_profile_read("gp_hop_cluster_lds")
        parity_case(w, K=2, dtype=gp.GP_BF16, agg=agg, budget=budget)       # bf16 rows: the pass needs a multiple of four columns
        launches_after, _ = gp.gp_profile_read("gp_hop_cluster_lds")
    finally:
        gp.gp_profile_enable(False)
    want_after = 4 if d % 4 == 0 else 2
    assert launches == 2 and launches_after == want_after, f"the LDS pass ran {launches} / {launches_after} times"
    gp.gp_set_option("hub_pass", 2)
    parity_case(w, K=2, dtype=gp.GP_F32, agg=agg, budget=budget)


@pytest.mark.parametrize("dtype,d", [(gp.GP_F32, 100), (gp.GP_F32, 37), (gp.GP_BF16, 72)])
def test_plane_layouts_give_the_same_bits(dtype, d, _mapping_defaults):
    """The buffer through which the LDS launch hands its sums to the segment launch can keep 1, 2,
    4 or 8 strips of a segment together: the layout changes who touches which line, not what is
    added, so every layout gives the bits of the default, with row clusters and with hubs, fp32
    rows (whole strips and a last strip moved back) and bf16 rows (vectors of two strips)."""
    for cfg, scale, option in ((4, 0.004, "lds_pass"), (3, 0.02, "hub_pass")):
        w = gp_synth.make_workload(cfg, scale=scale, d=d)
        gp.gp_set_option(option, 1)
        budget = max(20_000, w.m // 3)
        ref = parity_case(w, K=2, dtype=dtype, agg=gp.GP_AGG_SYM, budget=budget)
        for together in (1, 2, 4, 8):
            gp.gp_set_option("plane_strips", together)
            got = parity_case(w, K=2, dtype=dtype, agg=gp.GP_AGG_SYM, budget=budget)
            assert np.array_equal(ref, got), f"config {cfg}, {together} strips together"
        gp.gp_set_option("plane_strips", 0)
        gp.gp_set_option(option, 0)

