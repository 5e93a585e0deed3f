"""Pins for the oracle's A^^k X: dense brute force built straight from Eq. 1,
closed forms, algebraic invariants, and a library CSR product.  None of these
re-types the oracle's loop: each would fail on a dropped term, a wrong degree,
a transposed operand or a wrong index in it."""
import math

import numpy as np
import pytest

import gp_synth
import oracle
from oracle import ADD_SELF_LOOPS, AGG_MEAN, AGG_SUM, AGG_SYM, SYMMETRISE

BOTH = SYMMETRISE | ADD_SELF_LOOPS


def dense_operator(src, dst, n, flags, agg):
    """A^ as a dense fp64 matrix from the definitions: A~ = A + I, D~ = diag of
    row sums, S = D~^-1/2 A~ D~^-1/2 (Eq. 1); D^-1 A; A."""
    A = np.zeros((n, n))
    for s, t in zip(src, dst):
        if s != t:
            A[t, s] = 1.0
            if flags & SYMMETRISE:
                A[s, t] = 1.0
    if flags & ADD_SELF_LOOPS:
        A = A + np.eye(n)
    deg = A.sum(axis=1)
    with np.errstate(divide="ignore"):
        if agg == AGG_SYM:
            s = np.where(deg > 0, deg ** -0.5, 0.0)
            return s[:, None] * A * s[None, :]
        if agg == AGG_MEAN:
            return np.where(deg > 0, 1.0 / deg, 0.0)[:, None] * A
    return A


def random_graph(seed, n=None, m=None):
    rng = np.random.default_rng(seed)
    n = n or int(rng.integers(2, 64))
    m = m if m is not None else int(rng.integers(0, 6 * n))
    return rng.integers(0, n, m), rng.integers(0, n, m), n, rng


@pytest.mark.parametrize("agg", [AGG_SYM, AGG_MEAN, AGG_SUM])
@pytest.mark.parametrize("flags", [0, SYMMETRISE, ADD_SELF_LOOPS, BOTH])
@pytest.mark.parametrize("seed", range(4))
def test_dense_brute_force(agg, flags, seed):
    src, dst, n, rng = random_graph(seed)
    X = rng.standard_normal((n, 5))
    plan = oracle.plan_blocks(src, dst, n, 7, flags)
    got = oracle.propagate(plan, X, agg, 3)
    M = dense_operator(src, dst, n, flags, agg)
    want = X
    assert np.array_equal(got[0], X)
    for k in range(1, 4):
        want = M @ want
        scale = np.abs(np.linalg.matrix_power(np.abs(M), k)) @ np.abs(X) + 1e-300
        assert np.all(np.abs(got[k] - want) <= 1e-13 * scale + 1e-300)


def test_directed_orientation_is_destination_row():
    # one pair src=0 -> dst=1: node 1 aggregates node 0's features
    plan = oracle.plan_blocks([0], [1], 2, 1, 0)
    X = np.array([[3.0], [5.0]])
    assert oracle.hop(plan, X, AGG_SUM).ravel().tolist() == [0.0, 3.0]


def test_sum_of_ones_is_degree_and_column_sums():
    w = gp_synth.make_workload(2, scale=0.01, d=3)
    plan = oracle.plan_blocks(w.src, w.dst, w.n, 1000, w.flags)
    ones = np.ones((w.n, 2))
    Y = oracle.hop(plan, ones, AGG_SUM)
    assert np.array_equal(Y[:, 0], plan.deg.astype(np.float64))
    X = w.X.astype(np.float64)
    outdeg = np.bincount(plan.col, minlength=w.n).astype(np.float64)
    lhs = oracle.hop(plan, X, AGG_SUM).sum(axis=0)
    assert np.allclose(lhs, outdeg @ X, rtol=1e-11, atol=1e-9)


def test_mean_keeps_constants_and_stays_in_neighbour_range():
    src, dst, n, rng = random_graph(11, n=50, m=120)
    plan = oracle.plan_blocks(src, dst, n, 10**6, SYMMETRISE)      # no self-loops: isolated rows exist
    c = np.full((n, 2), 2.5)
    Y = oracle.hop(plan, c, AGG_MEAN)
    has = plan.deg > 0
    assert has.any() and (~has).any()
    assert np.allclose(Y[has], 2.5, rtol=1e-15) and np.all(Y[~has] == 0.0)
    X = rng.standard_normal((n, 3))
    Y = oracle.hop(plan, X, AGG_MEAN)
    for i in np.flatnonzero(has):
        nb = plan.col[plan.rowptr[i]:plan.rowptr[i + 1]]
        assert np.all(Y[i] <= X[nb].max(axis=0) + 1e-14) and np.all(Y[i] >= X[nb].min(axis=0) - 1e-14)


def regular_graphs():
    ring = ([i for i in range(12)], [(i + 1) % 12 for i in range(12)], 12)
    kn = ([i for i in range(7) for j in range(i)], [j for i in range(7) for j in range(i)], 7)
    cube = ([i for i in range(16) for b in range(4) if i < i ^ (1 << b)],
            [i ^ (1 << b) for i in range(16) for b in range(4) if i < i ^ (1 << b)], 16)
    return [ring, kn, cube]


@pytest.mark.parametrize("g", regular_graphs())
def test_sym_on_regular_graph_with_loops_keeps_constants(g):
    """Holds only when D~ is the row sum of A + I (degree + 1): the reading of
    the undefined D~ of Eq. 1.  With D~ = D it fails."""
    src, dst, n = g
    plan = oracle.plan_blocks(src, dst, n, 5, BOTH)
    assert len(set(plan.deg.tolist())) == 1
    out = oracle.propagate(plan, np.full((n, 2), -1.75), AGG_SYM, 3)
    for Y in out:
        assert np.allclose(Y, -1.75, rtol=1e-14)


def test_sym_complete_graph_gives_column_means():
    n = 9
    src = [i for i in range(n) for j in range(i)]
    dst = [j for i in range(n) for j in range(i)]
    plan = oracle.plan_blocks(src, dst, n, 10, BOTH)
    X = np.random.default_rng(5).standard_normal((n, 4))
    out = oracle.propagate(plan, X, AGG_SYM, 3)
    for k in (1, 2, 3):
        assert np.allclose(out[k], np.broadcast_to(X.mean(axis=0), X.shape), rtol=1e-13, atol=1e-15)


def trinomial_row(k):
    """Coefficients of (x^-1 + 1 + x)^k, index j+k for x^j, exact integers."""
    row = [1]
    for _ in range(k):
        new = [0] * (len(row) + 2)
        for i, c in enumerate(row):
            new[i] += c
            new[i + 1] += c
            new[i + 2] += c
        row = new
    return row


def test_sym_ring_gives_trinomial_coefficients():
    n, K = 15, 4                                       # n > 2K: no wrap-around
    plan = oracle.plan_blocks(list(range(n)), [(i + 1) % n for i in range(n)], n, 6, BOTH)
    e0 = np.zeros((n, 1))
    e0[0] = 1.0
    out = oracle.propagate(plan, e0, AGG_SYM, K)
    for k in range(1, K + 1):
        T = trinomial_row(k)
        want = np.zeros(n)
        for j in range(-k, k + 1):
            want[j % n] = T[j + k] / 3 ** k
        assert np.allclose(out[k].ravel(), want, rtol=1e-14, atol=0)


def test_sym_star_closed_form():
    n = 11                                             # centre 0, leaves 1..10
    plan = oracle.plan_blocks([0] * (n - 1), list(range(1, n)), n, 100, BOTH)
    a, b = 2.0, -3.0                                   # centre value, leaf value
    X = np.full((n, 1), b)
    X[0] = a
    out = oracle.propagate(plan, X, AGG_SYM, 3)
    for k in range(1, 4):
        a, b = a / n + (n - 1) * b / math.sqrt(2 * n), b / 2 + a / math.sqrt(2 * n)
        assert math.isclose(out[k][0, 0], a, rel_tol=1e-13)
        assert np.allclose(out[k][1:, 0], b, rtol=1e-13)


def test_sym_adjoint_and_eigenvector():
    w = gp_synth.make_workload(2, scale=0.01, d=4)
    plan = oracle.plan_blocks(w.src, w.dst, w.n, 10**9, w.flags)
    rng = np.random.default_rng(3)
    X = w.X.astype(np.float64)
    Z = rng.standard_normal(X.shape)
    lhs = np.sum(Z * oracle.hop(plan, X, AGG_SYM))
    rhs = np.sum(oracle.hop(plan, Z, AGG_SYM) * X)
    assert math.isclose(lhs, rhs, rel_tol=1e-10)
    v = np.sqrt(plan.deg.astype(np.float64))[:, None]
    assert np.allclose(oracle.hop(plan, v, AGG_SYM), v, rtol=1e-13)


@pytest.mark.parametrize("agg", [AGG_SYM, AGG_MEAN, AGG_SUM])
def test_matches_library_csr_product(agg):
    sp = pytest.importorskip("scipy.sparse")
    w = gp_synth.make_workload(3, scale=0.002, d=7)
    plan = oracle.plan_blocks(w.src, w.dst, w.n, 5000, BOTH)
    deg = plan.deg.astype(np.float64)
    r, c = plan.row.astype(np.int64), plan.col.astype(np.int64)
    val = {AGG_SYM: 1 / np.sqrt(deg[r] * deg[c]), AGG_MEAN: 1 / deg[r], AGG_SUM: np.ones(r.size)}[agg]
    M = sp.csr_matrix((val, (r, c)), shape=(w.n, w.n))
    X = w.X.astype(np.float64)
    got = oracle.propagate(plan, X, agg, 2)
    bound = oracle.bound_stack(plan, X, agg, 2)
    want = X
    for k in (1, 2):
        want = M @ want
        assert np.all(np.abs(got[k] - want) <= 1e-13 * bound[k] + 1e-300)


def test_linearity_blocks_relabel_threads_and_rows():
    w = gp_synth.make_workload(2, scale=0.02, d=6)
    n = w.n
    X = w.X.astype(np.float64)
    rng = np.random.default_rng(9)
    Z = rng.standard_normal(X.shape)
    plan1 = oracle.plan_blocks(w.src, w.dst, n, 10**9, w.flags)
    planb = oracle.plan_blocks(w.src, w.dst, n, 997, w.flags)
    assert planb.num_blocks > 10 and plan1.num_blocks == 1
    for agg in (AGG_SYM, AGG_MEAN, AGG_SUM):
        a = oracle.propagate(plan1, X, agg, 2)
        # the block count changes the schedule, never the result
        b = oracle.propagate(planb, X, agg, 2)
        assert all(np.array_equal(p, q) for p, q in zip(a, b))
        # threads only cut the list at row boundaries
        c = oracle.propagate(plan1, X, agg, 2, threads=3)
        assert all(np.array_equal(p, q) for p, q in zip(a, c))
        # linearity
        lin = oracle.hop(plan1, 2.0 * X - 0.5 * Z, agg)
        assert np.allclose(lin, 2.0 * a[1] - 0.5 * oracle.hop(plan1, Z, agg), rtol=1e-12, atol=1e-12)
        # relabel -> propagate -> unlabel
        perm = rng.permutation(n)
        planp = oracle.plan_blocks(perm[w.src], perm[w.dst], n, 10**9, w.flags)
        Xp = np.empty_like(X)
        Xp[perm] = X
        yp = oracle.hop(planp, Xp, agg)
        assert np.allclose(yp[perm], a[1], rtol=1e-12, atol=1e-13)
        # sampled rows one by one
        rows = rng.integers(0, n, 50)
        y, bnd = oracle.hop_rows(plan1, X, agg, rows)
        ref_b = oracle.bound_stack(plan1, X, agg, 1)[1]
        assert np.all(np.abs(y - a[1][rows]) <= 1e-14 * bnd + 1e-300)
        assert np.allclose(bnd, ref_b[rows], rtol=1e-13)


def test_bf16_helpers_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.140625], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    bits = gp_synth.f32_to_bf16_bits(x)
    back = gp_synth.bf16_bits_to_f32(bits)
    assert back.tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0, 3.140625]


@pytest.mark.parametrize("flags", [0, SYMMETRISE, ADD_SELF_LOOPS, BOTH])
def test_sampled_row_oracle_agrees_with_the_full_one(flags):
    """The pair-list scan used at sizes the full planner cannot hold must give the
    same neighbour sets, degrees and rows as the planner-based oracle."""
    from oracle import sampled
    w = gp_synth.make_workload(3, scale=0.002, d=6)
    plan = oracle.plan_blocks(w.src, w.dst, w.n, 10**9, flags)
    rng = np.random.default_rng(8)
    rows = np.concatenate([rng.integers(0, w.n, 40), np.argsort(plan.deg)[-3:], np.argsort(plan.deg)[:3]])
    cols, deg = sampled.neighbourhoods(w.src, w.dst, w.n, flags, rows, chunk=5000)
    for t, i in enumerate(rows):
        assert np.array_equal(cols[t], plan.col[plan.rowptr[i]:plan.rowptr[i + 1]])
    for node, g in deg.items():
        assert g == plan.deg[node]
    X = w.X.astype(np.float64)
    for agg in (AGG_SYM, AGG_MEAN, AGG_SUM):
        y, b = sampled.hop_rows(cols, deg, rows, X, agg)
        y2, b2 = oracle.hop_rows(plan, X, agg, rows)
        assert np.allclose(y, y2, rtol=1e-13, atol=1e-300) and np.allclose(b, b2, rtol=1e-13, atol=1e-300)
