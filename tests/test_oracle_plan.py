"""Pins for the oracle's block planner: hand-enumerated tiny cases, brute force
with Python sets, and the properties the paper states for the decomposition
(Section 3.2: the sets are disjoint, their union is the whole edge set, their
sizes are balanced)."""
import math

import numpy as np
import pytest

import gp_synth
import oracle
from oracle import ADD_SELF_LOOPS, SYMMETRISE, OracleError


def brute_set(src, dst, n, flags):
    """The non-zero set written straight from the definition, with Python sets."""
    P = set()
    for s, t in zip(src, dst):
        s, t = int(s), int(t)
        if s == t:
            continue
        P.add((t, s))
        if flags & SYMMETRISE:
            P.add((s, t))
    if flags & ADD_SELF_LOOPS:
        for i in range(n):
            P.add((i, i))
    return P


def check_plan(plan, src, dst, n, flags, budget):
    P = brute_set(src, dst, n, flags)
    listed = list(zip(plan.row.tolist(), plan.col.tolist()))
    assert listed == sorted(P)                       # a set, ascending (row, col)
    nnz = len(P)
    assert plan.nnz == nnz
    # degrees = row sums of the 0/1 matrix
    deg = [0] * n
    for r, _ in P:
        deg[r] += 1
    assert plan.deg.tolist() == deg
    assert plan.rowptr.tolist() == [0] + np.cumsum(deg).tolist()
    # blocks: disjoint, cover everything, balanced, smallest count within budget
    off = plan.block_off.tolist()
    b = len(off) - 1
    assert b == max(1, math.ceil(nnz / budget))
    assert off[0] == 0 and off[-1] == nnz
    sizes = [off[p + 1] - off[p] for p in range(b)]
    assert all(s >= 0 for s in sizes)
    assert max(sizes) - min(sizes) <= 1
    assert max(sizes) <= budget or nnz == 0
    seen = []
    for p in range(b):
        seen += listed[off[p]:off[p + 1]]
    assert sorted(seen) == sorted(P) and len(seen) == len(set(seen))
    for p in range(b):
        if sizes[p]:
            assert plan.block_row_lo[p] == listed[off[p]][0]
            assert plan.block_row_hi[p] == listed[off[p + 1] - 1][0]
        else:
            assert plan.block_row_lo[p] == 0 and plan.block_row_hi[p] == -1
    # norms: one correctly rounded recipe
    for i in range(n):
        if deg[i]:
            assert plan.dinv_sqrt[i] == np.float32(1.0 / math.sqrt(deg[i]))
            assert plan.dinv[i] == np.float32(1.0 / deg[i])
        else:
            assert plan.dinv_sqrt[i] == 0 and plan.dinv[i] == 0


def test_empty_graph_with_and_without_loops():
    p = oracle.plan_blocks([], [], 4, 3, ADD_SELF_LOOPS)
    assert p.row.tolist() == [0, 1, 2, 3] and p.col.tolist() == [0, 1, 2, 3]
    assert p.block_off.tolist() == [0, 2, 4]
    p = oracle.plan_blocks([], [], 4, 3, 0)
    assert p.nnz == 0 and p.block_off.tolist() == [0, 0]
    assert p.deg.tolist() == [0] * 4 and p.dinv.tolist() == [0.0] * 4
    assert p.block_row_lo.tolist() == [0] and p.block_row_hi.tolist() == [-1]


def test_single_directed_edge():
    # pair (src=2, dst=0): node 0 aggregates from node 2 -> non-zero at row 0, col 2
    p = oracle.plan_blocks([2], [0], 3, 10, 0)
    assert list(zip(p.row.tolist(), p.col.tolist())) == [(0, 2)]
    assert p.deg.tolist() == [1, 0, 0]
    p = oracle.plan_blocks([2], [0], 3, 10, SYMMETRISE)
    assert list(zip(p.row.tolist(), p.col.tolist())) == [(0, 2), (2, 0)]


def test_path_p3():
    p = oracle.plan_blocks([0, 1], [1, 2], 3, 4, SYMMETRISE | ADD_SELF_LOOPS)
    assert list(zip(p.row.tolist(), p.col.tolist())) == [
        (0, 0), (0, 1), (1, 0), (1, 1), (1, 2), (2, 1), (2, 2)]
    assert p.deg.tolist() == [2, 3, 2]
    assert p.block_off.tolist() == [0, 4, 7]          # 7 entries, budget 4 -> 2 blocks 4+3
    assert p.block_row_lo.tolist() == [0, 1] and p.block_row_hi.tolist() == [1, 2]
    p = oracle.plan_blocks([0, 1], [1, 2], 3, 4, 0)
    assert list(zip(p.row.tolist(), p.col.tolist())) == [(1, 0), (2, 1)]


def test_duplicates_reciprocals_and_self_pairs_collapse():
    src = [0, 0, 1, 2, 2, 1]
    dst = [1, 1, 0, 2, 2, 1]     # (0,1) twice, its reciprocal, self pairs on 2 and 1
    p = oracle.plan_blocks(src, dst, 3, 100, SYMMETRISE)
    assert list(zip(p.row.tolist(), p.col.tolist())) == [(0, 1), (1, 0)]
    p = oracle.plan_blocks(src, dst, 3, 100, SYMMETRISE | ADD_SELF_LOOPS)
    assert p.deg.tolist() == [2, 2, 1]                # diagonal exactly once


def test_single_node():
    p = oracle.plan_blocks([0], [0], 1, 1, ADD_SELF_LOOPS)
    assert p.nnz == 1 and p.deg.tolist() == [1]
    p = oracle.plan_blocks([0], [0], 1, 1, 0)
    assert p.nnz == 0


@pytest.mark.parametrize("flags", [0, SYMMETRISE, ADD_SELF_LOOPS, SYMMETRISE | ADD_SELF_LOOPS])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_against_brute_force(flags, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    m = int(rng.integers(0, 200))
    src = rng.integers(0, n, m)
    dst = rng.integers(0, n, m)
    for budget in (1, 3, 7, 50, 10**6):
        check_plan(oracle.plan_blocks(src, dst, n, budget, flags), src, dst, n, flags, budget)


def test_balance_on_workload():
    w = gp_synth.make_workload(1, scale=0.05, with_features=False)
    for budget in (1000, 977, 4096):
        p = oracle.plan_blocks(w.src, w.dst, w.n, budget, w.flags)
        sizes = np.diff(p.block_off)
        assert sizes.max() - sizes.min() <= 1 and sizes.max() <= budget
        assert p.num_blocks == math.ceil(p.nnz / budget)
    # G(n, M) draws M distinct non-loop pairs: exactly 2M + n non-zeros
    assert p.nnz == 2 * w.m + w.n


def test_errors():
    with pytest.raises(OracleError) as e:
        oracle.plan_blocks([0], [3], 3, 1, 0)
    assert e.value.kind == "INDEX_RANGE"
    with pytest.raises(OracleError) as e:
        oracle.plan_blocks([-1], [0], 3, 1, 0)
    assert e.value.kind == "INDEX_RANGE"
    for bad in (dict(n=0), dict(budget=0), dict(flags=4)):
        kw = dict(n=3, budget=1, flags=0)
        kw.update(bad)
        with pytest.raises(OracleError) as e:
            oracle.plan_blocks([0], [1], kw["n"], kw["budget"], kw["flags"])
        assert e.value.kind == "INVALID_ARG"


def test_paper_printed_sizes_pin_nonzero_accounting():
    """Section 4.2 prints 67 GB for the normalised adjacency and 57 GB for the
    features of the largest graph (Table 1: nodes, edges, 128 features)."""
    import os
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "papers100m_sizes.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = int(v)
    nnz = gp_synth.stored_nonzeros_upper_bound(vals["nodes"], vals["edges"],
                                               SYMMETRISE | ADD_SELF_LOOPS)
    assert nnz == 2 * vals["edges"] + vals["nodes"] == 3_342_431_700
    assert round(nnz * 20 / 1e9) == vals["normalised_adjacency_GB"]
    assert round(vals["nodes"] * vals["features"] * 4 / 1e9) == vals["feature_matrix_GB"]
