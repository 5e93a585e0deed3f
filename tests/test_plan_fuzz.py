"""Property-based comparison of gp_plan_blocks (host planner) with the oracle's
planner: arbitrary small pair lists (duplicates, reciprocals, self pairs, isolated
nodes), every flag combination, budgets from 1 upwards, several segment lengths."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
import paper_2207_12000_amd as gp
from test_plan_parity import assert_same_plan, check_schedule


@st.composite
def graphs(draw):
    n = draw(st.integers(1, 40))
    m = draw(st.integers(0, 120))
    ids = st.integers(0, n - 1)
    src = draw(st.lists(ids, min_size=m, max_size=m))
    dst = draw(st.lists(ids, min_size=m, max_size=m))
    return n, src, dst


@settings(max_examples=150, deadline=None)
@given(graphs(), st.integers(0, 3), st.integers(1, 60), st.sampled_from([0, 8, 9, 64]))
def test_plan_matches_oracle(g, flags, budget, seg_len):
    n, src, dst = g
    op = oracle.plan_blocks(src, dst, n, budget, flags)
    gp.gp_set_option("segment_edges", seg_len)
    try:
        with gp.gp_plan_blocks(src, dst, n, budget, flags) as lp:
            assert_same_plan(lp, op)
            check_schedule(lp, lp.segment_edges)
    finally:
        gp.gp_set_option("segment_edges", 0)
