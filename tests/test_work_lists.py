"""Host logic of the cache schedule: row clusters and the explicit per-XCD work lists."""
import numpy as np
import pytest

import gp_synth
import paper_2207_12000_amd as gp


@pytest.fixture(autouse=True)
def _defaults():
    yield
    for k in ("cache_schedule", "column_slices", "segment_edges"):
        gp.gp_set_option(k, 0)


def check_lists(plan, d, dtype, vec):
    S, elems, off, recs = plan.work_lists(d, dtype, vec)
    if S == 0:
        return 0
    segs = plan.segments
    assert elems % vec == 0 and (S - 1) * elems < d <= S * elems
    assert off[0] == 0 and np.all(np.diff(off) >= 0) and off[8] == recs.size == segs.size * S
    # every (segment, slice) pair exactly once: a record is a segment with its slice filled in
    key = lambda a: np.stack([a["start_lo"].astype(np.int64) | (a["start_hi"].astype(np.int64) << 32),
                              a["len"].astype(np.int64), a["row"].astype(np.int64), a["slot"].astype(np.int64)], 1)
    want = np.concatenate([np.concatenate([key(segs), np.full((segs.size, 1), s)], 1) for s in range(S)])
    got = np.concatenate([key(recs), recs["slice"].astype(np.int64)[:, None]], 1)
    assert np.array_equal(np.unique(want, axis=0), np.unique(got, axis=0)) and len(np.unique(got, axis=0)) == got.shape[0]
    return S


def test_sbm_clusters_are_found_and_lists_cover_everything():
    w = gp_synth.make_workload(4, scale=0.02, with_features=False)
    with gp.gp_plan_blocks(w.src, w.dst, w.n, w.block_budget_edges, w.flags) as plan:
        label, num, inside, typical = plan.row_clusters()
        assert num == 50 and inside > 0.85                 # the generator's 50 communities, 90 % of the draws inside
        assert np.all(np.bincount(label) == w.n // 50)
        # same label <=> same community of the generator is not visible here (ids are permuted), but a
        # row and most of its sources must share a label
        rp, col = plan.rowptr, plan.col
        rows = np.repeat(np.arange(w.n), np.diff(rp))
        assert abs(np.mean(label[rows] == label[col]) - inside) < 1e-12
        assert check_lists(plan, w.d, gp.GP_F32, 2) >= 1
        assert check_lists(plan, 128, gp.GP_BF16, 8) >= 1


def test_graph_without_clusters_keeps_implicit_lists_unless_forced():
    # one giant cluster whose rows cannot fit an L2 at any slice of >= 128 bytes
    w = gp_synth.make_workload(3, scale=0.01, with_features=False)
    with gp.gp_plan_blocks(w.src, w.dst, w.n, w.block_budget_edges, w.flags) as plan:
        assert plan.row_clusters()[3] > 0.5 * w.n
        assert plan.work_lists(w.d, gp.GP_F32, 4)[0] == 0
    gp.gp_set_option("cache_schedule", 1)
    for slices in (0, 1, 3, 5, 16):
        gp.gp_set_option("column_slices", slices)
        gp.gp_set_option("segment_edges", 8)
        with gp.gp_plan_blocks(w.src, w.dst, w.n, 5000, w.flags) as plan:
            S = check_lists(plan, 100, gp.GP_F32, 4)
            assert S >= 1 and (slices == 0 or S <= slices)
    gp.gp_set_option("cache_schedule", 2)
    w4 = gp_synth.make_workload(4, scale=0.005, with_features=False)
    with gp.gp_plan_blocks(w4.src, w4.dst, w4.n, w4.block_budget_edges, w4.flags) as plan:
        assert plan.work_lists(w4.d, gp.GP_F32, 2)[0] == 0


def test_clusters_do_not_depend_on_the_thread_split():
    # two disjoint cliques joined by one edge, plus isolated rows: labels are a function of the graph only
    a = np.arange(40)
    src = np.concatenate([np.repeat(a[:20], 20), np.repeat(a[20:], 20), [0]]).astype(np.int32)
    dst = np.concatenate([np.tile(a[:20], 20), np.tile(a[20:], 20), [39]]).astype(np.int32)
    with gp.gp_plan_blocks(src, dst, 44, 10**6, gp.GP_SYMMETRISE | gp.GP_ADD_SELF_LOOPS) as plan:
        label, num, inside, typical = plan.row_clusters()
        assert len(set(label[:20])) == 1 and len(set(label[20:40])) == 1 and label[0] != label[20]
        assert num == 2 + 4 and len(set(label[40:])) == 4
