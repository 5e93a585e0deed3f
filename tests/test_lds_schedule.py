"""Host logic of the LDS pass (no GPU): the schedule that orders the in-cluster reads of
every record is checked against the plan's own CSR and row clusters."""
import numpy as np
import pytest

import gp_synth
import paper_2207_12000_amd as gp


def pass_groups():
    """The four sets of 16 lanes whose 16-byte LDS reads are served together (gfx950)."""
    first = [l for l in range(32) if l < 4 or 12 <= l < 16 or 20 <= l < 28]
    second = [l for l in range(32) if l not in first]
    return [np.array(first), np.array(second), np.array(first) + 32, np.array(second) + 32]


def community_plan(n_comm, comm, pairs, seed, budget=None, segment_edges=0):
    g = gp_synth.rng_for(seed, 0)
    src, dst = gp_synth.sbm_pairs(n_comm, comm, pairs, 0.9, g)
    gp.gp_set_option("segment_edges", segment_edges)
    try:
        return gp.gp_plan_blocks(src, dst, n_comm * comm, budget or 10**9, gp_synth.SYMMETRISE | gp_synth.ADD_SELF_LOOPS)
    finally:
        gp.gp_set_option("segment_edges", 0)


def decode(plan, sched):
    """(row -> sorted in-cluster sources read for it, padding reads, steps x lanes table per group)."""
    label, num, _, _ = plan.row_clusters()
    order = np.argsort(label, kind="stable")            # a cluster's rows in ascending order
    counts = np.bincount(label, minlength=num)
    member_off = np.concatenate([[0], np.cumsum(counts)])
    got = {}
    tables = []
    for g in range(sched["group_cluster"].size):
        c = int(sched["group_cluster"][g])
        m = int(counts[c])
        steps = int(sched["group_steps"][g])
        assert steps % 8 == 0
        off = int(sched["group_id_off"][g])
        block = sched["ids"][off:off + steps * 64].reshape(steps // 8, 64, 8)
        table = block.transpose(0, 2, 1).reshape(steps, 64)      # [step, lane]
        tables.append((c, m, table))
        zero_lo = (m + 15) // 16 * 16
        assert np.all((table < m) | ((table >= zero_lo) & (table < zero_lo + 16))), "an index outside the rows and the zero rows"
        for lane in range(64):
            row = int(sched["rec_row"][g * 64 + lane])
            ids = table[:, lane]
            real = ids[ids < m]
            if row < 0:
                assert real.size == 0, "a lane without a record reads rows"
                continue
            assert label[row] == c
            got.setdefault(row, []).append(order[member_off[c] + real.astype(np.int64)])
    return label, got, tables


@pytest.mark.parametrize("order", [1, 2])
@pytest.mark.parametrize("segment_edges,budget", [(0, None), (16, 30_000)])
def test_every_in_cluster_source_is_read_exactly_once(order, segment_edges, budget):
    with community_plan(6, 300, 40_000, 5, budget, segment_edges) as plan:
        sched = plan.lds_schedule(order)
        assert sched is not None and sched["conflict_free"] == (order == 2)
        label, got, _ = decode(plan, sched)
        rowptr, col = plan.rowptr, plan.col
        for i in range(plan.n):
            src = col[rowptr[i]:rowptr[i + 1]]
            want = np.sort(src[label[src] == label[i]])
            have = np.sort(np.concatenate(got.get(i, [np.empty(0, np.int64)])))
            assert np.array_equal(want, have), f"row {i}"
        # a row finished by the pass itself (slot <= -2: "add that partial row, store the row") is one record
        # here, and the partial row it adds is none of the slots this pass writes
        slot, row = sched["rec_slot"], sched["rec_row"]
        joined = row[slot <= -2]
        assert joined.size == np.unique(joined).size and (joined.size > 0 or segment_edges)   # short segments: hardly a row is two pieces
        assert all(len(got[int(i)]) == 1 for i in joined)
        assert not np.intersect1d(-2 - slot[slot <= -2], slot[slot >= 0]).size


def test_conflict_free_order_never_puts_two_lanes_of_a_pass_on_one_bank():
    # rows of ~330 non-zeros kept whole (the default would cut them into 64s and the reads of 16 short
    # records spread less evenly over the 16 bank groups: more padding, checked below)
    with community_plan(6, 1500, 1_500_000, 9, segment_edges=1024) as plan:
        sched = plan.lds_schedule(2)
        assert sched is not None and sched["conflict_free"]
        _, _, tables = decode(plan, sched)
        for c, m, table in tables:
            for lanes in pass_groups():
                res = np.sort(table[:, lanes] & 15, axis=1)
                assert np.all(res == np.arange(16)), "two lanes of one pass share a bank group"
        # and it costs little on a dense community graph: the automatic choice takes it
        auto = plan.lds_schedule(0)
        assert auto is not None and auto["conflict_free"]
        hot = sum(int((t < m).sum()) for _, m, t in tables)
        assert sched["ids"].size <= 1.3 * hot
    with community_plan(5, 700, 120_000, 9) as plan:      # ~60 reads per record: the padding is too much, column-list order it is
        auto = plan.lds_schedule(0)
        assert auto is not None and not auto["conflict_free"]
        assert plan.lds_schedule(2)["ids"].size > 1.3 * hot_reads(plan, auto)


def hot_reads(plan, sched):
    _, _, tables = decode(plan, sched)
    return sum(int((t < m).sum()) for _, m, t in tables)


def test_conflict_free_order_on_short_records_too():
    with community_plan(5, 700, 120_000, 9, 30_000, 16) as plan:
        sched = plan.lds_schedule(2)
        _, _, tables = decode(plan, sched)
        for c, m, table in tables:
            for lanes in pass_groups():
                assert np.all(np.sort(table[:, lanes] & 15, axis=1) == np.arange(16))


def test_column_list_order_is_kept_by_order_1():
    with community_plan(4, 200, 10_000, 3) as plan:
        sched = plan.lds_schedule(1)
        label, _, tables = decode(plan, sched)
        order = np.argsort(label, kind="stable")
        member_off = np.concatenate([[0], np.cumsum(np.bincount(label))])
        rowptr, col = plan.rowptr, plan.col
        for g, (c, m, table) in enumerate(tables):
            for lane in range(64):
                row = int(sched["rec_row"][g * 64 + lane])
                if row < 0:
                    continue
                ids = table[:, lane]
                real = order[member_off[c] + ids[ids < m].astype(np.int64)]
                src = col[rowptr[row]:rowptr[row + 1]]
                want = src[label[src] == label[row]]
                if want.size == real.size:               # the row is one record
                    assert np.array_equal(real, want)
                    assert np.all(ids[real.size:] >= m), "padding comes after the reads"


def test_no_schedule_without_small_clusters():
    w = gp_synth.make_workload(2, scale=0.05, with_features=False)    # power law: one giant cluster
    with gp.gp_plan_blocks(w.src, w.dst, w.n, 10**9, w.flags) as plan:
        label, num, _, _ = plan.row_clusters()
        if np.bincount(label).max() > 10192:
            assert plan.lds_schedule(0) is None and plan.lds_schedule(2) is None
