"""Host logic of the LDS pass (no GPU): the schedule that cuts every segment into the non-zeros
served from LDS and the others, and orders the LDS reads, is checked against the plan's own
CSR, segments and row clusters."""
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


def power_law_plan(scale, forced=False):
    w = gp_synth.make_workload(2, scale=scale, with_features=False)    # power law: one giant cluster
    gp.gp_set_option("hub_pass", 1 if forced else 0)
    try:
        return gp.gp_plan_blocks(w.src, w.dst, w.n, 10**9, w.flags)
    finally:
        gp.gp_set_option("hub_pass", 0)


def tables_of(sched):
    """Per group: (set, list length, [step, lane] table of places)."""
    member_off, list_of_set = sched["member_off"], sched["list_of_set"]
    out = []
    for g in range(sched["group_set"].size):
        c = int(sched["group_set"][g])
        l = int(list_of_set[c])
        m = int(member_off[l + 1] - member_off[l])
        assert m <= 10192
        steps = int(sched["group_steps"][g])
        assert steps % 8 == 0
        off = int(sched["group_id_off"][g])
        block = sched["ids"][off:off + steps * 64].reshape(steps // 8, 64, 8)
        table = block.transpose(0, 2, 1).reshape(steps, 64)      # [step, lane]
        zero_lo = (m + 15) // 16 * 16
        assert np.all((table < m) | ((table >= zero_lo) & (table < zero_lo + 16))), "a place outside the list and the zero rows"
        out.append((c, l, m, table))
    return out


def check_schedule(plan, sched):
    """Every segment of the plan has one position; the reads of its lane (if any) and the rest
    record's non-zeros are together exactly the segment's sources, the former all on the list
    the row's set gathers from, the latter none of them (with hubs: a segment with fewer than
    three sources on the list has no reads and keeps them); positions go set by set, most reads
    first; a group is 64 consecutive positions of one set.  Returns the per-group tables."""
    members, member_off, list_of_set = sched["members"], sched["member_off"], sched["list_of_set"]
    on_list = np.full(plan.n, -1, dtype=np.int64)
    for l in range(member_off.size - 1):
        rows = members[member_off[l]:member_off[l + 1]]
        assert np.all(np.diff(rows) > 0), "a list's rows are ascending"
        on_list[rows] = l
    segs, rest, col = plan.segments, sched["rest"], sched["col"]
    assert rest.size == segs.size
    start_of = lambda a: a["start_lo"].astype(np.int64) | (a["start_hi"].astype(np.int64) << 32)
    key = lambda a: a["row"].astype(np.int64) * (2 ** 32) + (a["slot"].astype(np.int64) + 1)
    order = np.argsort(key(segs))
    at = order[np.searchsorted(key(segs)[order], key(rest))]          # position -> plan segment
    assert np.array_equal(np.sort(at), np.arange(segs.size)), "positions are a permutation of the segments"
    seg = segs[at]
    hot_len = seg["len"].astype(np.int64) - rest["len"].astype(np.int64)
    assert np.all(hot_len >= 0) and np.array_equal(start_of(rest), start_of(seg) + hot_len)
    assert np.array_equal(rest["slice"] == 0x80, hot_len > 0) and np.all((rest["slice"] == 0) | (rest["slice"] == 0x80))
    tables = tables_of(sched)
    lane_of = {}                                                     # position -> (group, lane)
    for g, (c, l, m, table) in enumerate(tables):
        pos = sched["rec_pos"][g * 64:(g + 1) * 64]
        has = pos >= 0
        assert has[0], "a group starts with a segment that has reads"
        assert np.array_equal(pos[has] - pos[0], np.flatnonzero(has)), "a group is 64 consecutive positions"
        assert np.all(table[:, ~has] >= m), "a lane without a segment reads only zero rows"
        for lane in np.flatnonzero(has):
            assert int(pos[lane]) not in lane_of
            lane_of[int(pos[lane])] = (g, int(lane))
    assert sorted(lane_of) == list(np.flatnonzero(hot_len > 0)), "exactly the segments with reads have a lane"
    plan_col = plan.col
    set_of_pos = np.full(rest.size, -1, dtype=np.int64)
    for p in range(rest.size):
        row = int(rest["row"][p])
        s0 = int(start_of(seg)[p])
        want = np.sort(plan_col[s0:s0 + int(seg["len"][p])])
        cold = col[int(start_of(rest)[p]):int(start_of(rest)[p]) + int(rest["len"][p])]
        if p in lane_of:
            g, lane = lane_of[p]
            c, l, m, table = tables[g]
            places = table[:, lane]
            hot = members[member_off[l] + places[places < m].astype(np.int64)]
            set_of_pos[p] = c
            assert np.all(on_list[cold] != l), f"position {p}: a source on the list was left to the segment kernel"
        else:
            hot = np.empty(0, np.int32)
        assert hot.size == hot_len[p]
        assert np.array_equal(np.sort(np.concatenate([hot, cold])), want), f"position {p} (row {row})"
        if p in lane_of or sched["hot_mode"] != 2:
            assert np.all(np.diff(cold) > 0)                          # the rest keeps its order
        else:
            # hubs: a segment with fewer than three sources on the list keeps them, ahead of its others
            mine = on_list[cold] == 0
            k = int(mine.sum())
            assert k < 3 and np.all(mine[:k]) and np.all(np.diff(cold[:k]) > 0) and np.all(np.diff(cold[k:]) > 0)
    # set by set, most reads first
    known = set_of_pos >= 0
    assert np.all(np.diff(set_of_pos[known]) >= 0)
    for c in np.unique(set_of_pos[known]):
        idx = np.flatnonzero(set_of_pos == c)
        assert np.all(np.diff(hot_len[idx]) <= 0)
    return tables, on_list, hot_len


@pytest.mark.parametrize("order", [1, 2])
@pytest.mark.parametrize("segment_edges,budget", [(0, None), (16, 30_000)])
def test_every_source_is_taken_exactly_once_clusters(order, segment_edges, budget):
    with community_plan(6, 300, 40_000, 5, budget, segment_edges) as plan:
        sched = plan.lds_schedule(order)
        assert sched is not None and sched["conflict_free"] == (order == 2) and sched["hot_mode"] == 1
        label, num, _, _ = plan.row_clusters()
        assert sched["list_of_set"].size == num and np.array_equal(sched["list_of_set"], np.arange(num))
        assert np.array_equal(sched["members"], np.argsort(label, kind="stable"))     # sets = lists = clusters
        check_schedule(plan, sched)


def extra_passes(sched):
    """(steps x pass groups, LDS passes beyond one per step and pass group) of a schedule."""
    total = extra = 0
    for c, l, m, table in tables_of(sched):
        for lanes in pass_groups():
            res = table[:, lanes] & 15
            most = np.array([np.bincount(r, minlength=16).max() for r in res])
            total += res.shape[0]
            extra += int((most - 1).sum())
    return total, extra


def test_conflict_free_order_keeps_the_lanes_of_a_pass_on_different_banks():
    """Order 2 reads as many 16-byte rows as the column list's order (same steps) and places them so that the
    16 lanes of a pass read 16 different bank groups, except where a bank group has more reads than there are
    steps: that surplus meets one other read (a two-way conflict).  On rows kept whole (~330 non-zeros) the
    surplus is small; the column list's order costs 2.5 extra passes per step."""
    with community_plan(6, 1500, 1_500_000, 9, segment_edges=1024) as plan:
        free, plain, auto = plan.lds_schedule(2), plan.lds_schedule(1), plan.lds_schedule(0)
        assert free["conflict_free"] and not plain["conflict_free"] and auto["conflict_free"]
        assert free["ids"].size == plain["ids"].size and np.array_equal(free["group_steps"], plain["group_steps"])
        total, extra = extra_passes(free)
        assert extra <= 0.25 * total
        for c, l, m, table in tables_of(free):
            for lanes in pass_groups():
                res = table[:, lanes] & 15
                assert max(np.bincount(r, minlength=16).max() for r in res) <= 6
        total_plain, extra_plain = extra_passes(plain)
        assert extra_plain >= 2.0 * total_plain
        check_schedule(plan, free)
    with community_plan(5, 700, 120_000, 9) as plan:      # five sets of ~60,000 reads each: too little work per staged strip, left to the L2s
        assert plan.lds_schedule(2)["ids"].size < 5 * 100_000 and plan.lds_schedule(0) is None
    with community_plan(4, 1500, 800_000, 11) as plan:    # ~60 reads per segment, 500,000 per set: taken
        auto = plan.lds_schedule(0)
        assert auto is not None and auto["conflict_free"] and auto["ids"].size >= 4 * 100_000


def test_conflict_free_order_on_short_segments_too():
    with community_plan(5, 700, 120_000, 9, 30_000, 16) as plan:
        free, plain = plan.lds_schedule(2), plan.lds_schedule(1)
        check_schedule(plan, free)
        (t2, e2), (t1, e1) = extra_passes(free), extra_passes(plain)
        assert t2 == t1 and e2 < 0.5 * e1


def test_column_list_order_is_kept_by_order_1():
    with community_plan(4, 200, 10_000, 3) as plan:
        sched = plan.lds_schedule(1)
        tables, on_list, hot_len = check_schedule(plan, sched)
        members, member_off, col = sched["members"], sched["member_off"], sched["col"]
        rest = sched["rest"]
        start = rest["start_lo"].astype(np.int64) | (rest["start_hi"].astype(np.int64) << 32)
        for g, (c, l, m, table) in enumerate(tables):
            for lane in range(64):
                p = int(sched["rec_pos"][g * 64 + lane])
                if p < 0:
                    continue
                places = table[:, lane]
                h = int(hot_len[p])
                assert np.all(places[:h] < m) and np.all(places[h:] >= m), "padding comes after the reads"
                # the hot part sits in front of the rest in the reordered column list, in the same order
                assert np.array_equal(members[member_off[l] + places[:h].astype(np.int64)], col[start[p] - h:start[p]])


@pytest.mark.parametrize("order", [1, 2])
def test_hubs_are_the_list_of_a_graph_without_clusters(order):
    with power_law_plan(0.2, forced=True) as plan:    # (the graph is too small for the automatic choice)
        sched = plan.lds_schedule(order, d=100)
        assert sched is not None and sched["hot_mode"] == 2
        assert sched["member_off"].size == 2 and np.all(sched["list_of_set"] == 0)
        hubs = sched["members"]
        assert hubs.size == min(10192, plan.n)
        # they are the most popular sources, ties to the smaller id
        uses = np.bincount(plan.col, minlength=plan.n)
        order_by_use = np.lexsort((np.arange(plan.n), -uses))
        assert np.array_equal(np.sort(order_by_use[:hubs.size]), hubs)
        check_schedule(plan, sched)
        # sets are ranges of consecutive rows
        rest = sched["rest"]
        flagged = rest["slice"] == 0x80
        sets = np.repeat(sched["group_set"], 64)[sched["rec_pos"] >= 0]
        rows = rest["row"][sched["rec_pos"][sched["rec_pos"] >= 0]]
        for c in np.unique(sets)[:-1]:
            assert rows[sets == c].max() < rows[sets == c + 1].min()
        assert flagged.sum() == (sched["rec_pos"] >= 0).sum()


def test_no_schedule_by_itself_for_a_small_power_law_graph():
    """One giant cluster of more rows than an L2 share holds, and too little work for hubs to be tried."""
    with power_law_plan(0.2) as plan:
        assert plan.nnz * 128 < 2e9 and plan.lds_schedule(0) is None and plan.lds_schedule(2) is None
