"""Bounds on the hop kernel's HBM fetch from the popularity of source rows alone.

Independent-reference model of the gathers of one hop (a source row is drawn with probability
proportional to the number of non-zeros it is the source of):

  * an LRU cache of C rows per XCD (Che's approximation): what a 4 MiB L2 does by itself,
  * an ideal cache that pins the C most popular rows: what no L2 can be made to do, and what
    the hubs-from-LDS pass does for its 10,192 rows,

for S column slices (a slice of a row that does not start on a 128-byte line boundary touches
one more line).  Prints one JSON line per (workload, S, share of the L2 counted on); the
measured figures to set beside them are FETCH_SIZE of bench_counters.py.

    python -m paper_2207_12000_amd.cache_model --workloads 2 3
"""
from __future__ import annotations

import argparse
import json

import numpy as np
from scipy.optimize import brentq

L2_BYTES = 4 << 20
LINE = 128
LDS_ROWS = 10192


def model(workload: int, scale: float = 1.0):
    import gp_synth
    import paper_2207_12000_amd as gp
    w = gp_synth.make_workload(workload, scale=scale, with_features=False)
    budget = w.block_budget_edges or -(-gp_synth.stored_nonzeros_upper_bound(w.n, w.m, w.flags) // w.n_blocks)
    out = []
    with gp.gp_plan_blocks(w.src, w.dst, w.n, budget, w.flags) as plan:
        uses = np.bincount(plan.col, minlength=w.n).astype(np.float64)
        nnz = plan.nnz
        p = uses / uses.sum()
        cum = np.cumsum(np.sort(uses)[::-1]) / nnz
        row_bytes = w.d * 4
        for S in (1, 2, 4):
            slice_bytes = -(-w.d // (4 * S)) * 16
            unaligned = row_bytes % LINE != 0 or (S > 1 and slice_bytes % LINE != 0)
            lines = 1 + (slice_bytes - 16) / LINE if unaligned else slice_bytes / LINE
            line_bytes = lines * LINE
            gathered = nnz * S * line_bytes            # bytes of the lines all gathers touch, per hop
            other = 4 * nnz * S + w.n * w.d * 4        # column ids once per slice, the rows written
            for share in (1.0, 0.75):
                C = int(L2_BYTES * share / line_bytes)
                pinned = float(cum[min(C, w.n) - 1])
                T = brentq(lambda t: np.sum(1 - np.exp(-p * t)) - C, 1, 1e13)
                lru = float(np.sum(p * (1 - np.exp(-p * T))))
                out.append({"workload": workload, "slices": S, "slice_bytes": slice_bytes, "lines_per_slice": round(lines, 2),
                            "l2_share": share, "rows_cached": C, "hit_pinned": round(pinned, 3), "hit_lru": round(lru, 3),
                            "fetch_GB_all_miss": round((gathered + other) / 1e9, 2),
                            "fetch_GB_pinned": round((gathered * (1 - pinned) + other) / 1e9, 2),
                            "fetch_GB_lru": round((gathered * (1 - lru) + other) / 1e9, 2)})
            if S == 1:
                hubs = float(cum[min(LDS_ROWS, w.n) - 1])
                # the hubs leave the gather stream altogether; what is left meets an L2 that holds none of it for long
                rest = gathered * (1 - hubs)
                planes = 2 * w.n * (-(-w.d // 32)) * LINE   # plane entries written by the LDS launch, read by the segment launch
                out.append({"workload": workload, "slices": 1, "rows_in_lds": min(LDS_ROWS, w.n), "hot_fraction": round(hubs, 3),
                            "fetch_GB_segment_launch_all_miss": round((rest + 4 * nnz + w.n * w.d * 4 + planes / 2) / 1e9, 2)})
    return out


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workloads", type=int, nargs="+", default=[2, 3])
    ap.add_argument("--scale", type=float, default=1.0)
    a = ap.parse_args()
    for wl in a.workloads:
        for rec in model(wl, a.scale):
            print(json.dumps(rec), flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
