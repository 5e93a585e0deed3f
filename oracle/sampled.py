"""Row-by-row oracle straight from the input pair list -- TEST INFRASTRUCTURE.

For graphs too large for the full oracle planner: the neighbour sets of a few
sampled destination rows, and the degrees of every node those rows touch, are
read off the definition (pairs with src != dst, both orientations when
symmetrising, the diagonal when self-loops are added, duplicates collapsing; degree =
row sum of that 0/1 matrix) by scanning the pair list with boolean look-up tables.
Nothing of the sorted / blocked plan is built, and nothing here comes from the library.
"""
from __future__ import annotations

import numpy as np

from .plan import ADD_SELF_LOOPS, SYMMETRISE, OracleError


def neighbourhoods(src, dst, n: int, flags: int, rows, chunk: int = 1 << 26, progress=None):
    """Returns (cols, deg): cols[t] = ascending distinct column ids of row rows[t];
    deg = dict node -> degree for every node in rows or in any cols[t]."""
    rows = np.asarray(rows, dtype=np.int64)
    if rows.size and (rows.min() < 0 or rows.max() >= n):
        raise OracleError("INDEX_RANGE", "sampled row outside [0, n)")
    sym, loops = bool(flags & SYMMETRISE), bool(flags & ADD_SELF_LOOPS)
    m = len(src)

    def pairs_into(targets: np.ndarray):
        """All non-zeros (row, col) with row in `targets`, as two int64 arrays (with duplicates)."""
        lut = np.zeros(n, dtype=bool)
        lut[targets] = True
        rr, cc = [], []
        for s0 in range(0, m, chunk):
            s = np.asarray(src[s0:s0 + chunk])
            t = np.asarray(dst[s0:s0 + chunk])
            ok = s != t
            hit = lut[t] & ok                     # pair (src=j, dst=i): non-zero (row i, col j)
            rr.append(t[hit].astype(np.int64))
            cc.append(s[hit].astype(np.int64))
            if sym:
                hit = lut[s] & ok                 # and its mirror (row j, col i)
                rr.append(s[hit].astype(np.int64))
                cc.append(t[hit].astype(np.int64))
            if progress:
                progress("pairs scanned", min(s0 + chunk, m), m)
        if loops:
            rr.append(targets.astype(np.int64))
            cc.append(targets.astype(np.int64))
        return np.concatenate(rr) if rr else np.empty(0, np.int64), np.concatenate(cc) if cc else np.empty(0, np.int64)

    urows = np.unique(rows)
    r, c = pairs_into(urows)
    keys = np.unique(r * n + c)                   # the set, ascending (row, col)
    r, c = keys // n, keys % n
    starts = np.searchsorted(r, urows, side="left")
    ends = np.searchsorted(r, urows, side="right")
    by_row = {int(i): c[a:b] for i, a, b in zip(urows, starts, ends)}
    cols = [by_row[int(i)] for i in rows]

    touched = np.unique(np.concatenate([urows] + [by_row[int(i)] for i in urows]))
    r2, c2 = pairs_into(touched)
    k2 = np.unique(r2 * n + c2)
    cnt = np.searchsorted(k2 // n, touched, side="right") - np.searchsorted(k2 // n, touched, side="left")
    deg = dict(zip(touched.tolist(), cnt.tolist()))
    return cols, deg


def hop_rows(cols, deg, rows, Xprev, agg: int):
    """Rows `rows` of A^ Xprev from their neighbour lists and degrees, fp64.
    Xprev[index_array] must return the (exactly widened) feature rows.
    Returns (values, bound) like oracle.hop_rows."""
    d = Xprev.shape[1]
    Y = np.zeros((len(rows), d))
    B = np.zeros((len(rows), d))
    for t, i in enumerate(rows):
        cs = cols[t]
        di = float(deg[int(i)])
        if agg == 0:
            dj = np.array([deg[int(j)] for j in cs], dtype=np.float64)
            with np.errstate(divide="ignore"):
                w = np.where((di > 0) & (dj > 0), 1.0 / np.sqrt(di * dj), 0.0)
        elif agg == 1:
            w = np.full(cs.size, 1.0 / di if di > 0 else 0.0)
        else:
            w = np.ones(cs.size)
        xs = np.asarray(Xprev[cs], dtype=np.float64)
        Y[t] = (w[:, None] * xs).sum(axis=0)
        B[t] = (w[:, None] * np.abs(xs)).sum(axis=0)
    return Y, B
