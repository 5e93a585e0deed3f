"""Oracle block planner (integers only) -- TEST INFRASTRUCTURE, not product code.

What it computes, from the paper's statement of the problem:

* the non-zero set of the matrix being normalised: the adjacency list
  {(i, j) : A~_ij = 1} of A~ = A + I for a simple 0/1 adjacency matrix A
  (Section 2 preliminaries; Section 3.2 "Precomputation on GPU");
* the diagonal degree matrix D~ as the row sums of that same matrix (Eq. 1 uses
  D~ without defining it; the row-sum reading is the one under which a constant
  vector is preserved on a regular graph with self-loops, see the tests);
* the decomposition of the edge set into `b` disjoint, balanced sets whose
  union is the whole set (Section 3.2, the sentence introducing E^(1..a) and the
  identity S = sum_l D~^-1/2 A~^(l) D~^-1/2);
* the smallest block count that respects a per-block budget (the minimisation
  of Eq. 11 with a single free parameter).

Where the paper leaves a choice open the reading is fixed here so that a second
implementation can be compared bit for bit:
  - input pair (src=j, dst=i) is the non-zero (row i, col j); self pairs in the
    input are dropped; the set has no duplicates;
  - entries are listed in ascending (row, col) order;
  - block p of b is the contiguous range [p*q + min(p,r), (p+1)*q + min(p+1,r))
    of that list with q = nnz div b, r = nnz mod b  (sizes differ by at most 1);
  - b = max(1, ceil(nnz / budget));
  - dinv_sqrt = float32(1/sqrt(float64(deg))), dinv = float32(1/float64(deg)),
    0 where deg = 0.

Written with numpy only.  Nothing here is imported by the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SYMMETRISE = 1
ADD_SELF_LOOPS = 2


class OracleError(Exception):
    """kind is one of INVALID_ARG, INDEX_RANGE, OVERFLOW."""

    def __init__(self, kind: str, msg: str = ""):
        super().__init__(f"{kind}: {msg}")
        self.kind = kind


@dataclass
class OraclePlan:
    n: int
    flags: int
    row: np.ndarray        # int32 [nnz]   ascending (row, col)
    col: np.ndarray        # int32 [nnz]
    rowptr: np.ndarray     # int64 [n+1]
    deg: np.ndarray        # int32 [n]
    dinv_sqrt: np.ndarray  # float32 [n]
    dinv: np.ndarray       # float32 [n]
    block_off: np.ndarray  # int64 [b+1]
    block_row_lo: np.ndarray  # int32 [b]  row of the block's first entry (0 if empty)
    block_row_hi: np.ndarray  # int32 [b]  row of the block's last entry (-1 if empty)

    @property
    def nnz(self) -> int:
        return int(self.row.shape[0])

    @property
    def num_blocks(self) -> int:
        return int(self.block_off.shape[0] - 1)


def block_offsets(nnz: int, budget: int) -> np.ndarray:
    """Equal-count contiguous split: smallest b with ceil(nnz/b) <= budget."""
    if budget <= 0:
        raise OracleError("INVALID_ARG", "budget must be positive")
    b = max(1, -(-nnz // budget))
    q, r = divmod(nnz, b)
    p = np.arange(b + 1, dtype=np.int64)
    return p * q + np.minimum(p, r)


def plan_blocks(src, dst, n: int, block_budget_edges: int, flags: int) -> OraclePlan:
    src = np.asarray(src)
    dst = np.asarray(dst)
    if src.shape != dst.shape or src.ndim != 1:
        raise OracleError("INVALID_ARG", "src and dst must be 1-D and equally long")
    if n <= 0 or n > 2**31 - 1:
        raise OracleError("INVALID_ARG", "n out of range")
    if block_budget_edges <= 0:
        raise OracleError("INVALID_ARG", "budget must be positive")
    if flags & ~(SYMMETRISE | ADD_SELF_LOOPS):
        raise OracleError("INVALID_ARG", "unknown flag")
    s = src.astype(np.int64)
    t = dst.astype(np.int64)
    if s.size and (s.min() < 0 or t.min() < 0 or s.max() >= n or t.max() >= n):
        raise OracleError("INDEX_RANGE", "node id outside [0, n)")

    keep = s != t                      # input self pairs are dropped
    s, t = s[keep], t[keep]
    keys = [(t << 32) | s]             # (row = destination, col = source)
    if flags & SYMMETRISE:
        keys.append((s << 32) | t)
    if flags & ADD_SELF_LOOPS:
        i = np.arange(n, dtype=np.int64)
        keys.append((i << 32) | i)
    keys = np.unique(np.concatenate(keys))   # a set, in ascending (row, col) order
    nnz = int(keys.size)

    row = (keys >> 32).astype(np.int32)
    col = (keys & 0xFFFFFFFF).astype(np.int32)
    deg64 = np.bincount(row, minlength=n).astype(np.int64)
    deg = deg64.astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg64, out=rowptr[1:])

    degf = deg64.astype(np.float64)
    with np.errstate(divide="ignore"):
        dinv_sqrt = np.where(deg64 > 0, 1.0 / np.sqrt(degf), 0.0).astype(np.float32)
        dinv = np.where(deg64 > 0, 1.0 / degf, 0.0).astype(np.float32)

    off = block_offsets(nnz, block_budget_edges)
    b = off.size - 1
    lo = np.zeros(b, dtype=np.int32)
    hi = np.full(b, -1, dtype=np.int32)
    for p in range(b):
        if off[p + 1] > off[p]:
            lo[p] = row[off[p]]
            hi[p] = row[off[p + 1] - 1]
    return OraclePlan(n, flags, row, col, rowptr, deg, dinv_sqrt, dinv, off, lo, hi)
