"""CPU oracle for the K-hop feature precompute -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  The HIP library never does, and this package never imports the
HIP library: the two share no code.

  plan.py       integer block planner (numpy)
  gp_oracle.c   one hop of A^ X as a plain fp64 loop over the adjacency list
  this file     builds/loads the C file and strings hops together
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .plan import (ADD_SELF_LOOPS, SYMMETRISE, OracleError, OraclePlan,  # noqa: F401
                   block_offsets, plan_blocks)

AGG_SYM, AGG_MEAN, AGG_SUM = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libgp_oracle.so")
_lib = None
_lock = threading.Lock()


def build(force: bool = False) -> str:
    """Compile gp_oracle.c with gcc (strict IEEE: no fast-math)."""
    src = os.path.join(_HERE, "gp_oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-ffp-contract=off",
                               "-o", tmp, src, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            lib.gpo_hop_range.restype = ctypes.c_int
            lib.gpo_hop_range.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                          ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
            _lib = lib
    return _lib


def _hop_range(plan: OraclePlan, agg: int, X: np.ndarray, Y: np.ndarray, lo: int, hi: int):
    lib = _load()
    rc = lib.gpo_hop_range(lo, hi, plan.row.ctypes.data, plan.col.ctypes.data,
                           plan.deg.ctypes.data, agg, X.shape[1], X.ctypes.data, Y.ctypes.data)
    if rc != 0:
        raise OracleError("INVALID_ARG", "gpo_hop_range rejected its arguments")


def hop(plan: OraclePlan, X: np.ndarray, agg: int, threads: int = 1) -> np.ndarray:
    """One hop Y = A^ X in fp64 (Algorithm 1's result for one k, without blocks).

    threads > 1 cuts the list at row boundaries and runs the same loop on the
    pieces concurrently; every row still adds its entries in list order, so the
    result is bit-identical to threads = 1."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    if X.ndim != 2 or X.shape[0] != plan.n:
        raise OracleError("INVALID_ARG", "X must be n x d")
    Y = np.zeros_like(X)
    nnz = plan.nnz
    if threads <= 1 or nnz == 0:
        _hop_range(plan, agg, X, Y, 0, nnz)
        return Y
    rows = np.searchsorted(plan.rowptr, np.linspace(0, nnz, threads + 1).astype(np.int64),
                           side="left")
    rows[0], rows[-1] = 0, plan.n
    cuts = plan.rowptr[np.clip(rows, 0, plan.n)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        futs = [ex.submit(_hop_range, plan, agg, X, Y, int(cuts[t]), int(cuts[t + 1]))
                for t in range(threads) if cuts[t + 1] > cuts[t]]
        for f in futs:
            f.result()
    return Y


def propagate(plan: OraclePlan, X: np.ndarray, agg: int, K: int, threads: int = 1):
    """[X, A^ X, ..., A^^K X] in fp64, no rounding between hops (Algorithm 1's
    list plus the k = 0 term that the Appendix A model consumes)."""
    if K < 0:
        raise OracleError("INVALID_ARG", "K must be >= 0")
    out = [np.ascontiguousarray(X, dtype=np.float64)]
    for _ in range(K):
        out.append(hop(plan, out[-1], agg, threads))
    return out


def bound_stack(plan: OraclePlan, X: np.ndarray, agg: int, K: int, threads: int = 1):
    """B_k = A^^k |X|: every weight is non-negative, so this is |A^|^k |X|, the
    cancellation-free magnitude the float tolerance is relative to."""
    return propagate(plan, np.abs(np.asarray(X, dtype=np.float64)), agg, K, threads)


def hop_rows(plan: OraclePlan, Xprev: np.ndarray, agg: int, rows) -> np.ndarray:
    """Rows `rows` of A^ Xprev computed one by one from the definition (numpy
    fp64); Xprev may be any float dtype and is widened exactly.  Returns
    (values, bound) with bound = the same sum over |Xprev|."""
    rows = np.asarray(rows, dtype=np.int64)
    d = Xprev.shape[1]
    Y = np.zeros((rows.size, d), dtype=np.float64)
    B = np.zeros((rows.size, d), dtype=np.float64)
    deg = plan.deg.astype(np.float64)
    for t, i in enumerate(rows):
        lo, hi = int(plan.rowptr[i]), int(plan.rowptr[i + 1])
        cols = plan.col[lo:hi].astype(np.int64)
        if agg == AGG_SYM:
            with np.errstate(divide="ignore"):
                w = np.where((deg[i] > 0) & (deg[cols] > 0), 1.0 / np.sqrt(deg[i] * deg[cols]), 0.0)
        elif agg == AGG_MEAN:
            w = np.full(cols.size, 1.0 / deg[i] if deg[i] > 0 else 0.0)
        else:
            w = np.ones(cols.size)
        xs = np.asarray(Xprev[cols], dtype=np.float64)
        Y[t] = (w[:, None] * xs).sum(axis=0)
        B[t] = (w[:, None] * np.abs(xs)).sum(axis=0)
    return Y, B


def combine(plan: OraclePlan, X: np.ndarray, agg: int, coeff, threads: int = 1):
    """sum_k coeff[k] * A^^k X in fp64, term by term from the hop stack (Appendix A,
    Eq. 13 with constant coefficients).  Returns (value, bound) with
    bound = sum_k |coeff[k]| * A^^k |X|."""
    coeff = [float(c) for c in coeff]
    K = len(coeff) - 1
    Y = propagate(plan, X, agg, K, threads)
    B = bound_stack(plan, X, agg, K, threads)
    val = np.zeros_like(Y[0])
    bnd = np.zeros_like(Y[0])
    for k in range(K + 1):
        val += coeff[k] * Y[k]
        bnd += abs(coeff[k]) * B[k]
    return val, bnd


def ppr_coefficients(alpha: float, K: int):
    """K-step Personalized-PageRank diffusion written as a polynomial in A^:
    Z_0 = X, Z_{t+1} = (1 - alpha) A^ Z_t + alpha X  gives
    Z_K = sum_{k<K} alpha (1-alpha)^k A^^k X + (1-alpha)^K A^^K X."""
    return [alpha * (1 - alpha) ** k for k in range(K)] + [(1 - alpha) ** K]
