"""CPU oracle for the LC-version forward pass over the hop stack -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this module; it shares no code with the HIP library.

What it computes (Appendix A, the LC version of GPRGNN, the equation after Eq. 13;
Section 3.1, the H^LC formula, for the single-branch special case):

    H^LC[batch] = sum_{k=0..K} gamma_k * MLP(X_k[batch]),
    MLP(Z)      = sigma(... sigma(Z W_1) ... W_{T-1}) W_T,      sigma = ReLU,

where X_k = S^k X is slab k of the precomputed hop stack and the T weight
matrices are shared by all hops.  No bias terms: the paper's formula has none.
With gamma = e_K and T = K the sum keeps the one branch
sigma(...sigma(S^K X W_1)...)W_K, which is the LC version of a K-layer GCN
(Section 3.1: COMB returning only the last term).

The general H^LC of Section 3.1 (the LC version of JKNet) combines branches of
different depth: branch k runs the first depth_k weight matrices on X_k,

    branch_k = sigma(... sigma(X_k[batch] W_1) ... W_{depth_k - 1}) W_{depth_k},
    H^LC     = COMB_k(gamma_k * branch_k),   COMB = sum, concatenation or element-wise max

(the paper's formula has depth_k = k for k = 1..K and no gamma; JKNet's COMB is
concatenation or max pooling, Appendix B).  lc_forward_branches below is that;
lc_forward is its special case depth_k = T, COMB = sum.

Everything is fp64 numpy, written as the definition: one matmul per layer, one
max(., 0) per hidden layer, one combination over hops.
"""
from __future__ import annotations

import numpy as np


def lc_forward(stack, ids, gamma, weights):
    """H^LC for the rows `ids` (Appendix A, LC version of GPRGNN).

    stack    (K+1, n, d) array-like, slab k = S^k X
    ids      (B,) row numbers of the mini-batch
    gamma    (K+1,) hop coefficients
    weights  list of T matrices, W_1 (d x h_1), W_l (h_{l-1} x h_l)
    returns  (B, h_T) float64
    """
    ids = np.asarray(ids, dtype=np.int64)
    Ws = [np.asarray(W, dtype=np.float64) for W in weights]
    H = np.zeros((ids.size, Ws[-1].shape[1]), dtype=np.float64)
    for k in range(len(gamma)):
        Z = np.asarray(stack[k][ids], dtype=np.float64)
        for W in Ws[:-1]:
            Z = np.maximum(Z @ W, 0.0)
        H += float(gamma[k]) * (Z @ Ws[-1])
    return H


def lc_bound(stack, ids, gamma, weights):
    """Entry-wise magnitude bound sum_k |gamma_k| |X_k[batch]| |W_1| ... |W_T|
    (ReLU never increases a magnitude), the scale rounding errors are measured
    against."""
    ids = np.asarray(ids, dtype=np.int64)
    Ws = [np.abs(np.asarray(W, dtype=np.float64)) for W in weights]
    Bd = np.zeros((ids.size, Ws[-1].shape[1]), dtype=np.float64)
    for k in range(len(gamma)):
        Z = np.abs(np.asarray(stack[k][ids], dtype=np.float64))
        for W in Ws:
            Z = Z @ W
        Bd += abs(float(gamma[k])) * Z
    return Bd


COMB_SUM, COMB_CONCAT, COMB_MAX = 0, 1, 2


def lc_forward_branches(stack, ids, gamma, weights, depth, comb):
    """H^LC with one branch per hop (Section 3.1, the H^LC formula).

    depth[k]  number of weight matrices branch k applies (W_1 .. W_depth[k]; the last
              one without ReLU); 0 leaves hop k out
    comb      COMB_SUM, COMB_CONCAT (branches side by side, in hop order) or COMB_MAX
    returns   (B, width) float64; sum and max need branches of one common width
    """
    ids = np.asarray(ids, dtype=np.int64)
    Ws = [np.asarray(W, dtype=np.float64) for W in weights]
    parts = []
    for k in range(len(gamma)):
        if depth[k] == 0:
            continue
        Z = np.asarray(stack[k][ids], dtype=np.float64)
        for W in Ws[:depth[k] - 1]:
            Z = np.maximum(Z @ W, 0.0)
        parts.append(float(gamma[k]) * (Z @ Ws[depth[k] - 1]))
    if comb == COMB_CONCAT:
        return np.concatenate(parts, axis=1)
    if comb == COMB_MAX:
        return np.maximum.reduce(parts)
    return np.add.reduce(parts)


def lc_bound_branches(stack, ids, gamma, weights, depth, comb):
    """Magnitude bound of every branch, combined the same way (max and sum: the sum of
    the branch bounds, which dominates both)."""
    ids = np.asarray(ids, dtype=np.int64)
    Ws = [np.abs(np.asarray(W, dtype=np.float64)) for W in weights]
    parts = []
    for k in range(len(gamma)):
        if depth[k] == 0:
            continue
        Z = np.abs(np.asarray(stack[k][ids], dtype=np.float64))
        for W in Ws[:depth[k]]:
            Z = Z @ W
        parts.append(abs(float(gamma[k])) * Z)
    if comb == COMB_CONCAT:
        return np.concatenate(parts, axis=1)
    return np.add.reduce(parts)


def softmax_rows(H):
    """Y = softmax(H^LC), row by row (Section 3.1: the predicted label matrix):
    y_c = exp(h_c) / sum_c' exp(h_c'), evaluated after subtracting the row maximum,
    which leaves the value unchanged and keeps exp in range."""
    H = np.asarray(H, dtype=np.float64)
    E = np.exp(H - H.max(axis=1, keepdims=True))
    return E / E.sum(axis=1, keepdims=True)
