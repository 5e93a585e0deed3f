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

Everything is fp64 numpy, written as the definition: one matmul per layer, one
max(., 0) per hidden layer, one weighted sum over hops.
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
