"""Pins of the LC-forward oracle (Appendix A, LC version of GPRGNN) against things
other than itself: a hand-worked example, scalar brute force from the formula,
the collapse to one matrix product when no ReLU is active, the ReLU that kills
everything, the T = 1 identity-weight case that must equal the pinned polynomial
filter of the hop oracle, and the symmetries of the formula."""
import numpy as np

import oracle
from oracle import lc


def test_hand_worked_example():
    # two hops, one batch row each worked by hand:
    #  hop 0 row [2, 1]:  [2, 1] W1 = [2.5, 0]   -> relu [2.5, 0] -> . [2, 3] = 5
    #  hop 1 row [-1, 1]: [-1, 1] W1 = [-0.5, 3] -> relu [0, 3]   -> . [2, 3] = 9
    #  H = 0.5 * 5 + 2 * 9 = 20.5
    stack = np.array([[[2.0, 1.0]], [[-1.0, 1.0]]])
    W1 = np.array([[1.0, -1.0], [0.5, 2.0]])
    W2 = np.array([[2.0], [3.0]])
    H = lc.lc_forward(stack, [0], [0.5, 2.0], [W1, W2])
    assert H.shape == (1, 1) and H[0, 0] == 20.5


def _brute(stack, ids, gamma, Ws):
    out = []
    for i in ids:
        acc = [0.0] * Ws[-1].shape[1]
        for k, g in enumerate(gamma):
            z = [float(v) for v in stack[k][i]]
            for t, W in enumerate(Ws):
                nz = []
                for c in range(W.shape[1]):
                    s = 0.0
                    for r in range(W.shape[0]):
                        s += z[r] * float(W[r, c])
                    if t < len(Ws) - 1 and s < 0.0:
                        s = 0.0
                    nz.append(s)
                z = nz
            for c in range(len(acc)):
                acc[c] += g * z[c]
        out.append(acc)
    return np.array(out)


def test_scalar_brute_force():
    rng = np.random.default_rng(11)
    for T in (1, 2, 3, 4):
        dims = [5] + [6, 4, 7][:T - 1] + [3]
        stack = rng.normal(size=(3, 9, 5))
        Ws = [rng.normal(size=(dims[t], dims[t + 1])) for t in range(T)]
        ids = [8, 0, 3, 3]
        gamma = rng.normal(size=3)
        got = lc.lc_forward(stack, ids, gamma, Ws)
        assert np.allclose(got, _brute(stack, ids, gamma, Ws), rtol=1e-12, atol=1e-12)


def test_no_active_relu_collapses_to_one_product():
    rng = np.random.default_rng(12)
    stack = rng.uniform(0, 1, size=(4, 20, 6))
    Ws = [rng.uniform(0, 1, size=s) for s in ((6, 8), (8, 8), (8, 5))]
    gamma = np.array([0.4, 0.3, 0.2, 0.1])
    ids = np.arange(20)[::-1]
    P = Ws[0] @ (Ws[1] @ Ws[2])                       # right-to-left association
    want = np.tensordot(gamma, stack[:, ids, :], axes=1) @ P
    assert np.allclose(lc.lc_forward(stack, ids, gamma, Ws), want, rtol=1e-12)


def test_relu_kills_negative_first_layer():
    rng = np.random.default_rng(13)
    stack = rng.uniform(0, 1, size=(2, 5, 4))
    Ws = [-rng.uniform(0.1, 1, size=(4, 6)), rng.normal(size=(6, 3))]
    assert np.all(lc.lc_forward(stack, [0, 1, 2], [1.0, 1.0], Ws) == 0.0)
    # without a hidden layer nothing is clipped
    assert np.all(lc.lc_forward(stack, [0, 1, 2], [1.0, 1.0], Ws[:1]) < 0.0)


def test_identity_weight_equals_polynomial_filter():
    rng = np.random.default_rng(14)
    n, d, K = 40, 6, 3
    src = rng.integers(0, n, 150).astype(np.int32)
    dst = rng.integers(0, n, 150).astype(np.int32)
    plan = oracle.plan_blocks(src, dst, n, 60, oracle.SYMMETRISE | oracle.ADD_SELF_LOOPS)
    X = rng.normal(size=(n, d))
    stack = oracle.propagate(plan, X, oracle.AGG_SYM, K)
    gamma = oracle.ppr_coefficients(0.15, K)
    ids = rng.permutation(n)[:17]
    H = lc.lc_forward(stack, ids, gamma, [np.eye(d)])
    assert np.allclose(H, oracle.combine(plan, X, oracle.AGG_SYM, gamma)[0][ids], rtol=1e-12, atol=1e-14)


def test_single_branch_is_the_gcn_form():
    rng = np.random.default_rng(15)
    stack = rng.normal(size=(3, 12, 4))
    Ws = [rng.normal(size=(4, 5)), rng.normal(size=(5, 2))]
    H = lc.lc_forward(stack, np.arange(12), [0.0, 0.0, 1.0], Ws)
    assert np.allclose(H, np.maximum(stack[2] @ Ws[0], 0) @ Ws[1], rtol=1e-13)


def test_symmetries():
    rng = np.random.default_rng(16)
    stack = rng.normal(size=(3, 30, 7))
    Ws = [rng.normal(size=s) for s in ((7, 9), (9, 6), (6, 4))]
    gamma = rng.normal(size=3)
    ids = rng.integers(0, 30, 11)
    H = lc.lc_forward(stack, ids, gamma, Ws)
    # batch rows are independent: permuting the batch permutes the output rows
    p = rng.permutation(11)
    assert np.array_equal(lc.lc_forward(stack, ids[p], gamma, Ws), H[p])
    # relabelling hidden units (columns of W_l, rows of W_{l+1}) changes nothing
    q1, q2 = rng.permutation(9), rng.permutation(6)
    Wp = [Ws[0][:, q1], Ws[1][q1][:, q2], Ws[2][q2]]
    assert np.allclose(lc.lc_forward(stack, ids, gamma, Wp), H, rtol=1e-12, atol=1e-13)
    # linear in gamma, positively homogeneous in each weight matrix
    assert np.allclose(lc.lc_forward(stack, ids, 2 * gamma, Ws), 2 * H, rtol=1e-13)
    assert np.allclose(lc.lc_forward(stack, ids, gamma, [3 * Ws[0], Ws[1], 0.5 * Ws[2]]), 1.5 * H, rtol=1e-12)
    # the bound dominates
    assert np.all(np.abs(H) <= lc.lc_bound(stack, ids, gamma, Ws) * (1 + 1e-12))


def test_matches_an_independent_library_chain():
    """The same formula through torch's CPU linear / relu in fp64 (another library's
    matmul and clamp, applied hop by hop and stacked the other way round)."""
    import torch
    rng = np.random.default_rng(17)
    stack = rng.normal(size=(4, 50, 12))
    Ws = [rng.normal(size=s) for s in ((12, 20), (20, 20), (20, 20), (20, 5))]
    gamma = rng.normal(size=4)
    ids = rng.integers(0, 50, 23)
    Z = torch.from_numpy(stack[:, ids, :])                      # (hops, B, d): all hops at once
    for W in Ws[:-1]:
        Z = torch.relu(torch.nn.functional.linear(Z, torch.from_numpy(W.T.copy())))
    Z = torch.nn.functional.linear(Z, torch.from_numpy(Ws[-1].T.copy()))
    want = torch.einsum("k,kbc->bc", torch.from_numpy(gamma), Z).numpy()
    assert np.allclose(lc.lc_forward(stack, ids, gamma, Ws), want, rtol=1e-12, atol=1e-12)


def test_branches_written_out_for_two_hops():
    """The H^LC formula of Section 3.1 for K = 2, typed out term by term:
    branch 1 = (S X) W_1, branch 2 = relu((S^2 X) W_1) W_2."""
    rng = np.random.default_rng(18)
    stack = rng.normal(size=(3, 9, 4))                      # slabs X, SX, S^2 X
    W1, W2 = rng.normal(size=(4, 5)), rng.normal(size=(5, 5))
    ids = np.array([3, 1, 8])
    b1 = stack[1][ids] @ W1
    b2 = np.maximum(stack[2][ids] @ W1, 0.0) @ W2
    g = [1.0, 1.0, 1.0]
    for comb, want in ((lc.COMB_CONCAT, np.hstack([b1, b2])), (lc.COMB_MAX, np.maximum(b1, b2)), (lc.COMB_SUM, b1 + b2)):
        got = lc.lc_forward_branches(stack, ids, g, [W1, W2], depth=[0, 1, 2], comb=comb)
        assert np.allclose(got, want, rtol=1e-13, atol=1e-13)


def test_branches_reduce_to_the_shared_depth_case_and_to_single_branches():
    rng = np.random.default_rng(19)
    stack = rng.normal(size=(4, 15, 6))
    Ws = [rng.normal(size=s) for s in ((6, 7), (7, 7), (7, 7))]
    gamma = rng.normal(size=4)
    ids = rng.integers(0, 15, 8)
    # equal depth + sum is the GPRGNN form
    assert np.allclose(lc.lc_forward_branches(stack, ids, gamma, Ws, [3, 3, 3, 3], lc.COMB_SUM),
                       lc.lc_forward(stack, ids, gamma, Ws), rtol=1e-13)
    # every branch alone is a shared-depth call with one non-zero coefficient and a truncated weight list
    depth = [0, 1, 2, 3]
    singles = []
    for k in (1, 2, 3):
        e = np.zeros(4)
        e[k] = gamma[k]
        singles.append(lc.lc_forward(stack, ids, e, Ws[:depth[k]]))
    assert np.allclose(lc.lc_forward_branches(stack, ids, gamma, Ws, depth, lc.COMB_CONCAT), np.hstack(singles), rtol=1e-13)
    assert np.allclose(lc.lc_forward_branches(stack, ids, gamma, Ws, depth, lc.COMB_MAX), np.maximum.reduce(singles), rtol=1e-13)
    assert np.allclose(lc.lc_forward_branches(stack, ids, gamma, Ws, depth, lc.COMB_SUM), np.add.reduce(singles), rtol=1e-13)
    # the bound dominates under every combination
    for comb in (lc.COMB_SUM, lc.COMB_CONCAT, lc.COMB_MAX):
        H = lc.lc_forward_branches(stack, ids, gamma, Ws, depth, comb)
        assert np.all(np.abs(H) <= lc.lc_bound_branches(stack, ids, gamma, Ws, depth, comb) * (1 + 1e-12))


def test_softmax_rows():
    from scipy.special import softmax
    rng = np.random.default_rng(20)
    H = rng.normal(size=(13, 7)) * 5
    Y = lc.softmax_rows(H)
    assert np.allclose(Y, softmax(H, axis=1), rtol=1e-13)                 # library routine
    assert np.allclose(Y.sum(axis=1), 1.0, rtol=1e-14) and np.all(Y > 0)
    assert np.allclose(lc.softmax_rows(H + 1000.0), Y, rtol=1e-10)          # shift invariance, no overflow
    assert np.allclose(lc.softmax_rows(np.zeros((2, 4))), 0.25)            # uniform on equal scores
    two = lc.softmax_rows(np.array([[0.0, np.log(3.0)]]))                   # closed form: 1/4, 3/4
    assert np.allclose(two, [[0.25, 0.75]], rtol=1e-15)
