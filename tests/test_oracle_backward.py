"""Pins of the oracle's backward pass (gradients through the fixed N:M selection) against things
other than itself: automatic differentiation of the same function written with library routines in
float64 (mask held constant), the dense special case N = M, central finite differences on an input
whose selection cannot flip, and structural facts (rows of dS sum to zero, dropped keys get no dV).
None of these needs a GPU.
"""
import numpy as np
import torch

import oracle


def _rng(seed):
    return np.random.default_rng(seed)


def _forward_pieces(Q, K, V, N, M, scale, bias=None):
    S = oracle.scores(Q, K, scale)
    if bias is not None:
        S = oracle.add_key_bias(S, bias)
    mask, vals, kidx = oracle.prune(S, N, M)
    P = oracle.softmax_kept(vals)
    return S, mask, kidx, P


def _autograd_reference(Q, K, V, dO, mask, scale, bias=None):
    """The forward function with library routines in float64, mask as a constant; gradients by autograd."""
    q = torch.tensor(Q, dtype=torch.float64, requires_grad=True)
    k = torch.tensor(K, dtype=torch.float64, requires_grad=True)
    v = torch.tensor(V, dtype=torch.float64, requires_grad=True)
    s = q @ k.T * scale
    if bias is not None:
        s = s + torch.tensor(bias, dtype=torch.float64)
    s = s.masked_fill(~torch.tensor(mask.astype(bool)), float("-inf"))
    o = torch.softmax(s, -1) @ v
    o.backward(torch.tensor(dO, dtype=torch.float64))
    return q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


def test_backward_matches_autograd_with_constant_mask():
    r = _rng(31)
    Lq, Lk, d = 20, 32, 16
    Q, K, V, dO = (r.standard_normal(s).astype(np.float32) for s in ((Lq, d), (Lk, d), (Lk, d), (Lq, d)))
    for N, M in ((2, 4), (1, 2)):
        S, mask, kidx, P = _forward_pieces(Q, K, V, N, M, 0.3)
        dQ, dK, dV = oracle.attention_backward(Q, K, V, dO, P, kidx, 0.3)
        rQ, rK, rV = _autograd_reference(Q, K, V, dO, mask, 0.3)
        for got, ref in ((dQ, rQ), (dK, rK), (dV, rV)):
            assert np.max(np.abs(got - ref)) < 1e-5 * max(1.0, np.max(np.abs(ref)))


def test_backward_dense_case_is_plain_attention_backward():
    r = _rng(32)
    Lq, Lk, d = 12, 16, 8
    Q, K, V, dO = (r.standard_normal(s).astype(np.float32) for s in ((Lq, d), (Lk, d), (Lk, d), (Lq, d)))
    S, mask, kidx, P = _forward_pieces(Q, K, V, 4, 4, 0.5)
    assert mask.all()
    dQ, dK, dV = oracle.attention_backward(Q, K, V, dO, P, kidx, 0.5)
    q, k, v = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    (torch.softmax(q @ k.T * 0.5, -1) @ v).backward(torch.tensor(dO, dtype=torch.float64))
    for got, ref in ((dQ, q.grad), (dK, k.grad), (dV, v.grad)):
        assert np.max(np.abs(got - ref.numpy())) < 1e-5


def test_backward_with_key_bias_matches_autograd():
    r = _rng(33)
    Lq, Lk, d = 10, 24, 8
    Q, K, V, dO = (r.standard_normal(s).astype(np.float32) for s in ((Lq, d), (Lk, d), (Lk, d), (Lq, d)))
    bias = np.zeros(Lk, np.float32)
    bias[17:] = -np.inf
    S, mask, kidx, P = _forward_pieces(Q, K, V, 2, 4, 0.4, bias)
    dQ, dK, dV = oracle.attention_backward(Q, K, V, dO, P, kidx, 0.4)
    rQ, rK, rV = _autograd_reference(Q, K, V, dO, mask * np.isfinite(bias)[None, :], 0.4, np.where(np.isfinite(bias), bias, 0.0))
    for got, ref in ((dQ, rQ), (dK, rK), (dV, rV)):
        assert np.max(np.abs(got - ref)) < 1e-5
    assert np.all(dV[17:] == 0) and np.all(dK[17:] == 0)      # masked keys receive nothing


def test_backward_against_finite_differences_on_a_stable_selection():
    """Keys built so that two keys of every run of four score far above the other two: small
    perturbations cannot change the selection, so the function is smooth and central differences of
    the oracle's own forward pass must agree with the analytic gradient."""
    r = _rng(34)
    Lq, Lk, d = 4, 8, 6
    Q = r.standard_normal((Lq, d)).astype(np.float64) * 0.3
    K = r.standard_normal((Lk, d)).astype(np.float64) * 0.3
    V = r.standard_normal((Lk, d)).astype(np.float64)
    Q[:, 0] = 3.0
    K[[0, 3, 5, 6], 0] = 4.0          # the survivors of each run, for every query
    dO = r.standard_normal((Lq, d))

    def loss(q, k, v):
        return float(np.sum(oracle.attention(q, k, v, 2, 4, 0.5).astype(np.float64) * dO))

    S, mask, kidx, P = _forward_pieces(Q, K, V, 2, 4, 0.5)
    assert np.array_equal(np.unique(kidx), [0, 3, 5, 6])
    dQ, dK, dV = oracle.attention_backward(Q, K, V, dO, P, kidx, 0.5)
    eps = 1e-2
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for idx in [(0, 0), (1, 2), (3, 5), (2, 1)] + ([(5, 3), (6, 0)] if name != "Q" else []):
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - G[idx]) < 2e-3 * max(1.0, abs(fd)), (name, idx, fd, G[idx])


def test_backward_structure():
    r = _rng(35)
    Lq, Lk, d = 16, 32, 8
    Q, K, V, dO = (r.standard_normal(s).astype(np.float32) for s in ((Lq, d), (Lk, d), (Lk, d), (Lq, d)))
    S, mask, kidx, P = _forward_pieces(Q, K, V, 2, 4, 0.3)
    dQ, dK, dV, dS = oracle.attention_backward(Q, K, V, dO, P, kidx, 0.3, return_dS=True)
    assert np.max(np.abs(dS.sum(-1))) < 1e-6                 # softmax Jacobian: rows of dS sum to zero
    never_kept = ~mask.any(0)
    if never_kept.any():
        assert np.all(dV[never_kept] == 0) and np.all(dK[never_kept] == 0)
    # dV is the transposed sparse product: check it against a dense scatter of P
    Pd = np.zeros((Lq, Lk))
    np.put_along_axis(Pd, kidx.astype(np.int64), P.astype(np.float64), axis=1)
    assert np.max(np.abs(dV - Pd.T @ dO.astype(np.float64))) < 1e-5
