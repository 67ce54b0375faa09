"""Pins of the oracle's additive key bias (padding mask) against things other than itself.

The paper has no mask; the reading taken is: bias[j] is added to the scaled score in fp32 BEFORE
the N:M comparison, -inf masks a key.  Pins: identities (zero bias, constant bias), reduction to
the unmasked function on a truncated key set, a library routine for N = M, brute force on tiny
inputs, and a planted mistake (bias applied after the selection) that the brute-force case catches.
None of these needs a GPU.
"""
import numpy as np
import torch

import oracle


def _rng(seed):
    return np.random.default_rng(seed)


def _int_qkv(r, BH, Lq, Lk, d):
    Q = r.integers(-4, 5, size=(BH, Lq, d)).astype(np.float32)
    K = r.integers(-4, 5, size=(BH, Lk, d)).astype(np.float32)
    V = r.standard_normal((BH, Lk, d)).astype(np.float32)
    return Q, K, V


def test_zero_bias_is_no_bias():
    r = _rng(11)
    Q, K, V = (r.standard_normal(s).astype(np.float32) for s in ((4, 16, 32), (4, 24, 32), (4, 24, 32)))
    a = oracle.attention(Q, K, V, 2, 4, 0.2)
    b = oracle.attention(Q, K, V, 2, 4, 0.2, key_bias=np.zeros((2, 24), np.float32), heads_per_batch=2)
    assert np.array_equal(a, b)


def test_add_key_bias_is_a_row_broadcast_fp32_add():
    r = _rng(12)
    S = r.standard_normal((5, 12)).astype(np.float32)
    bias = r.standard_normal(12).astype(np.float32)
    bias[3] = -np.inf
    got = oracle.add_key_bias(S, bias)
    assert np.array_equal(got, (S + bias[None, :]).astype(np.float32))
    assert np.all(np.isneginf(got[:, 3]))


def test_constant_bias_changes_nothing():
    """A constant over all keys shifts every score alike: same selection, same softmax.
    Integer scores and a power-of-two constant keep the shifted scores exact."""
    r = _rng(13)
    Q, K, V = _int_qkv(r, 2, 16, 32, 64)
    a = oracle.attention(Q, K, V, 2, 4, 0.125)
    b = oracle.attention(Q, K, V, 2, 4, 0.125, key_bias=np.full((2, 32), 4.0, np.float32))
    assert np.max(np.abs(a - b)) < 1e-6


def test_masked_aligned_suffix_equals_truncated_keys():
    """Keys Lv.. masked with Lv a multiple of M: every group is all-real or all-masked, masked groups
    get weight exactly 0, so the result is the unmasked function on the first Lv keys."""
    r = _rng(14)
    BH, Lq, Lk, d, Lv = 3, 16, 48, 32, 28
    Q, K, V = (r.standard_normal(s).astype(np.float32) for s in ((BH, Lq, d), (BH, Lk, d), (BH, Lk, d)))
    bias = np.zeros((BH, Lk), np.float32)
    bias[:, Lv:] = -np.inf
    for N, M in ((2, 4), (1, 2)):
        got = oracle.attention(Q, K, V, N, M, 0.3, key_bias=bias)
        ref = oracle.attention(Q, K[:, :Lv], V[:, :Lv], N, M, 0.3)
        assert np.max(np.abs(got - ref)) < 1e-6


def test_per_batch_bias_is_shared_by_the_heads_of_a_batch_element():
    r = _rng(15)
    B, H, Lq, Lk, d = 2, 3, 8, 16, 16
    Q, K, V = (r.standard_normal(s).astype(np.float32) for s in ((B * H, Lq, d), (B * H, Lk, d), (B * H, Lk, d)))
    bias = np.zeros((B, Lk), np.float32)
    bias[0, 12:] = -np.inf
    bias[1, 4:8] = -np.inf
    got = oracle.attention(Q, K, V, 2, 4, 0.25, key_bias=bias, heads_per_batch=H)
    for h in range(B * H):
        ref = oracle.attention(Q[h], K[h], V[h], 2, 4, 0.25, key_bias=bias[h // H])
        assert np.array_equal(got[h], ref)


def test_dense_case_equals_library_masked_softmax():
    """N = M keeps everything: Eq. 1 with an additive mask, checked against torch in float64
    with arbitrary (unaligned, scattered) masked keys and finite biases."""
    r = _rng(16)
    Lq, Lk, d = 12, 20, 16
    Q, K, V = (r.standard_normal(s).astype(np.float32) for s in ((Lq, d), (Lk, d), (Lk, d)))
    bias = (r.standard_normal(Lk) * 2).astype(np.float32)
    bias[[1, 2, 7, 13, 19]] = -np.inf
    got = oracle.attention(Q, K, V, 4, 4, 0.25, key_bias=bias)
    S = torch.from_numpy(Q).double() @ torch.from_numpy(K).double().T * 0.25 + torch.from_numpy(bias).double()
    ref = (torch.softmax(S, -1) @ torch.from_numpy(V).double()).numpy()
    assert np.max(np.abs(got - ref)) < 1e-5


def _brute_force(Q, K, V, bias, N, M, scale):
    """Definition written out with Python numbers: per group the N largest biased scores (ties ->
    lower index), softmax over the kept ones, weighted sum of V rows."""
    Lq, Lk = Q.shape[0], K.shape[0]
    S = (Q.astype(np.float64) @ K.astype(np.float64).T) * scale + bias.astype(np.float64)[None, :]
    O = np.zeros((Lq, V.shape[1]))
    masks = np.zeros((Lq, Lk), np.uint8)
    for i in range(Lq):
        kept = []
        for g in range(Lk // M):
            idx = list(range(g * M, (g + 1) * M))
            order = sorted(idx, key=lambda j: (-S[i, j], j))     # larger first, then lower index
            kept += sorted(order[:N])
        masks[i, kept] = 1
        m = max(S[i, j] for j in kept)
        w = np.array([np.exp(S[i, j] - m) for j in kept])
        w /= w.sum()
        for wj, j in zip(w, kept):
            O[i] += wj * V[j].astype(np.float64)
    return O, masks


def test_unaligned_mask_against_brute_force():
    """Integer Q, K (exact scores, many ties) and masked keys that cut through groups."""
    r = _rng(17)
    Lq, Lk, d = 10, 24, 16
    Q = r.integers(-3, 4, size=(Lq, d)).astype(np.float32)
    K = r.integers(-3, 4, size=(Lk, d)).astype(np.float32)
    V = r.standard_normal((Lk, d)).astype(np.float32)
    bias = np.zeros(Lk, np.float32)
    bias[[0, 5, 6, 7, 9, 14, 17, 18, 19, 22]] = -np.inf     # groups with 1, 2, 3 masked keys; no group fully masked
    bias[20:24] = -np.inf                                    # ... and one fully masked group
    for N, M in ((2, 4), (1, 2)):
        ref, ref_mask = _brute_force(Q, K, V, bias, N, M, 0.125)
        got = oracle.attention(Q, K, V, N, M, 0.125, key_bias=bias)
        assert np.max(np.abs(got - ref)) < 1e-5
        S = oracle.add_key_bias(oracle.scores(Q, K, 0.125), bias)
        mask, vals, kidx = oracle.prune(S, N, M)
        assert np.array_equal(mask, ref_mask)
        assert np.all(mask.reshape(Lq, -1, M).sum(-1) == N)          # masked groups still emit N entries
        P = oracle.softmax_kept(vals)
        assert np.all(P[np.isneginf(vals)] == 0.0)                    # ... with weight exactly 0
        # a masked key is kept only where its group has fewer than N real keys
        real_in_group = (~np.isneginf(bias)).reshape(-1, M).sum(-1)
        kept_masked = (mask * np.isneginf(bias)[None, :]).reshape(Lq, -1, M).sum(-1)
        assert np.array_equal(kept_masked, np.broadcast_to(np.maximum(0, N - real_in_group), kept_masked.shape))


def test_planted_mistake_bias_after_selection_is_caught():
    """If the mask were applied after the selection, masked keys would displace real ones."""
    r = _rng(18)
    Lq, Lk, d = 6, 16, 8
    Q, K, V = (r.standard_normal(s).astype(np.float32) for s in ((Lq, d), (Lk, d), (Lk, d)))
    bias = np.zeros(Lk, np.float32)
    bias[[1, 6, 11, 12]] = -np.inf
    ref, _ = _brute_force(Q, K, V, bias, 2, 4, 0.3)
    # wrong order of operations, built from the oracle's own (separately pinned) pieces
    S = oracle.scores(Q, K, 0.3)
    mask, vals, kidx = oracle.prune(S, 2, 4)
    wrong = oracle.spmm(oracle.softmax_kept(vals + bias[kidx]), kidx, V)
    right = oracle.attention(Q, K, V, 2, 4, 0.3, key_bias=bias)
    assert np.max(np.abs(right - ref)) < 1e-5
    assert np.max(np.abs(wrong - ref)) > 1e-3
