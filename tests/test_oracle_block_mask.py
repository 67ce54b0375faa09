"""Pins of the oracle's block mask (hybrid blocked-ELL x N:M sparsity, App. A.1.2: blocks of the
score matrix that the block pattern prunes are skipped) against things other than itself:
identities, reduction to the unmasked function on gathered keys, a library routine for N = M, and
brute force with Python numbers.  None of these needs a GPU.
"""
import numpy as np
import torch

import oracle


def _rng(seed):
    return np.random.default_rng(seed)


def _qkv(r, Lq, Lk, d):
    return (r.standard_normal((Lq, d)).astype(np.float32), r.standard_normal((Lk, d)).astype(np.float32),
            r.standard_normal((Lk, d)).astype(np.float32))


def test_all_ones_block_mask_is_no_mask():
    r = _rng(21)
    Q, K, V = _qkv(r, 16, 32, 16)
    a = oracle.attention(Q, K, V, 2, 4, 0.3)
    b = oracle.attention(Q, K, V, 2, 4, 0.3, block_mask=np.ones((2, 4), np.uint8), block_size=8)
    assert np.array_equal(a, b)


def test_apply_block_mask_sets_exactly_the_pruned_blocks():
    r = _rng(22)
    S = r.standard_normal((12, 20)).astype(np.float32)
    bm = np.array([[1, 0, 1, 1, 0], [0, 1, 1, 0, 0], [1, 1, 0, 0, 1]], np.uint8)
    got = oracle.apply_block_mask(S, bm, 4)
    full = np.kron(bm, np.ones((4, 4), np.uint8)).astype(bool)      # library routine: block expansion
    assert np.array_equal(got[full], S[full])
    assert np.all(np.isneginf(got[~full]))


def test_each_row_block_equals_attention_on_its_gathered_key_blocks():
    """Within a row block the kept key blocks are whole multiples of M, so the masked function equals
    the unmasked function on the keys of the kept blocks, gathered in order."""
    r = _rng(23)
    bs, nq, nk, d = 8, 3, 5, 16
    Q, K, V = _qkv(r, nq * bs, nk * bs, d)
    bm = np.array([[1, 0, 0, 1, 1], [0, 1, 0, 0, 0], [1, 1, 1, 0, 1]], np.uint8)
    for N, M in ((2, 4), (1, 2)):
        got = oracle.attention(Q, K, V, N, M, 0.25, block_mask=bm, block_size=bs)
        for i in range(nq):
            keys = np.concatenate([np.arange(j * bs, (j + 1) * bs) for j in range(nk) if bm[i, j]])
            ref = oracle.attention(Q[i * bs:(i + 1) * bs], K[keys], V[keys], N, M, 0.25)
            assert np.max(np.abs(got[i * bs:(i + 1) * bs] - ref)) < 1e-6


def test_same_mask_in_every_row_block_equals_a_key_bias():
    r = _rng(24)
    bs, nq, nk, d = 4, 4, 6, 8
    Q, K, V = _qkv(r, nq * bs, nk * bs, d)
    row = np.array([1, 0, 1, 1, 0, 1], np.uint8)
    bias = np.where(np.repeat(row, bs) != 0, 0.0, -np.inf).astype(np.float32)
    a = oracle.attention(Q, K, V, 2, 4, 0.3, block_mask=np.tile(row, (nq, 1)), block_size=bs)
    b = oracle.attention(Q, K, V, 2, 4, 0.3, key_bias=bias)
    assert np.array_equal(a, b)


def test_dense_case_equals_library_masked_softmax():
    r = _rng(25)
    bs, nq, nk, d = 4, 3, 4, 8
    Q, K, V = _qkv(r, nq * bs, nk * bs, d)
    bm = np.array([[1, 1, 0, 0], [0, 1, 1, 0], [1, 0, 0, 1]], np.uint8)
    got = oracle.attention(Q, K, V, 4, 4, 0.5, block_mask=bm, block_size=bs)
    full = torch.from_numpy(np.kron(bm, np.ones((bs, bs), np.uint8)).astype(bool))
    S = (torch.from_numpy(Q).double() @ torch.from_numpy(K).double().T * 0.5).masked_fill(~full, float("-inf"))
    ref = (torch.softmax(S, -1) @ torch.from_numpy(V).double()).numpy()
    assert np.max(np.abs(got - ref)) < 1e-5


def test_block_mask_and_key_bias_together_against_brute_force():
    """Integer Q, K (ties), a block pattern and a padding mask that cuts through a kept block."""
    r = _rng(26)
    bs, nq, nk, d = 8, 2, 3, 16
    Lq, Lk = nq * bs, nk * bs
    Q = r.integers(-3, 4, size=(Lq, d)).astype(np.float32)
    K = r.integers(-3, 4, size=(Lk, d)).astype(np.float32)
    V = r.standard_normal((Lk, d)).astype(np.float32)
    bm = np.array([[1, 0, 1], [1, 1, 0]], np.uint8)
    bias = np.zeros(Lk, np.float32)
    bias[5:8] = -np.inf            # inside block 0, not aligned to groups
    got = oracle.attention(Q, K, V, 2, 4, 0.125, key_bias=bias, block_mask=bm, block_size=bs)
    S = (Q.astype(np.float64) @ K.astype(np.float64).T) * 0.125 + bias.astype(np.float64)[None, :]
    ref = np.zeros((Lq, d))
    for i in range(Lq):
        s = S[i].copy()
        for j in range(nk):
            if not bm[i // bs, j]:
                s[j * bs:(j + 1) * bs] = -np.inf
        kept = []
        for g in range(Lk // 4):
            idx = list(range(4 * g, 4 * g + 4))
            kept += sorted(sorted(idx, key=lambda j: (-s[j], j))[:2])
        m = max(s[j] for j in kept)
        w = np.array([np.exp(s[j] - m) for j in kept])
        w /= w.sum()
        for wj, j in zip(w, kept):
            ref[i] += wj * V[j].astype(np.float64)
    assert np.max(np.abs(got - ref)) < 1e-5
