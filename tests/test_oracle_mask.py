"""Pins of the oracle's per-(query, key) additive mask and of the causal mask, against things other than itself.

The paper has no mask.  Reading taken: mask[i][j] is added to the scaled score in fp32 BEFORE the N:M
comparison (as for the key bias); -inf hides key j from query i.  The causal mask hides the keys after the
query's own position, the queries being the last Lq of the Lk positions.  Pins: the mask written out by hand,
brute force on tiny inputs (pure Python selection and softmax), rows of the causal result against the unmasked
function on a truncated key set, library routines for N = M (no pruning), agreement with the key bias where the
two coincide, and planted mistakes that these cases catch.  None of these needs a GPU.
"""
import math

import numpy as np
import pytest
import torch

import oracle


def _rng(seed):
    return np.random.default_rng(seed)


def _int_qkv(r, BH, Lq, Lk, d):
    Q = r.integers(-4, 5, size=(BH, Lq, d)).astype(np.float32)
    K = r.integers(-4, 5, size=(BH, Lk, d)).astype(np.float32)
    V = r.standard_normal((BH, Lk, d)).astype(np.float32)
    return Q, K, V


def test_causal_mask_written_out():
    m = oracle.causal_mask(3, 3)
    ninf = -np.inf
    assert np.array_equal(m, np.array([[0, ninf, ninf], [0, 0, ninf], [0, 0, 0]], np.float32))
    # more keys than queries: the queries are the last positions
    m = oracle.causal_mask(2, 5)
    assert np.array_equal(m, np.array([[0, 0, 0, 0, ninf], [0, 0, 0, 0, 0]], np.float32))
    with pytest.raises(ValueError):
        oracle.causal_mask(5, 2)
    for Lq, Lk in ((7, 7), (5, 12), (1, 9)):
        m = oracle.causal_mask(Lq, Lk)
        assert np.array_equal((m == 0).sum(1), np.arange(Lq) + 1 + Lk - Lq)   # row i sees i + 1 + (Lk - Lq) keys
        assert np.all((m == 0) | np.isneginf(m))
        assert np.all(np.diff((m == 0).astype(int), axis=1) <= 0)              # visible keys form a prefix


def test_add_mask_is_an_elementwise_fp32_add():
    r = _rng(21)
    S = r.standard_normal((6, 12)).astype(np.float32)
    mask = r.standard_normal((6, 12)).astype(np.float32)
    mask[2, 5] = -np.inf
    got = oracle.add_mask(S, mask)
    assert np.array_equal(got, (S + mask).astype(np.float32))
    assert np.isneginf(got[2, 5]) and np.isfinite(np.delete(got.reshape(-1), 2 * 12 + 5)).all()


def _brute_force(Q, K, V, mask, N, M, scale):
    """One head, pure Python: scores, mask, rank rule (larger first, then lower index), softmax, weighted sum."""
    Lq, Lk = Q.shape[0], K.shape[0]
    O = np.zeros((Lq, V.shape[1]))
    kept = np.zeros((Lq, Lk), bool)
    for i in range(Lq):
        s = [float(np.float32(np.float32(np.dot(Q[i].astype(np.float64), K[j].astype(np.float64))) * np.float32(scale))
                   + np.float32(mask[i, j])) for j in range(Lk)]
        keep = []
        for g in range(0, Lk, M):
            order = sorted(range(g, g + M), key=lambda j: (-s[j], j))
            keep += sorted(order[:N])
        mx = max(s[j] for j in keep)
        w = [math.exp(s[j] - mx) if s[j] != -math.inf else 0.0 for j in keep]
        tot = sum(w)
        for j, wj in zip(keep, w):
            O[i] += wj / tot * V[j].astype(np.float64)
            kept[i, j] = True
    return O, kept


@pytest.mark.parametrize("N,M", [(2, 4), (1, 2)])
def test_brute_force_general_mask_and_causal(N, M):
    """Integer Q, K (exact scores, many ties) with a mask of small integers and -inf entries placed so that they cut
    through runs of M; and the causal mask, whose diagonal cuts through every run."""
    r = _rng(22 + N)
    Lq, Lk, d = 12, 16, 8
    Q, K, V = (a[0] for a in _int_qkv(r, 1, Lq, Lk, d))
    mask = r.integers(-2, 3, size=(Lq, Lk)).astype(np.float32)
    mask[r.random((Lq, Lk)) < 0.3] = -np.inf
    mask[:, 0] = 0.0        # every query keeps one visible key
    for m in (mask, oracle.causal_mask(Lq, Lk)):
        ref, kept = _brute_force(Q, K, V, m, N, M, 0.125)
        got = oracle.attention(Q, K, V, N, M, 0.125, mask=m)
        assert np.max(np.abs(got - ref)) < 1e-5
        S = oracle.add_mask(oracle.scores(Q, K, 0.125), m)
        okept = oracle.prune(S, N, M)[0].astype(bool)
        assert np.array_equal(okept, kept)
    # causal=True is the causal mask
    assert np.array_equal(oracle.attention(Q, K, V, N, M, 0.125, causal=True),
                          oracle.attention(Q, K, V, N, M, 0.125, mask=oracle.causal_mask(Lq, Lk)))


@pytest.mark.parametrize("Lq,Lk", [(32, 32), (16, 40)])
def test_causal_rows_equal_the_unmasked_function_on_truncated_keys(Lq, Lk):
    """Row i sees n = i + 1 + (Lk - Lq) keys.  Where n is a multiple of M every run is all-visible or all-hidden,
    hidden runs weigh exactly 0, so the row equals the unmasked function of the first n keys."""
    r = _rng(24)
    d, N, M = 16, 2, 4
    Q, K, V = (r.standard_normal(s).astype(np.float32) for s in ((Lq, d), (Lk, d), (Lk, d)))
    got = oracle.attention(Q, K, V, N, M, 0.25, causal=True)
    checked = 0
    for i in range(Lq):
        n = i + 1 + Lk - Lq
        if n % M == 0:
            ref = oracle.attention(Q[i:i + 1], K[:n], V[:n], N, M, 0.25)
            assert np.max(np.abs(got[i] - ref[0])) < 1e-6
            checked += 1
    assert checked >= Lq // M
    # the first query of a square problem sees key 0 only
    if Lq == Lk:
        assert np.allclose(got[0], V[0], atol=1e-7)


def test_without_pruning_causal_is_the_library_causal_attention():
    """N = M keeps every score: Eq. 1 with a causal mask, against torch's scaled_dot_product_attention in fp64."""
    r = _rng(25)
    BH, L, d = 3, 24, 16
    Q, K, V = (r.standard_normal((BH, L, d)).astype(np.float32) for _ in range(3))
    got = oracle.attention(Q, K, V, 4, 4, 0.25, causal=True)
    tq, tk, tv = (torch.from_numpy(a).double() for a in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=0.25).numpy()
    assert np.max(np.abs(got - ref)) < 1e-5


def test_without_pruning_general_mask_is_the_library_masked_attention():
    """A mask that is not symmetric (a transposed mask would fail) with finite and -inf entries; Lq != Lk."""
    r = _rng(26)
    BH, Lq, Lk, d = 2, 12, 20, 16
    Q, K, V = (r.standard_normal(s).astype(np.float32) for s in ((BH, Lq, d), (BH, Lk, d), (BH, Lk, d)))
    mask = r.standard_normal((Lq, Lk)).astype(np.float32)
    mask[r.random((Lq, Lk)) < 0.4] = -np.inf
    mask[:, 3] = 0.5
    got = oracle.attention(Q, K, V, 1, 1, 0.25, mask=mask)
    tq, tk, tv = (torch.from_numpy(a).double() for a in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(mask).double(),
                                                           scale=0.25).numpy()
    assert np.max(np.abs(got - ref)) < 1e-5
    # rectangular causal = bottom-right aligned triangle
    tri = torch.ones(Lq, Lk, dtype=torch.bool).tril(diagonal=Lk - Lq)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=tri, scale=0.25).numpy()
    assert np.max(np.abs(oracle.attention(Q, K, V, 2, 2, 0.25, causal=True) - ref)) < 1e-5


def test_mask_with_equal_rows_is_the_key_bias():
    r = _rng(27)
    BH, Lq, Lk, d = 4, 16, 24, 32
    Q, K, V = _int_qkv(r, BH, Lq, Lk, d)
    bias = r.integers(-3, 4, size=Lk).astype(np.float32)
    bias[[5, 6, 17]] = -np.inf
    a = oracle.attention(Q, K, V, 2, 4, 0.125, key_bias=np.tile(bias, (BH, 1)))
    b = oracle.attention(Q, K, V, 2, 4, 0.125, mask=np.tile(bias, (Lq, 1)))
    assert np.array_equal(a, b)
    # and the two add up when both are given
    c = oracle.attention(Q, K, V, 2, 4, 0.125, key_bias=np.tile(bias, (BH, 1)), causal=True)
    d2 = oracle.attention(Q, K, V, 2, 4, 0.125, mask=np.tile(bias, (Lq, 1)) + oracle.causal_mask(Lq, Lk))
    assert np.array_equal(c, d2)


def test_planted_mistakes_are_caught():
    """The pins above tell the reading from its plausible neighbours: a strict diagonal (j < i), a top-left aligned
    triangle for Lq != Lk, and a mask applied after the selection."""
    r = _rng(28)
    Lq, Lk, d = 8, 12, 8
    Q, K, V = (a[0] for a in _int_qkv(r, 1, Lq, Lk, d))
    right = oracle.attention(Q, K, V, 2, 4, 0.125, causal=True)
    off = Lk - Lq
    i, j = np.arange(Lq)[:, None], np.arange(Lk)[None, :]
    strict = np.where(j < i + off, 0.0, -np.inf).astype(np.float32)
    top_left = np.where(j <= i, 0.0, -np.inf).astype(np.float32)
    for wrong_mask in (strict, top_left):
        wrong = oracle.attention(Q, K, V, 2, 4, 0.125, mask=wrong_mask)
        assert np.max(np.abs(wrong - right)) > 1e-3
    # mask applied after the selection: hidden keys may win their run and then weigh 0
    cm = oracle.causal_mask(Lq, Lk)
    S = oracle.scores(Q, K, 0.125)
    _, vals, kidx = oracle.prune(S, 2, 4)
    late = vals + np.take_along_axis(cm, kidx.astype(np.int64), axis=1)
    wrong = oracle.spmm(oracle.softmax_kept(late), kidx, V)
    ref, _ = _brute_force(Q, K, V, cm, 2, 4, 0.125)
    assert np.max(np.abs(right - ref)) < 1e-5 < 1e-3 < np.max(np.abs(wrong - ref))
