"""Pins of the CPU oracle against things other than itself.

Each test names the passage of arXiv 2203.00091 it pins and the kind of pin:
printed value, closed form, invariant, library routine, or brute force.
None of them needs a GPU.
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from conftest import read_golden


def _rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------
# scores (Eq. 1, argument of the softmax)
# --------------------------------------------------------------------------
def test_scores_exact_on_integers():
    """Integer Q, K: every product and partial sum is exact in fp32, so the
    oracle must equal integer arithmetic bit for bit.  Lq != Lk catches a
    transposed operand, the distinct shapes a swapped index."""
    r = _rng(1)
    Q = r.integers(-4, 5, size=(24, 64))
    K = r.integers(-4, 5, size=(40, 64))
    S = oracle.scores(Q, K, 0.125)
    ref = (Q.astype(np.int64) @ K.astype(np.int64).T).astype(np.float64) * 0.125
    assert S.shape == (24, 40)
    assert np.array_equal(S.astype(np.float64), ref)


def test_scores_close_to_float64_on_gaussians():
    r = _rng(2)
    Q = r.standard_normal((32, 64)).astype(np.float32)
    K = r.standard_normal((48, 64)).astype(np.float32)
    S = oracle.scores(Q, K, 1 / 8)
    ref = (Q.astype(np.float64) @ K.astype(np.float64).T) / 8
    assert np.max(np.abs(S - ref)) < 1e-5


def test_scale_is_applied_once_after_the_sum():
    r = _rng(3)
    Q = r.integers(-4, 5, size=(8, 16)).astype(np.float32)
    K = r.integers(-4, 5, size=(8, 16)).astype(np.float32)
    S1 = oracle.scores(Q, K, 1.0)
    S3 = oracle.scores(Q, K, 0.3)
    assert np.array_equal(S3, (S1 * np.float32(0.3)).astype(np.float32))


# --------------------------------------------------------------------------
# N:M selection (Sec. 2.3, App. A.1.1)
# --------------------------------------------------------------------------
def _brute_force_keep(group, N):
    """All C(M,N) subsets: maximal exact sum; among equal sums the
    lexicographically smallest index tuple (= lower index wins a tie)."""
    best = None
    for comb in itertools.combinations(range(len(group)), N):
        s = sum(Fraction(float(group[t])) for t in comb)
        if best is None or s > best[0]:
            best = (s, comb)
    return best[1]


@pytest.mark.parametrize("N,M", [(2, 4), (1, 2), (1, 4), (3, 4), (2, 8), (4, 4)])
def test_prune_matches_brute_force_with_ties(N, M):
    r = _rng(10 + N * 10 + M)
    # few distinct values => many ties, including all-equal groups and signed zeros
    S = r.integers(-2, 3, size=(12, 8 * M)).astype(np.float32)
    S[0, :M] = 0.0
    S[0, 1] = -0.0  # -0 == +0 is a tie
    mask, vals, kidx = oracle.prune(S, N, M)
    for i in range(S.shape[0]):
        for g in range(S.shape[1] // M):
            grp = S[i, g * M:(g + 1) * M]
            keep = _brute_force_keep(grp, N)
            got = tuple(np.nonzero(mask[i, g * M:(g + 1) * M])[0])
            assert got == keep, (i, g, grp, got, keep)
            assert tuple(kidx[i, g * N:(g + 1) * N] - g * M) == keep
            assert np.array_equal(vals[i, g * N:(g + 1) * N], grp[list(keep)])


@pytest.mark.parametrize("N,M", [(2, 4), (1, 2)])
def test_prune_invariants_on_gaussians(N, M):
    r = _rng(20 + M)
    S = r.standard_normal((64, 256)).astype(np.float32)
    mask, vals, kidx = oracle.prune(S, N, M)
    m = mask.reshape(64, -1, M).astype(bool)
    g = S.reshape(64, -1, M)
    assert np.all(m.sum(-1) == N)  # exactly N survivors per group
    kept_min = np.where(m, g, np.inf).min(-1)
    drop_max = np.where(~m, g, -np.inf).max(-1)
    assert np.all(kept_min >= drop_max)  # survivors dominate the dropped
    # kept values are the dense scores at their positions, in key order
    assert np.array_equal(vals, np.take_along_axis(S, kidx, axis=1))
    assert np.all(np.diff(kidx, axis=1) > 0)
    assert np.array_equal(np.sort(np.nonzero(mask[3])[0]), kidx[3])


def test_prune_is_signed_not_absolute():
    """Softmax is monotone (Sec. 3.1), so the larger *signed* score survives."""
    S = np.array([[-9.0, 1.0, -8.0, 0.5]], np.float32)
    mask, vals, _ = oracle.prune(S, 2, 4)
    assert mask.tolist() == [[0, 1, 0, 1]]
    mask, _, _ = oracle.prune(S, 1, 2)
    assert mask.tolist() == [[0, 1, 0, 1]]


def test_two_of_four_keeps_at_least_the_mass_of_one_of_two():
    """Deterministic form of Q_{2:4} >= Q_{1:2} (Prop. 4.2): per run of four keys."""
    r = _rng(30)
    S = r.standard_normal((32, 128)).astype(np.float32)
    m24, _, _ = oracle.prune(S, 2, 4)
    m12, _, _ = oracle.prune(S, 1, 2)
    g = S.reshape(32, -1, 4).astype(np.float64)
    s24 = (g * m24.reshape(32, -1, 4)).sum(-1)
    s12 = (g * m12.reshape(32, -1, 4)).sum(-1)
    assert np.all(s24 >= s12)


def test_pattern_frequencies_are_uniform_on_iid_scores():
    """Exchangeable scores: each of the 6 (2:4) / 2 (1:2) patterns is equally likely."""
    r = _rng(31)
    S = r.standard_normal((256, 1024)).astype(np.float32)
    m24, _, _ = oracle.prune(S, 2, 4)
    codes = (m24.reshape(-1, 4) * np.array([1, 2, 4, 8])).sum(-1)
    counts = np.array([np.sum(codes == c) for c in (3, 5, 9, 6, 10, 12)], float)
    assert counts.sum() == codes.size
    expect = codes.size / 6
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 25.0  # 5 dof; P(chi2 > 25) ~ 1e-4
    m12, _, _ = oracle.prune(S, 1, 2)
    first = m12.reshape(-1, 2)[:, 0].mean()
    assert abs(first - 0.5) < 0.01


# --------------------------------------------------------------------------
# metadata (Sec. 2.3, App. A.1.1, A.1.2)
# --------------------------------------------------------------------------
def test_meta_codes_printed_in_the_paper():
    gold = read_golden("meta_codes.txt")
    # one run of four slots per case, padded to a full 16-key word with the same pattern
    first = np.array([[0, 1] * 1 + [4, 5, 8, 9, 12, 13]], np.int32)
    second = np.array([[2, 3, 6, 7, 10, 11, 14, 15]], np.int32)
    w_first = int(oracle.encode_meta(first, 16)[0, 0])
    w_second = int(oracle.encode_meta(second, 16)[0, 0])
    c4 = int(gold["keep_slots_0_1"], 16)
    ce = int(gold["keep_slots_2_3"], 16)
    assert w_first == c4 * 0x1111
    assert w_second == ce * 0x1111


def test_meta_code_k_sits_at_bits_4k():
    """App. A.1.2: the k-th of four consecutive codes occupies bits [4k, 4k+3]."""
    gold = read_golden("meta_codes.txt")
    c4 = int(gold["keep_slots_0_1"], 16)
    ce = int(gold["keep_slots_2_3"], 16)
    for k in range(4):
        kidx = []
        for run in range(4):
            kidx += [4 * run + 2, 4 * run + 3] if run == k else [4 * run, 4 * run + 1]
        w = int(oracle.encode_meta(np.array([kidx], np.int32), 16)[0, 0])
        assert (w >> (4 * k)) & 0xF == ce
        for other in range(4):
            if other != k:
                assert (w >> (4 * other)) & 0xF == c4


def test_meta_all_six_codes_are_two_bit_positions():
    for lo, hi in itertools.combinations(range(4), 2):
        kidx = np.array([[lo, hi, 4, 5, 8, 9, 12, 13]], np.int32)
        w = int(oracle.encode_meta(kidx, 16)[0, 0])
        assert w & 0xF == (lo | (hi << 2))


def test_meta_size_and_footprint():
    gold = read_golden("meta_codes.txt")
    Lq, Lk = 64, 256
    r = _rng(40)
    S = r.standard_normal((Lq, Lk)).astype(np.float32)
    _, vals, kidx = oracle.prune(S, 2, 4)
    meta = oracle.encode_meta(kidx, Lk)
    dense_bits_2B = Lq * Lk * 16
    assert meta.nbytes * 8 / dense_bits_2B == float(gold["meta_fraction_of_dense_bits"])
    # Sec. 3.4 counts 32-bit entries: n^2/2 values + n^2/16 metadata words of 32 bit
    frac = (vals.size * 32 + (Lq * Lk // 16) * 32) / (Lq * Lk * 32)
    assert frac == float(gold["footprint_fraction"])


@pytest.mark.parametrize("N,M", [(2, 4), (1, 2)])
def test_meta_round_trip(N, M):
    r = _rng(41 + M)
    S = r.standard_normal((16, 128)).astype(np.float32)
    mask, vals, kidx = oracle.prune(S, N, M)
    meta = oracle.encode_meta(kidx, 128)
    back = oracle.decode_meta(meta, 128)
    assert np.array_equal(back, kidx)
    dense = np.zeros_like(S)
    np.put_along_axis(dense, back, vals, axis=1)
    assert np.array_equal(dense, S * mask)
    if (N, M) == (1, 2):
        # 1:2 on 2-byte data: one position from {0,1}, one from {2,3}
        codes = {int((w >> (4 * k)) & 0xF) for w in meta.reshape(-1) for k in range(4)}
        assert codes <= {0x8, 0xC, 0x9, 0xD}


# --------------------------------------------------------------------------
# softmax over kept entries (Sec. 3.1, App. A.1.3)
# --------------------------------------------------------------------------
def test_softmax_matches_library_and_invariants():
    r = _rng(50)
    x = (r.standard_normal((32, 96)) * 3).astype(np.float32)
    P = oracle.softmax_kept(x)
    ref = scipy.special.softmax(x.astype(np.float64), axis=1)
    assert np.max(np.abs(P - ref)) < 1e-7
    assert np.max(np.abs(P.sum(1, dtype=np.float64) - 1)) < 1e-6
    assert np.max(np.abs(oracle.softmax_kept(x + np.float32(5.0)) - P)) < 1e-6
    # large offsets must not overflow (max-subtracted form)
    big = oracle.softmax_kept(x + np.float32(300.0))
    assert np.all(np.isfinite(big)) and np.max(np.abs(big - P)) < 1e-4
    # a spread wider than the exponent range only survives if the *maximum* is subtracted
    wide = oracle.softmax_kept(np.array([[0.0, -1000.0, 1000.0, 999.0]], np.float32))
    e = math.exp(-1.0)
    assert np.allclose(wide[0], [0.0, 0.0, 1 / (1 + e), e / (1 + e)], atol=1e-7)


# --------------------------------------------------------------------------
# compressed weights times V, and the whole path
# --------------------------------------------------------------------------
def test_spmm_against_dense_scatter():
    r = _rng(60)
    Lq, Lk, d = 16, 64, 8
    S = r.standard_normal((Lq, Lk)).astype(np.float32)
    V = r.standard_normal((Lk, d)).astype(np.float32)
    mask, vals, kidx = oracle.prune(S, 2, 4)
    P = oracle.softmax_kept(vals)
    O = oracle.spmm(P, kidx, V)
    dense = np.zeros((Lq, Lk))
    np.put_along_axis(dense, kidx, P.astype(np.float64), axis=1)
    assert np.max(np.abs(O - dense @ V.astype(np.float64))) < 1e-6


@pytest.mark.parametrize("M", [1, 2, 4])
def test_n_equals_m_is_full_attention(M):
    """N = M keeps everything: the path must equal Eq. 1 computed by library routines."""
    r = _rng(70 + M)
    BH, Lq, Lk, d = 2, 24, 40, 16
    Q = r.standard_normal((BH, Lq, d)).astype(np.float32)
    K = r.standard_normal((BH, Lk, d)).astype(np.float32)
    V = r.standard_normal((BH, Lk, d)).astype(np.float32)
    O = oracle.attention(Q, K, V, M, M, 0.25)
    tq, tk, tv = (torch.from_numpy(a).double() for a in (Q, K, V))
    ref = torch.softmax(tq @ tk.transpose(1, 2) * 0.25, dim=-1) @ tv
    assert np.max(np.abs(O - ref.numpy())) < 2e-6


@pytest.mark.parametrize("N,M", [(2, 4), (1, 2)])
def test_path_equals_masked_dense_softmax_by_library(N, M):
    """DFSS output == dense softmax with dropped scores at -inf, built from numpy/scipy only
    (mask from an argsort-based selection that does not call the oracle)."""
    r = _rng(80 + M)
    Lq, Lk, d = 32, 64, 16
    Q = r.standard_normal((Lq, d)).astype(np.float32)
    K = r.standard_normal((Lk, d)).astype(np.float32)
    V = r.standard_normal((Lk, d)).astype(np.float32)
    S = (Q.astype(np.float64) @ K.astype(np.float64).T) * 0.25
    g = S.reshape(Lq, -1, M)
    order = np.argsort(-g, axis=-1, kind="stable")  # descending, lower index first among equals
    keep = np.zeros_like(g, dtype=bool)
    np.put_along_axis(keep, order[..., :N], True, axis=-1)
    masked = np.where(keep.reshape(Lq, Lk), S, -np.inf)
    ref = scipy.special.softmax(masked, axis=1) @ V.astype(np.float64)
    O = oracle.attention(Q, K, V, N, M, 0.25)
    assert np.max(np.abs(O - ref)) < 5e-6


def test_separable_groups_reduce_to_full_attention():
    """If in every group N scores exceed the rest by >= 40, the dropped weights are
    < e^-40 and DFSS equals full attention to fp32 precision."""
    r = _rng(90)
    Lq, Lk, d = 16, 64, 32
    Q = np.zeros((Lq, d), np.float32)
    Q[:, 0] = 1.0
    Q[:, 1:] = r.standard_normal((Lq, d - 1)).astype(np.float32) * 0.01
    K = r.standard_normal((Lk, d)).astype(np.float32) * 0.01
    K[:, 0] = 0.0
    hot = np.concatenate([g * 4 + r.permutation(4)[:2] for g in range(Lk // 4)])
    K[hot, 0] = 50.0
    V = r.standard_normal((Lk, d)).astype(np.float32)
    O = oracle.attention(Q, K, V, 2, 4, 1.0)
    full = oracle.attention(Q, K, V, 4, 4, 1.0)
    assert np.max(np.abs(O - full)) < 1e-6


def test_permutation_symmetries():
    r = _rng(91)
    Lq, Lk, d = 16, 64, 8
    Q = r.standard_normal((Lq, d)).astype(np.float32)
    K = r.standard_normal((Lk, d)).astype(np.float32)
    V = r.standard_normal((Lk, d)).astype(np.float32)
    O = oracle.attention(Q, K, V, 2, 4, 0.3)
    # moving whole groups of keys (with their values) changes nothing
    gp = r.permutation(Lk // 4)
    kp = (gp[:, None] * 4 + np.arange(4)[None]).reshape(-1)
    O2 = oracle.attention(Q, K[kp], V[kp], 2, 4, 0.3)
    assert np.max(np.abs(O - O2)) < 1e-6
    # permuting queries permutes output rows
    qp = r.permutation(Lq)
    O3 = oracle.attention(Q[qp], K, V, 2, 4, 0.3)
    assert np.array_equal(O3, O[qp])


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 3.14159],
                 np.float32)
    got = oracle.round_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, ref)
    # exact ties: 1 + 2^-8 -> 1 (even), 1 + 3*2^-8 -> 1 + 2^-6 (even)
    assert got[3] == 1.0 and got[4] == np.float32(1.0 + 2 ** -6)
    r = _rng(92)
    y = r.standard_normal(10000).astype(np.float32) * 37
    assert np.array_equal(oracle.round_bf16(y),
                          torch.from_numpy(y).to(torch.bfloat16).to(torch.float32).numpy())


# --------------------------------------------------------------------------
# L^p quality (Def. 4.1) against the closed form of Prop. 4.2
# --------------------------------------------------------------------------
def test_closed_form_values_printed_in_the_paper():
    gold = read_golden("quality_closed_form.txt")
    q7 = (1 + math.erf(7 / 2)) / 2
    assert abs(q7 - float(gold["q12_at_psigma_7"])) < 5e-8
    q1 = (1 + math.erf(1 / 2)) / 2
    assert q1 >= float(gold["q12_at_psigma_1_lower"]) and q1 < 0.77


@pytest.mark.parametrize("psigma,tol", [(1.0, 0.004), (2.0, 0.02)])
def test_quality_of_one_of_two_matches_closed_form(psigma, tol):
    r = _rng(100)
    sigma = 1.0
    S = (r.standard_normal((128, 8192)) * sigma + 0.3).astype(np.float32)
    m12, _, _ = oracle.prune(S, 1, 2)
    q = oracle.quality_p(S, m12, psigma / sigma)
    closed = (1 + math.erf(psigma / 2)) / 2
    assert abs(q - closed) < tol, (q, closed)
    m24, _, _ = oracle.prune(S, 2, 4)
    q24 = oracle.quality_p(S, m24, psigma / sigma)
    assert q24 >= q  # Prop. 4.2: Q_{2:4} >= Q_{1:2}
    # a fixed mask of density 1/2 has quality 1/2 (Prop. 4.2, Q_fix = s)
    fixed = np.zeros_like(m12)
    fixed[:, ::2] = 1
    assert abs(oracle.quality_p(S, fixed, psigma / sigma) - 0.5) < 2.5 * tol
    # the full mask has quality exactly 1
    assert abs(oracle.quality_p(S, np.ones_like(m12), 1.0) - 1.0) < 1e-12


def test_two_byte_storage_branch_against_torch():
    """store_bf16 = 1 models the method's 2-byte compressed matrix: the kept scores and the weights pass through
    bfloat16 where they are stored (Sec. 2.3: the nonzeros keep the data type of the dense matrix).  Pinned against
    the same chain in torch: its own bfloat16 conversion, topk selection, softmax and matmul (Gaussian inputs: no
    ties, so topk's tie order does not matter)."""
    r = np.random.default_rng(77)
    Lq, Lk, d, N, M = 48, 96, 32, 2, 4
    Q, K, V = (r.standard_normal(s).astype(np.float32) for s in ((Lq, d), (Lk, d), (Lk, d)))
    got = oracle.attention(Q, K, V, N, M, 0.25, store_bf16=True)
    S = torch.from_numpy(oracle.scores(Q, K, 0.25))                    # fp32 scores (pinned elsewhere)
    G = S.view(Lq, Lk // M, M)
    idx = G.topk(N, dim=-1).indices.sort(-1).values                    # kept positions, key order
    vals = G.gather(-1, idx).to(torch.bfloat16).double()               # stored in 2 bytes
    P = torch.softmax(vals.view(Lq, -1), dim=-1).to(torch.bfloat16).double().view(Lq, Lk // M, N)
    W = torch.zeros(Lq, Lk // M, M, dtype=torch.float64).scatter_(-1, idx, P).view(Lq, Lk)
    ref = (W @ torch.from_numpy(V).double()).numpy()
    assert np.max(np.abs(got - ref)) < 1e-5
    # and the storage matters: the unrounded function differs, by no more than the roundings allow
    exact = oracle.attention(Q, K, V, N, M, 0.25, store_bf16=False)
    diff = np.max(np.abs(got - exact))
    assert 1e-5 < diff < 2e-2
