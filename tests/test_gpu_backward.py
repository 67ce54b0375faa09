"""Backward pass on the GPU against the CPU oracle, through the C ABI (needs an MI355X).

The kernels are fed the ORACLE's forward results (weights rounded to bfloat16, metadata converted
to the library's order), so that both sides differentiate through exactly the same selection; the
composition with the GPU forward pass is checked on integer-valued Q, K, where the selection is exact.
Tolerances: operands are bfloat16 (8 significant bits) and sums run in fp32, so results agree to
about 2^-8 of the magnitudes involved; each bound below is stated next to its check.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2203_00091_amd as dfss
from paper_2203_00091_amd import Shape, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(t):
    return t.to(DEV).contiguous()


def _np(t):
    return t.detach().to("cpu", torch.float32).numpy()


def _bf16(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)


def _oracle_forward(Qn, Kn, N, M, scale):
    """Per head: kept indices, bf16-rounded weights, canonical metadata."""
    kidx, P, meta = [], [], []
    for h in range(Qn.shape[0]):
        S = oracle.scores(Qn[h], Kn[h], scale)
        _, vals, ki = oracle.prune(S, N, M)
        P.append(oracle.round_bf16(oracle.softmax_kept(oracle.round_bf16(vals))))
        kidx.append(ki)
        meta.append(oracle.encode_meta(ki, Kn.shape[1]))
    return np.stack(kidx), np.stack(P), np.stack(meta)


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M", [
    (2, 128, 256, 64, 2, 4),
    (3, 192, 128, 64, 1, 2),      # more queries than keys, three query steps
    (2, 64, 384, 128, 2, 4),      # d = 128, one query step
])
def test_transposed_spmm(BH, Lq, Lk, d, N, M):
    Q, K, _ = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=9300 + Lq + Lk)
    g = torch.Generator().manual_seed(9301 + d)
    X = torch.randn(BH, Lq, d, generator=g).to(torch.bfloat16)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    Qn, Kn, Xn = (synth.to_numpy_f32(t) for t in (Q, K, X))
    kidx, P, meta_c = _oracle_forward(Qn, Kn, N, M, 1.0 / math.sqrt(d))
    meta = dfss.dfss_meta_from_canonical(_dev(torch.from_numpy(meta_c.view(np.int16))), s)
    out = dfss.dfss_spmm_t(_dev(_bf16(P)), meta, _dev(X), s)
    torch.cuda.synchronize()
    out = _np(out)
    for h in range(BH):
        Pd = np.zeros((Lq, Lk))
        np.put_along_axis(Pd, kidx[h].astype(np.int64), P[h].astype(np.float64), axis=1)
        ref = Pd.T @ Xn[h].astype(np.float64)
        # bf16 output rounding (2^-9 relative) + fp32 accumulation of <= Lq terms
        assert np.max(np.abs(out[h] - ref)) <= 2.0 ** -8 * np.max(np.abs(ref)) + 1e-4


def _oracle_backward_case(BH, Lq, Lk, d, N, M, seed, scale):
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=seed)
    g = torch.Generator().manual_seed(seed + 1)
    dO = torch.randn(BH, Lq, d, generator=g).to(torch.bfloat16)
    Qn, Kn, Vn, dOn = (synth.to_numpy_f32(t) for t in (Q, K, V, dO))
    kidx, P, meta_c = _oracle_forward(Qn, Kn, N, M, scale)
    O = np.stack([oracle.round_bf16(oracle.spmm(P[h], kidx[h], Vn[h])) for h in range(BH)])
    return (Q, K, V, dO), (Qn, Kn, Vn, dOn), kidx, P, meta_c, O


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M", [
    (2, 128, 256, 64, 2, 4),       # 32 queries per wave in the dS kernel
    (2, 192, 384, 64, 1, 2),       # 16 queries per wave, key range split three ways
    (2, 128, 128, 128, 2, 4),      # d = 128
])
def test_backward_against_oracle_through_the_same_selection(BH, Lq, Lk, d, N, M):
    scale = 1.0 / math.sqrt(d)
    (Q, K, V, dO), (Qn, Kn, Vn, dOn), kidx, P, meta_c, O = _oracle_backward_case(BH, Lq, Lk, d, N, M, 9400 + Lq + d, scale)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    meta = dfss.dfss_meta_from_canonical(_dev(torch.from_numpy(meta_c.view(np.int16))), s)
    dQ, dK, dV = dfss.dfss_attention_backward(_dev(dO), _dev(Q), _dev(K), _dev(V), _dev(_bf16(O)), _dev(_bf16(P)),
                                              meta, s, scale)
    torch.cuda.synchronize()
    dQ, dK, dV = _np(dQ), _np(dK), _np(dV)
    for h in range(BH):
        rQ, rK, rV = oracle.attention_backward(Qn[h], Kn[h], Vn[h], dOn[h], P[h], kidx[h], scale)
        for name, got, ref in (("dQ", dQ[h], rQ), ("dK", dK[h], rK), ("dV", dV[h], rV)):
            # operands (P, dS, O) and results are bfloat16 (2^-9 relative each); observed <= 0.0053 of the largest entry
            tol = 2.0 ** -7 * np.max(np.abs(ref)) + 1e-4
            err = np.max(np.abs(got - ref))
            assert err <= tol, (name, h, err, tol)


def test_forward_stages_then_backward_on_exact_scores():
    """GPU forward (three stage calls, integer Q and K: the selection equals the oracle's exactly)
    followed by the GPU backward, against the oracle end to end."""
    BH, L, d = 2, 256, 64
    Q, K, V = synth.integer_qkv(BH, L, L, d, seed=9500)
    Q, K = (Q.float() * 0.25).to(torch.bfloat16), (K.float() * 0.25).to(torch.bfloat16)   # keeps the softmax soft
    g = torch.Generator().manual_seed(9501)
    dO = torch.randn(BH, L, d, generator=g).to(torch.bfloat16)
    s = Shape(1, BH, L, L, d, 2, 4)
    Qd, Kd, Vd, dOd = _dev(Q), _dev(K), _dev(V), _dev(dO)
    vals, meta = dfss.dfss_sddmm_prune(Qd, Kd, s, 0.125)
    dfss.dfss_sparse_softmax(vals, s)
    O = dfss.dfss_spmm(vals, meta, Vd, s)
    dQ, dK, dV = dfss.dfss_attention_backward(dOd, Qd, Kd, Vd, O, vals, meta, s, 0.125)
    torch.cuda.synchronize()
    Qn, Kn, Vn, dOn = (synth.to_numpy_f32(t) for t in (Q, K, V, dO))
    kidx, P, meta_c = _oracle_forward(Qn, Kn, 2, 4, 0.125)
    canon = dfss.dfss_meta_to_canonical(meta, s)
    torch.cuda.synchronize()
    assert np.array_equal(canon.cpu().numpy().view(np.uint16), meta_c)       # same selection on both sides
    for h in range(BH):
        rQ, rK, rV = oracle.attention_backward(Qn[h], Kn[h], Vn[h], dOn[h], P[h], kidx[h], 0.125)
        for name, got, ref in (("dQ", _np(dQ[h]), rQ), ("dK", _np(dK[h]), rK), ("dV", _np(dV[h]), rV)):
            tol = 2.0 ** -7 * np.max(np.abs(ref)) + 1e-4
            assert np.max(np.abs(got - ref)) <= tol, (name, h)


# ----------------------------------------------------------------------------------
# lengths that are not tile multiples: P, meta and dS' keep the layout of the padded lengths
# ----------------------------------------------------------------------------------
def _padded_forward(Qn, Kn, N, M, scale, s):
    """The oracle's forward results in the padded layout: absent keys count as -inf; the rows past Lq hold finite
    junk (weights 0.25, codes 0x4) that no gradient may depend on."""
    BH, Lq, Lk = Qn.shape[0], Qn.shape[1], Kn.shape[1]
    kidx, P = [], []
    Pp = np.full((BH, s.LqP, s.Lc), 0.25, dtype=np.float32)
    mp = np.full((BH, s.LqP, s.meta_words), 0x4444, dtype=np.uint16)
    for h in range(BH):
        Sp = np.full((Lq, s.LkP), -np.inf, dtype=np.float32)
        Sp[:, :Lk] = oracle.scores(Qn[h], Kn[h], scale)
        _, vals, ki = oracle.prune(Sp, N, M)
        Ph = oracle.round_bf16(oracle.softmax_kept(oracle.round_bf16(vals)))
        Pp[h, :Lq] = Ph
        mp[h, :Lq] = oracle.encode_meta(ki, s.LkP)
        # for the oracle's backward pass: the kept entries that are real keys (the absent ones have weight 0)
        kidx.append(ki)
        P.append(Ph)
    return kidx, P, Pp, mp


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M", [
    (2, 100, 132, 64, 2, 4),       # fused dQ; one partial query tile, a partial second key block
    (2, 250, 516, 64, 1, 2),       # 32 queries per wave in the dS kernel (LqP = 256), 4 real keys in the last block
    (2, 70, 260, 128, 2, 4),       # d = 128: dQ through the forward product kernel
])
def test_backward_on_unpadded_lengths(BH, Lq, Lk, d, N, M):
    scale = 1.0 / math.sqrt(d)
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=9700 + Lq + d)
    g = torch.Generator().manual_seed(9701 + Lq)
    dO = torch.randn(BH, Lq, d, generator=g).to(torch.bfloat16)
    Qn, Kn, Vn, dOn = (synth.to_numpy_f32(t) for t in (Q, K, V, dO))
    s = Shape(1, BH, Lq, Lk, d, N, M)
    assert (s.LqP, s.LkP) != (Lq, Lk)
    kidx, P, Pp, mp = _padded_forward(Qn, Kn, N, M, scale, s)
    # O of the forward pass from the real keys only (weights of absent keys are 0; their indices point past Lk)
    O = []
    for h in range(BH):
        Pd = np.zeros((Lq, s.LkP))
        np.put_along_axis(Pd, kidx[h].astype(np.int64), P[h].astype(np.float64), axis=1)
        O.append(oracle.round_bf16((Pd[:, :Lk] @ Vn[h].astype(np.float64)).astype(np.float32)))
    O = np.stack(O)
    meta = dfss.dfss_meta_from_canonical(_dev(torch.from_numpy(mp.view(np.int16))), s)
    guard = 4096
    bufs = [torch.full((n + guard,), 777.0, dtype=torch.bfloat16, device=DEV) for n in (BH * Lq * d, BH * Lk * d, BH * Lk * d)]
    dQ, dK, dV = (b[:b.numel() - guard].view(BH, L, d) for b, L in zip(bufs, (Lq, Lk, Lk)))
    dfss.dfss_attention_backward(_dev(dO), _dev(Q), _dev(K), _dev(V), _dev(_bf16(O)), _dev(_bf16(Pp)), meta, s, scale,
                                 dQ=dQ, dK=dK, dV=dV)
    X = torch.randn(BH, Lq, d, generator=g).to(torch.bfloat16)
    T = dfss.dfss_spmm_t(_dev(_bf16(Pp)), meta, _dev(X), s)
    torch.cuda.synchronize()
    for b in bufs:
        assert bool((b[b.numel() - guard:] == 777.0).all()), "wrote behind a gradient"
    assert tuple(T.shape) == (BH, Lk, d)
    dQ, dK, dV, T, Xn = _np(dQ), _np(dK), _np(dV), _np(T), synth.to_numpy_f32(X)
    for h in range(BH):
        real = kidx[h] < Lk                          # kept entries that are real keys
        ki = np.where(real, kidx[h], 0)
        Pr = np.where(real, P[h], 0.0).astype(np.float32)
        assert np.all(P[h][~real] == 0.0)
        rQ, rK, rV = oracle.attention_backward(Qn[h], Kn[h], Vn[h], dOn[h], Pr, ki.astype(np.int32), scale)
        for name, got, ref in (("dQ", dQ[h], rQ), ("dK", dK[h], rK), ("dV", dV[h], rV)):
            assert np.isfinite(got).all(), name
            tol = 2.0 ** -7 * np.max(np.abs(ref)) + 1e-4
            err = np.max(np.abs(got - ref))
            assert err <= tol, (name, h, err, tol)
        Pd = np.zeros((Lq, s.LkP))
        np.put_along_axis(Pd, kidx[h].astype(np.int64), P[h].astype(np.float64), axis=1)
        refT = Pd[:, :Lk].T @ Xn[h].astype(np.float64)
        assert np.max(np.abs(T[h] - refT)) <= 2.0 ** -8 * np.max(np.abs(refT)) + 1e-4
