"""Lengths that are not tile multiples, through dfss_attention_ragged / dense_attention_fused_ragged
(needs an MI355X).  The oracle takes any Lq and any Lk that is a multiple of M, so it is run on the
unpadded arrays directly; the bar is that of the whole path elsewhere (max-abs 2e-2 on O).  The arrays
handed to the library are exactly as large as the shape says, and O sits in front of a guard region that
must stay untouched.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2203_00091_amd as dfss
from paper_2203_00091_amd import DFSS_BF16, DFSS_F32_BF16X3, Shape, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
GUARD = 4096   # elements behind O that no call may write


def _dev(t):
    return t.to(DEV).contiguous()


def _np(t):
    return t.detach().to("cpu", torch.float32).numpy()


def _inputs(BH, Lq, Lk, d, dtype, seed):
    tdt = torch.bfloat16 if dtype == DFSS_BF16 else torch.float32
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=seed, dtype=tdt)
    return Q, K, V, tuple(synth.to_numpy_f32(t) for t in (Q, K, V))


def _guarded_out(s):
    n = s.BH * s.Lq * s.d
    buf = torch.full((n + GUARD,), 777.0, dtype=s.torch_dtype, device=DEV)
    return buf, buf[:n].view(s.BH, s.Lq, s.d)


def _run(fn, Q, K, V, bias, s, scale):
    buf, O = _guarded_out(s)
    fn(_dev(Q), _dev(K), _dev(V), None if bias is None else _dev(bias), s, scale, O=O)
    torch.cuda.synchronize()
    assert bool((buf[O.numel():] == 777.0).all()), "wrote behind O"
    out = _np(O)
    assert np.isfinite(out).all()
    return out


def _max_err(O, ref, Qn, Kn, scale, dtype, bias=None, H=1, tie=1e-4):
    """Largest |O - ref|.  For float data (1:2) rows that hold a pair of scores closer than `tie` are set
    aside: the split products differ from the oracle's fp32 products by up to ~1e-5, so there the other key
    of the pair may rightly be kept, which moves a short row (few keys, large weights) by far more than
    rounding does.  (Long rows need no such care: no single weight is large enough.)"""
    if dtype == DFSS_BF16 or tie == 0:
        return np.abs(O - ref).max()
    worst, rows, kept = 0.0, 0, 0
    for h in range(O.shape[0]):
        S = oracle.scores(Qn[h], Kn[h], scale)
        if bias is not None:
            S = oracle.add_key_bias(S, bias[h // H])
        with np.errstate(invalid="ignore"):
            gap = np.abs(S[:, 0::2] - S[:, 1::2])          # nan where both keys are masked
        safe = ~(gap < tie).any(-1)
        rows, kept = rows + safe.size, kept + int(safe.sum())
        if safe.any():
            worst = max(worst, float(np.abs(O[h] - ref[h])[safe].max()))
    assert kept >= 0.95 * rows
    return worst


CASES = [
    # B, H, Lq, Lk, d
    (2, 2, 100, 100, 64),      # one partial query tile per head, keys end inside the second block
    (1, 3, 1, 4, 64),          # the smallest: one query, one run of keys
    (1, 2, 333, 500, 128),     # d = 128; several tiles and a ragged tail on both sides
    (2, 1, 64, 36, 64),        # a single, partial key block
    (1, 2, 130, 192, 64),      # keys a multiple of 64 (not of 128), queries ragged
    (1, 2, 128, 132, 64),      # queries a tile multiple, one run of keys in the last block
    (4, 12, 2001, 100, 64),    # enough query tiles for the 128-query workgroups of long inputs
    (4, 12, 1990, 68, 128),    # ... and at d = 128
]


@pytest.mark.parametrize("B,H,Lq,Lk,d", CASES)
@pytest.mark.parametrize("dtype,N,M", [(DFSS_BF16, 2, 4), (DFSS_BF16, 1, 2), (DFSS_F32_BF16X3, 1, 2)])
def test_ragged_attention_against_oracle(B, H, Lq, Lk, d, dtype, N, M):
    Q, K, V, (Qn, Kn, Vn) = _inputs(B * H, Lq, Lk, d, dtype, 8100 + Lq + Lk + d)
    s = Shape(B, H, Lq, Lk, d, N, M, dtype)
    scale = 1.0 / math.sqrt(d)
    O = _run(dfss.dfss_attention_ragged, Q, K, V, None, s, scale)
    Od = _run(dfss.dense_attention_fused_ragged, Q, K, V, None, s, scale)
    ref = oracle.attention(Qn, Kn, Vn, N, M, scale)
    ref_dense = oracle.attention(Qn, Kn, Vn, 1, 1, scale)
    assert O.shape == ref.shape
    assert _max_err(O, ref, Qn, Kn, scale, dtype) <= 2e-2
    assert np.abs(Od - ref_dense).max() <= 2e-2


@pytest.mark.parametrize("dtype,N,M", [(DFSS_BF16, 2, 4), (DFSS_F32_BF16X3, 1, 2)])
@pytest.mark.parametrize("scale", [0.125, 0.11])     # bias as initial accumulator value / added after the scaling
@pytest.mark.parametrize("Lq,Lk", [(150, 332), (70, 1284)])   # 6 and 21 key blocks: both ways of scanning the bias row
def test_ragged_attention_with_key_bias(dtype, N, M, scale, Lq, Lk):
    """A padding mask (lengths not aligned to anything) plus a finite bias on unpadded arrays whose rows
    of key_bias are Lk floats long."""
    B, H, d = 3, 2, 64
    Q, K, V, (Qn, Kn, Vn) = _inputs(B * H, Lq, Lk, d, dtype, 8200)
    lengths = synth.padding_lengths(B, Lk, 8201)
    bias = synth.key_padding_bias(lengths, Lk)
    g = torch.Generator().manual_seed(8202)
    bias[1] += torch.randn(Lk, generator=g)          # finite terms next to the -inf of the padding
    s = Shape(B, H, Lq, Lk, d, N, M, dtype)
    O = _run(dfss.dfss_attention_ragged, Q, K, V, bias, s, scale)
    Od = _run(dfss.dense_attention_fused_ragged, Q, K, V, bias, s, scale)
    ref = oracle.attention(Qn, Kn, Vn, N, M, scale, key_bias=bias.numpy(), heads_per_batch=H)
    ref_dense = oracle.attention(Qn, Kn, Vn, 1, 1, scale, key_bias=bias.numpy(), heads_per_batch=H)
    assert _max_err(O, ref, Qn, Kn, scale, dtype, bias.numpy(), H) <= 2e-2
    assert np.abs(Od - ref_dense).max() <= 2e-2


@pytest.mark.parametrize("dtype,N,M", [(DFSS_BF16, 2, 4), (DFSS_F32_BF16X3, 1, 2)])
def test_ragged_equals_padded_and_masked(dtype, N, M):
    """The definition: the call on unpadded arrays gives what the tile-multiple call gives on arrays padded
    with arbitrary (finite) rows whose keys are masked -- bit for bit, since the kept scores are the same."""
    B, H, Lq, Lk, d = 2, 2, 100, 200, 64
    Lqp, Lkp = 128, 256
    Q, K, V, _ = _inputs(B * H, Lq, Lk, d, dtype, 8300)
    Qp, Kp, Vp, _ = _inputs(B * H, Lqp, Lkp, d, dtype, 8301)
    Qp[:, :Lq], Kp[:, :Lk], Vp[:, :Lk] = Q, K, V
    bias = torch.zeros((B, Lkp), dtype=torch.float32)
    bias[:, Lk:] = float("-inf")
    s, sp = Shape(B, H, Lq, Lk, d, N, M, dtype), Shape(B, H, Lqp, Lkp, d, N, M, dtype)
    O = _run(dfss.dfss_attention_ragged, Q, K, V, None, s, 0.125)
    Op = dfss.dfss_attention_bias(_dev(Qp), _dev(Kp), _dev(Vp), _dev(bias), sp, 0.125)
    torch.cuda.synchronize()
    assert np.array_equal(O, _np(Op)[:, :Lq])


@pytest.mark.parametrize("dtype,N,M", [(DFSS_BF16, 2, 4), (DFSS_F32_BF16X3, 1, 2)])
def test_ragged_call_on_tile_multiples_equals_the_plain_call(dtype, N, M):
    B, H, L, d = 2, 2, 256, 64
    Q, K, V, _ = _inputs(B * H, L, L, d, dtype, 8400)
    s = Shape(B, H, L, L, d, N, M, dtype)
    O = _run(dfss.dfss_attention_ragged, Q, K, V, None, s, 0.125)
    O1 = dfss.dfss_attention(_dev(Q), _dev(K), _dev(V), s, 0.125)
    torch.cuda.synchronize()
    assert np.array_equal(O, _np(O1))


@pytest.mark.parametrize("dtype,N,M", [(DFSS_BF16, 2, 4), (DFSS_F32_BF16X3, 1, 2)])
def test_ragged_length_4000(dtype, N, M):
    """The sequence length of the paper's retrieval task (Sec. 5.1): 4000 = 62.5 blocks of 64 keys.
    Sampled query rows against the oracle (every key of those rows)."""
    B, H, L, d = 1, 2, 4000, 64
    Q, K, V, (Qn, Kn, Vn) = _inputs(B * H, L, L, d, dtype, 8500)
    s = Shape(B, H, L, L, d, N, M, dtype)
    O = _run(dfss.dfss_attention_ragged, Q, K, V, None, s, 0.125)
    rows = np.r_[0:8, 1990:2010, 3960:4000]      # first rows, middle, the ragged last tile
    for h in range(B * H):
        ref = oracle.attention(Qn[h][rows], Kn[h], Vn[h], N, M, 0.125)
        assert _max_err(O[h][rows][None], ref[None], Qn[h][rows][None], Kn[h][None], 0.125, dtype, tie=0) <= 2e-2


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M,scale", [
    (96, 700, 332, 64, 2, 4, 0.125),                              # 576 workgroups of 128 queries: the 32-query kernel
    (128, 417, 1284, 64, 1, 2, float(np.float32(1.0 / 3.0))),     # a last tile of 33 queries, a last block of 4 keys
    (64, 1000, 260, 128, 2, 4, 0.125),                            # d = 128
    (24, 4000, 4000, 64, 2, 4, 0.125),                            # the retrieval length at the bench's head count
])
def test_ragged_lengths_on_grids_that_fill_the_chip(BH, Lq, Lk, d, N, M, scale):
    """Calls without a mask whose 128-query workgroups fill the chip take the 32-queries-per-wave kernel.  Sampled
    heads and query rows against the oracle (every key of those rows); O in front of a guard region."""
    Q, K, V, (Qn, Kn, Vn) = _inputs(BH, Lq, Lk, d, DFSS_BF16, 8800 + Lq)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    O = _run(dfss.dfss_attention_ragged, Q, K, V, None, s, scale)
    rows = np.unique(np.r_[0:6, Lq // 2:Lq // 2 + 6, max(Lq - 40, 0):Lq])
    for h in (0, BH // 2, BH - 1):
        ref = oracle.attention(Qn[h][rows], Kn[h], Vn[h], N, M, scale)
        assert np.abs(O[h][rows] - ref).max() <= 2e-2, h
    # every head and row: against the 16-queries-per-wave kernel (a zero key bias selects it)
    O16 = _run(dfss.dfss_attention_ragged, Q, K, V, torch.zeros((1, Lk)), s, scale)
    assert np.abs(O - O16).max() <= 2e-2


@pytest.mark.parametrize("dtype,N,M", [(DFSS_BF16, 2, 4), (DFSS_BF16, 1, 2), (DFSS_F32_BF16X3, 1, 2)])
def test_ragged_random_shapes(dtype, N, M):
    """Seeded random lengths (any Lq, Lk a multiple of 4), with and without a padding mask."""
    rng = np.random.default_rng(8700 + N)
    for case in range(8):
        B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        Lq, Lk = int(rng.integers(1, 300)), 4 * int(rng.integers(1, 200))
        d = 64 if case % 2 == 0 else 128
        Q, K, V, (Qn, Kn, Vn) = _inputs(B * H, Lq, Lk, d, dtype, 8710 + case)
        bias = None
        if case % 3 == 0:
            bias = synth.key_padding_bias(synth.padding_lengths(B, Lk, 8750 + case), Lk)
        s = Shape(B, H, Lq, Lk, d, N, M, dtype)
        scale = 1.0 / math.sqrt(d)
        O = _run(dfss.dfss_attention_ragged, Q, K, V, bias, s, scale)
        kb = None if bias is None else bias.numpy()
        ref = oracle.attention(Qn, Kn, Vn, N, M, scale, key_bias=kb, heads_per_batch=H)
        assert _max_err(O, ref, Qn, Kn, scale, dtype, kb, H) <= 2e-2, (case, B, H, Lq, Lk, d)


def test_ragged_rejects_what_it_cannot_run():
    Q, K, V, _ = _inputs(1, 64, 64, 64, DFSS_BF16, 8600)
    with pytest.raises(dfss.DfssError):      # Lk not a multiple of 4
        s = Shape(1, 1, 64, 62, 64, 2, 4)
        dfss.dfss_attention_ragged(_dev(Q), _dev(K[:, :62]), _dev(V[:, :62]), None, s, 0.125)
    with pytest.raises(dfss.DfssError):      # exact fp32 products have no one-kernel path
        s = Shape(1, 1, 64, 64, 64, 1, 2, dfss.DFSS_F32)
        dfss.dfss_attention_ragged(_dev(Q.float()), _dev(K.float()), _dev(V.float()), None, s, 0.125)
    torch.cuda.synchronize()


# ----------------------------------------------------------------------------------
# the stage calls on unpadded lengths (2-byte dtype): the compressed arrays take the layout of the
# padded lengths (Lq to a multiple of 64, Lk to one of 128); Q, K, V, key_bias and O are the caller's
# ----------------------------------------------------------------------------------
def _meta_canonical(meta, s):
    return dfss.dfss_meta_to_canonical(meta, s).cpu().numpy().view(np.uint16).reshape(s.BH, s.LqP, s.meta_words)


@pytest.mark.parametrize("B,H,Lq,Lk,d,N,M,scale", [
    (1, 2, 100, 132, 64, 2, 4, 0.125),       # one partial row tile, a partial second key block
    (2, 2, 250, 1000, 64, 1, 2, 0.11),       # Lq_P % 128 == 0, scale applied to the scores
    (1, 3, 200, 516, 128, 2, 4, 0.0884),     # d = 128; Lq_P = 256 with rows 200..255 absent; 4 real keys in the last block
    (1, 1, 4000, 4000, 64, 2, 4, 0.125),     # the long-sequence length of Sec. 5.1
    (1, 2, 70, 128, 64, 2, 4, 0.125),        # Lk a tile multiple, Lq not: the upper half of the workgroup stores nothing
])
def test_stage_calls_on_unpadded_lengths(B, H, Lq, Lk, d, N, M, scale):
    s = Shape(B, H, Lq, Lk, d, N, M)
    assert (s.LqP, s.LkP) != (Lq, Lk)
    bias = torch.zeros((B, Lk), dtype=torch.float32)
    bias[0, Lk // 2:Lk // 2 + 37] = float("-inf")
    bias[-1, 5:Lk:7] = -0.75
    # stage 1 on integer inputs: kept values and positions of the real rows bit for bit; absent keys count as -inf
    if Lq <= 250:
        Q, K, _ = synth.integer_qkv(B * H, Lq, Lk, d, seed=8700 + Lq + Lk)
        Qn, Kn = synth.to_numpy_f32(Q), synth.to_numpy_f32(K)
        for kb in (None, bias):
            vals, meta = dfss.dfss_sddmm_prune_bias(_dev(Q), _dev(K), None if kb is None else _dev(kb), s, scale)
            torch.cuda.synchronize()
            assert tuple(vals.shape) == (s.BH, s.LqP, s.Lc)
            v, mc = vals.float().cpu().numpy(), _meta_canonical(meta, s)
            for h in range(s.BH):
                S = oracle.scores(Qn[h], Kn[h], scale)
                if kb is not None:
                    S = oracle.add_key_bias(S, kb[h // H].numpy())
                Sp = np.full((Lq, s.LkP), -np.inf, dtype=np.float32)
                Sp[:, :Lk] = S
                _, vref, kidx = oracle.prune(Sp, N, M)
                assert np.array_equal(mc[h, :Lq], oracle.encode_meta(kidx, s.LkP)), f"metadata differs in head {h}"
                assert np.array_equal(v[h, :Lq], oracle.round_bf16(vref)), f"kept scores differ in head {h}"
    # the whole path on Gaussian inputs: the three stage calls, the staged call, the three-kernel baseline
    Q, K, V = synth.gaussian_qkv(B * H, Lq, Lk, d, 1.0, seed=8701 + Lq + Lk)
    Qd, Kd, Vd = _dev(Q), _dev(K), _dev(V)
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    gscale = 1.0 / math.sqrt(d) if scale != 0.125 else 0.125
    for kb in (None, bias):
        kw = {} if kb is None else dict(key_bias=kb.numpy(), heads_per_batch=H)
        kbd = None if kb is None else _dev(kb)
        ref = oracle.attention(Qn, Kn, Vn, N, M, gscale, **kw)
        refd = oracle.attention(Qn, Kn, Vn, 1, 1, gscale, **kw)
        vals, meta = dfss.dfss_sddmm_prune_bias(Qd, Kd, kbd, s, gscale)
        dfss.dfss_sparse_softmax(vals, s)
        buf, O3 = _guarded_out(s)
        dfss.dfss_spmm(vals, meta, Vd, s, O=O3)
        bufs, Os = _guarded_out(s)
        dfss.dfss_attention_staged_bias(Qd, Kd, Vd, kbd, s, gscale, O=Os)
        bufd, Od = _guarded_out(s)
        dfss.dense_attention_bias(Qd, Kd, Vd, kbd, s, gscale, O=Od)
        Of = dfss.dfss_attention_ragged(Qd, Kd, Vd, kbd, s, gscale)
        torch.cuda.synchronize()
        for name, b_, o_, r_ in (("three stages", buf, O3, ref), ("staged", bufs, Os, ref), ("dense", bufd, Od, refd)):
            assert bool((b_[o_.numel():] == 777.0).all()), f"{name}: wrote behind O"
            got = _np(o_)
            assert np.isfinite(got).all(), name
            assert np.abs(got - r_).max() <= 2e-2, name
        assert np.abs(_np(Os) - _np(Of)).max() <= 2e-2     # the one-kernel call on the same lengths


def test_unpadded_stage_calls_refuse_what_they_cannot_run():
    Q, K, V, _ = _inputs(1, 100, 132, 64, DFSS_BF16, 8800)
    s = Shape(1, 1, 100, 132, 64, 2, 4)
    with pytest.raises(dfss.DfssError):      # the causal mask is defined on tile multiples only
        dfss.dfss_sddmm_prune_causal(_dev(Q), _dev(K), None, s, 0.125)
    with pytest.raises(dfss.DfssError):      # the one-kernel call for these lengths is dfss_attention_ragged
        dfss.dfss_attention(_dev(Q), _dev(K), _dev(V), s, 0.125)
    sf = Shape(1, 1, 100, 132, 64, 1, 2, DFSS_F32_BF16X3)
    assert dfss.dfss_vals_bytes(sf) == 0     # 4-byte dtypes: tile multiples only
    torch.cuda.synchronize()
