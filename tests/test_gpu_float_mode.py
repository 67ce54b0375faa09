"""Parity of the 4-byte mode (float data, 1:2 selection; Sec. 2.3, App. A.1.1) against the CPU oracle,
through the C ABI (needs an MI355X).

Bars:
  * kept scores and metadata bit-exact on integer-valued Q, K (every product and sum exact in fp32);
  * on Gaussian inputs a pair may be decided differently only if its two scores are closer than the
    rounding error both sides can have; kept scores within that error bound.  The bound is the
    textbook forward error of a length-d dot product accumulated in fp32 in any order,
    d * 2^-24 * sum_k |q_k k_k|, plus one rounding for the multiplication by scale;
  * softmax and SpMM stages, fed with the GPU's own stage-1 output, within fp32 rounding of the oracle;
  * whole path within 2e-2 of the oracle everywhere and within 1e-4 on rows whose selection agrees.

Every test runs for both ways of forming the products: DFSS_F32 (fp32 matrix instruction) and DFSS_F32_BF16X3
(each operand split as x = hi + lo, hi = bf16(x), lo = bf16(x - hi); a*b ~ hi*hi + hi*lo + lo*hi).  For the
second the bound gains the dropped terms: |x - hi - lo| <= 2^-18 |x| and |lo| <= 2^-9 |x| (1 + 2^-9), so
a*b - (three products) = a_lo b_lo + r_a b + a r_b is at most 3.01 * 2^-18 |a b|; three times as many terms
are accumulated.  Integer-valued inputs have lo = 0: the bit-exact bar is unchanged.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2203_00091_amd as dfss
from paper_2203_00091_amd import DFSS_F32, DFSS_F32_BF16X3, Shape, synth

pytestmark = pytest.mark.gpu

DTYPES = pytest.mark.parametrize("dtype", [DFSS_F32, DFSS_F32_BF16X3], ids=["fp32_mfma", "bf16x3"])

DEV = "cuda:0"
U = 2.0 ** -24   # unit roundoff of fp32


def _dev(t):
    return t.to(DEV).contiguous()


def _meta_np(meta, s):
    """Metadata of a stage-1 call in canonical word order, as uint16 [BH, Lq, Lk/8]."""
    canon = dfss.dfss_meta_to_canonical(meta, s)
    torch.cuda.synchronize()
    return canon.cpu().numpy().view(np.uint16).reshape(s.BH, s.Lq, s.meta_words)


def _shape(B, H, Lq, Lk, d, dtype=DFSS_F32):
    return Shape(B, H, Lq, Lk, d, 1, 2, dtype)


def _score_error_bound(Q, K, scale, dtype=DFSS_F32):
    """Per-element bound on |computed - exact| of scale * q.k for fp32 accumulation in any order
    (plus the dropped terms of the bf16 split where the products are formed that way)."""
    d = Q.shape[-1]
    absdot = np.abs(Q).astype(np.float64) @ np.abs(K).astype(np.float64).T
    if dtype == DFSS_F32_BF16X3:
        return (3.01 * 2.0 ** -18 * absdot + 3 * d * U * absdot + U * absdot) * scale
    return (d * U * absdot + U * absdot) * scale


# whole-path and SpMM tolerances: fp32 rounding, resp. the split's dropped terms (3.01 * 2^-18 per product)
TOL_SPMM = {DFSS_F32: 1e-5, DFSS_F32_BF16X3: 3e-5}
TOL_O = {DFSS_F32: 1e-4, DFSS_F32_BF16X3: 5e-4}


@pytest.mark.parametrize("BH,Lq,Lk,d,scale", [
    (1, 256, 256, 64, 0.125),
    (3, 128, 384, 64, 0.125),                                   # several heads, rectangular
    (2, 192, 256, 128, 0.125),                                  # d = 128
    (1, 64, 128, 128, float(np.float32(1 / math.sqrt(128)))),   # smallest legal shape, scale not a power of two
    (1, 64, 8192, 64, 0.125),                                   # longest key sequence
    (64, 1024, 128, 64, 0.125),                                 # enough work for the 32-queries-per-wave tiling
    (64, 1024, 128, 128, 0.125),
])
@DTYPES
def test_stage1_bit_exact_on_integer_inputs(BH, Lq, Lk, d, scale, dtype):
    Q, K, _ = synth.integer_qkv(BH, Lq, Lk, d, seed=6100 + Lq + d, dtype=torch.float32)
    s = _shape(1, BH, Lq, Lk, d, dtype)
    vals, meta = dfss.dfss_sddmm_prune(_dev(Q), _dev(K), s, scale)
    torch.cuda.synchronize()
    vals, meta = vals.cpu().numpy(), _meta_np(meta, s)
    ties = 0
    for h in range(BH):
        S = oracle.scores(Q[h].numpy(), K[h].numpy(), scale)
        _, ovals, kidx = oracle.prune(S, 1, 2)
        assert np.array_equal(meta[h], oracle.encode_meta_f32(kidx, Lk)), f"metadata differs in head {h}"
        assert np.array_equal(vals[h], ovals), f"kept scores differ in head {h}"
        ties += int(np.sum(S[:, 0::2] == S[:, 1::2]))
    assert ties > 0   # the tie rule was exercised


@DTYPES
def test_stage1_all_equal_scores_keep_the_first(dtype):
    Q = torch.zeros(1, 64, 64)
    K = torch.ones(1, 128, 64)
    s = _shape(1, 1, 64, 128, 64, dtype)
    vals, meta = dfss.dfss_sddmm_prune(_dev(Q), _dev(K), s, 0.125)
    torch.cuda.synchronize()
    assert np.all(_meta_np(meta, s) == 0x4444) and np.all(vals.cpu().numpy() == 0)


def test_meta_order_conversions_round_trip():
    """Library order = canonical 32-bit words blocked as [row/16][key block of 64][row%16][4 words]."""
    Q, K, _ = synth.integer_qkv(2, 64, 256, 64, seed=6200, dtype=torch.float32)
    s = _shape(1, 2, 64, 256, 64)
    _, meta = dfss.dfss_sddmm_prune(_dev(Q), _dev(K), s, 0.125)
    canon = dfss.dfss_meta_to_canonical(meta, s)
    back = dfss.dfss_meta_from_canonical(canon, s)
    torch.cuda.synchronize()
    assert torch.equal(back, meta)
    lib = meta.cpu().numpy().view(np.uint32).reshape(2, 64 // 16, 256 // 64, 16, 4)
    can = canon.cpu().numpy().view(np.uint32).reshape(2, 64 // 16, 16, 256 // 64, 4)
    assert np.array_equal(lib.transpose(0, 1, 3, 2, 4), can)


@pytest.mark.parametrize("name", ["tiny_1to2_f32", "bert_base_L512_1to2_f32", "large_head_L2048_d128_1to2_f32"])
@DTYPES
def test_stages_on_gaussian_inputs(name, dtype):
    w = synth.WORKLOADS[name]
    Q, K, V = synth.make(w)
    s = _shape(w.B, w.H, w.L, w.L, w.d, dtype)
    vals, meta = dfss.dfss_sddmm_prune(_dev(Q), _dev(K), s, w.scale)
    torch.cuda.synchronize()
    scores_gpu = vals.cpu().numpy()
    meta_np = _meta_np(meta, s)
    P = dfss.dfss_sparse_softmax(vals.clone(), s)
    O = dfss.dfss_spmm(P, meta, _dev(V), s)
    torch.cuda.synchronize()
    P, O = P.cpu().numpy(), O.cpu().numpy()

    heads = range(w.BH) if w.BH <= 4 else [0, w.BH // 2, w.BH - 1]     # sampled heads at the full sizes
    pairs = differ_total = 0
    for h in heads:
        Qn, Kn, Vn = Q[h].numpy(), K[h].numpy(), V[h].numpy()
        S = oracle.scores(Qn, Kn, w.scale)
        _, ovals, okidx = oracle.prune(S, 1, 2)
        kidx = oracle.decode_meta_f32(meta_np[h], w.L)        # raises on any code other than 0x4 / 0xE
        bound = _score_error_bound(Qn, Kn, w.scale, dtype)
        # stage 1: the score each side kept, and where they chose differently
        err_kept = np.abs(scores_gpu[h] - np.take_along_axis(S, kidx, 1))
        assert np.all(err_kept <= 2 * np.take_along_axis(bound, kidx, 1) + 1e-12)
        differ = kidx != okidx
        gap = np.abs(S[:, 0::2] - S[:, 1::2])
        room = 2 * (bound[:, 0::2] + bound[:, 1::2])
        assert np.all(gap[differ] <= room[differ]), "a pair was decided differently outside the rounding error"
        pairs += differ.size
        differ_total += int(differ.sum())
        # stage 2 and 3 on the GPU's own selection
        Pref = oracle.softmax_kept(scores_gpu[h])
        assert np.abs(P[h] - Pref).max() <= 1e-6
        assert np.abs(P[h].sum(-1) - 1).max() <= 1e-5
        Oref = oracle.spmm(P[h], kidx, Vn)
        assert np.abs(O[h] - Oref).max() <= TOL_SPMM[dtype] * max(1.0, float(np.abs(Vn).max()))
    assert differ_total <= 1e-3 * pairs


@pytest.mark.parametrize("BH,Lq,Lk,d", [(2, 128, 256, 64), (2, 64, 384, 128), (1, 192, 128, 64)])
@DTYPES
@pytest.mark.parametrize("path", ["default", "staged"])
def test_attention_and_dense_baseline(BH, Lq, Lk, d, dtype, path):
    """default: one kernel where the library has one (bf16x3 products), else the three stages."""
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=6300 + Lq + d, dtype=torch.float32)
    scale = 1 / math.sqrt(d)
    s = _shape(1, BH, Lq, Lk, d, dtype)
    attention = dfss.dfss_attention_staged if path == "staged" else dfss.dfss_attention
    O = attention(_dev(Q), _dev(K), _dev(V), s, scale)
    if path == "default" and dtype == DFSS_F32_BF16X3:
        Od = dfss.dense_attention_fused(_dev(Q), _dev(K), _dev(V), s, scale)
    else:
        Od = dfss.dense_attention(_dev(Q), _dev(K), _dev(V), s, scale)
    torch.cuda.synchronize()
    O, Od = O.cpu().numpy(), Od.cpu().numpy()
    Qn, Kn, Vn = Q.numpy(), K.numpy(), V.numpy()
    ref = oracle.attention(Qn, Kn, Vn, 1, 2, scale, store_bf16=False)
    assert np.abs(O - ref).max() <= 2e-2
    # rows whose selection cannot have differed (no pair inside the rounding error): fp32 accuracy
    for h in range(BH):
        S = oracle.scores(Qn[h], Kn[h], scale)
        bound = _score_error_bound(Qn[h], Kn[h], scale, dtype)
        safe = (np.abs(S[:, 0::2] - S[:, 1::2]) > 2 * (bound[:, 0::2] + bound[:, 1::2])).all(-1)
        assert safe.sum() > Lq // 2
        assert np.abs(O[h] - ref[h])[safe].max() <= TOL_O[dtype]
    # full attention (Eq. 1): N = M in the oracle
    refd = oracle.attention(Qn, Kn, Vn, 2, 2, scale, store_bf16=False)
    assert np.abs(Od - refd).max() <= TOL_O[dtype]


@DTYPES
def test_stage_calls_compose_to_attention(dtype):
    w = synth.WORKLOADS["tiny_1to2_f32"]
    Q, K, V = (_dev(t) for t in synth.make(w))
    s = _shape(w.B, w.H, w.L, w.L, w.d, dtype)
    vals, meta = dfss.dfss_sddmm_prune(Q, K, s, w.scale)
    O1 = dfss.dfss_spmm(dfss.dfss_sparse_softmax(vals, s), meta, V, s)
    O2 = dfss.dfss_attention_staged(Q, K, V, s, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2)
    if dtype == DFSS_F32_BF16X3:
        # the one-kernel path computes the same function with the softmax in another order
        O3 = dfss.dfss_attention(Q, K, V, s, w.scale)
        torch.cuda.synchronize()
        assert (O3 - O1).abs().max().item() <= 2e-5
        assert not torch.equal(O3, O1)          # (it really is the other kernel)


@pytest.mark.parametrize("name", ["bert_base_L512_1to2_f32", "long_L4096_1to2_f32", "large_head_L2048_d128_1to2_f32"])
def test_fused_kernels_at_full_size(name):
    """One-kernel DFSS and full attention of the bf16x3 mode on sampled heads of the full-size workloads."""
    w = synth.WORKLOADS[name]
    Q, K, V = synth.make(w)
    s = _shape(w.B, w.H, w.L, w.L, w.d, DFSS_F32_BF16X3)
    Qd, Kd, Vd = _dev(Q), _dev(K), _dev(V)
    O = dfss.dfss_attention(Qd, Kd, Vd, s, w.scale)
    Od = dfss.dense_attention_fused(Qd, Kd, Vd, s, w.scale)
    torch.cuda.synchronize()
    O, Od = O.cpu().numpy(), Od.cpu().numpy()
    assert np.isfinite(O).all() and np.isfinite(Od).all()
    for h in (0, w.BH - 1):
        Qn, Kn, Vn = Q[h].numpy(), K[h].numpy(), V[h].numpy()
        rows = slice(0, w.L, max(1, w.L // 256))            # every row block, a sample of rows
        ref = oracle.attention(Qn[rows], Kn, Vn, 1, 2, w.scale, store_bf16=False)
        assert np.abs(O[h][rows] - ref).max() <= 2e-2
        S = oracle.scores(Qn[rows], Kn, w.scale)
        bound = _score_error_bound(Qn[rows], Kn, w.scale, DFSS_F32_BF16X3)
        safe = (np.abs(S[:, 0::2] - S[:, 1::2]) > 2 * (bound[:, 0::2] + bound[:, 1::2])).all(-1)
        assert safe.sum() > 0
        assert np.abs(O[h][rows] - ref)[safe].max() <= TOL_O[DFSS_F32_BF16X3]
        refd = oracle.attention(Qn[rows], Kn, Vn, 2, 2, w.scale, store_bf16=False)
        assert np.abs(Od[h][rows] - refd).max() <= TOL_O[DFSS_F32_BF16X3]


@DTYPES
def test_unsupported_combinations_are_refused(dtype):
    s24 = Shape(1, 1, 64, 128, 64, 2, 4, dtype)
    assert dfss.dfss_vals_bytes(s24) == 0
    s = _shape(1, 1, 64, 128, 64, dtype)
    Q = torch.zeros(1, 64, 64, device=DEV)
    K = torch.zeros(1, 128, 64, device=DEV)
    if dtype == DFSS_F32:
        with pytest.raises(dfss.DfssError):
            dfss.dense_attention_fused(Q, K, K, s, 0.125)
    if dtype == DFSS_F32:      # block patterns and the one-kernel forms are taken with bf16x3 products only
        with pytest.raises(dfss.DfssError):
            dfss.dfss_attention_blocked(Q, K, K, None, torch.ones(1, 2, dtype=torch.uint8, device=DEV), s, 0.125)
        with pytest.raises(dfss.DfssError):
            dfss.dense_attention_fused_bias(Q, K, K, torch.zeros(1, 128, device=DEV), s, 0.125)
    with pytest.raises(ValueError):          # bfloat16 tensors with a float shape
        dfss.dfss_attention(Q.bfloat16(), K.bfloat16(), K.bfloat16(), s, 0.125)


def test_split_products_equal_fp32_on_bf16_exact_operands():
    """Operands that are exact in bfloat16 have lo = 0: both ways of forming the products then agree bit
    for bit in stage 1 whenever the fp32 sums are exact (small integers)."""
    Q, K, _ = synth.integer_qkv(2, 128, 256, 64, seed=6400, dtype=torch.float32)
    out = []
    for dtype in (DFSS_F32, DFSS_F32_BF16X3):
        s = _shape(1, 2, 128, 256, 64, dtype)
        vals, meta = dfss.dfss_sddmm_prune(_dev(Q), _dev(K), s, 0.125)
        torch.cuda.synchronize()
        out.append((vals.cpu(), meta.cpu()))
    assert torch.equal(out[0][0], out[1][0]) and torch.equal(out[0][1], out[1][1])


@DTYPES
def test_calls_replay_correctly_from_a_hip_graph(dtype):
    """The float-mode entry points enqueued into one graph: each replay (eager work, synchronisations and
    changed inputs in between) must reproduce the eager result of the same inputs bit for bit."""
    s = _shape(2, 2, 128, 256, 64, dtype)
    Q, K, V = (_dev(t) for t in synth.gaussian_qkv(4, 128, 256, 64, 1.0, seed=6500, dtype=torch.float32))
    ws = torch.empty(max(dfss.dfss_workspace_bytes(s), dfss.dense_workspace_bytes(s)), dtype=torch.uint8, device=DEV)
    split = dtype == DFSS_F32_BF16X3
    names = ["attention", "dense", "stages"] + (["dense_fused", "dQ", "dK", "dV"] if split else [])
    outs = {k: torch.empty_like(K if k in ("dK", "dV") else Q) for k in names}
    dO = torch.randn(Q.shape, generator=torch.Generator().manual_seed(6501)).to(DEV)
    ws_b = torch.empty(max(dfss.dfss_backward_workspace_bytes(s), 256), dtype=torch.uint8, device=DEV)
    vals = torch.empty((s.BH, s.Lq, s.Lc), dtype=torch.float32, device=DEV)
    meta = torch.empty((s.BH * s.Lq * s.meta_words,), dtype=torch.int16, device=DEV)

    def run_all():
        dfss.dfss_attention(Q, K, V, s, 0.125, O=outs["attention"], ws=ws)
        dfss.dense_attention(Q, K, V, s, 0.125, O=outs["dense"], ws=ws)
        if "dense_fused" in outs:
            dfss.dense_attention_fused(Q, K, V, s, 0.125, O=outs["dense_fused"])
        dfss.dfss_sddmm_prune(Q, K, s, 0.125, vals=vals, meta=meta)
        dfss.dfss_sparse_softmax(vals, s)
        dfss.dfss_spmm(vals, meta, V, s, O=outs["stages"])
        if split:
            dfss.dfss_attention_backward(dO, Q, K, V, outs["stages"], vals, meta, s, 0.125, dQ=outs["dQ"],
                                         dK=outs["dK"], dV=outs["dV"], ws=ws_b)

    run_all()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    for rep in range(3):
        Q.copy_(torch.randn(Q.shape, generator=torch.Generator().manual_seed(6600 + rep)))
        run_all()
        torch.cuda.synchronize()
        eager = {k: v.clone() for k, v in outs.items()}
        for v in outs.values():
            v.zero_()
        g.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(outs[k], eager[k]), (rep, k)


def test_one_kernel_path_when_every_block_raises_the_maximum():
    """Scores that grow with the key index: the running maximum of every query rises in every block, so the
    output accumulators are rescaled each time; and a row whose early weights underflow to zero."""
    BH, Lq, Lk, d = 2, 128, 1024, 64
    g = torch.Generator().manual_seed(6700)
    Q = torch.ones(BH, Lq, d) + 0.01 * torch.randn(BH, Lq, d, generator=g)
    ramp = torch.linspace(-3.0, 3.0, Lk).view(1, Lk, 1)
    K = ramp * torch.ones(BH, Lk, d) + 0.01 * torch.randn(BH, Lk, d, generator=g)
    K[1] *= 4.0                                   # head 1: range of scores ~ 190, early weights underflow
    V = torch.randn(BH, Lk, d, generator=g)
    s = _shape(1, BH, Lq, Lk, d, DFSS_F32_BF16X3)
    scale = 0.125
    O = dfss.dfss_attention(_dev(Q), _dev(K), _dev(V), s, scale)
    Od = dfss.dense_attention_fused(_dev(Q), _dev(K), _dev(V), s, scale)
    torch.cuda.synchronize()
    ref = oracle.attention(Q.numpy(), K.numpy(), V.numpy(), 1, 2, scale, store_bf16=False)
    refd = oracle.attention(Q.numpy(), K.numpy(), V.numpy(), 2, 2, scale, store_bf16=False)
    assert np.isfinite(O.cpu().numpy()).all()
    # (near-tied pairs may be decided differently: neighbouring keys differ by little here, hence the path bar)
    assert np.abs(O.cpu().numpy() - ref).max() <= 2e-2
    assert np.abs(Od.cpu().numpy() - refd).max() <= TOL_O[DFSS_F32_BF16X3]


# ----------------------------------------------------------------------------------
# additive key bias (padding mask) in the float mode: bf16x3 products only
# ----------------------------------------------------------------------------------
def _padding_case(B, H, Lq, Lk, d, seed, integer):
    """Float inputs of a padded batch: lengths that cut through pairs and blocks, bias 0 / -inf, plus a few
    finite bias values (multiples of 1/4: exact in every sum that occurs on integer inputs)."""
    gen = synth.integer_qkv if integer else synth.gaussian_qkv
    args = (B * H, Lq, Lk, d, seed) if integer else (B * H, Lq, Lk, d, 1.0, seed)
    Q, K, V = gen(*args, dtype=torch.float32)
    lengths = synth.padding_lengths(B, Lk, seed + 1, min_frac=0.3)
    lengths[lengths % 2 == 0] -= 1                       # odd lengths: the mask cuts a pair
    lengths[0] = Lk
    bias = synth.key_padding_bias(lengths, Lk)
    g = torch.Generator().manual_seed(seed + 2)
    finite = torch.randint(-8, 9, (B, Lk), generator=g).float() / 4
    bias = torch.where(torch.isinf(bias), bias, torch.where(torch.rand(B, Lk, generator=g) < 0.2, finite, bias))
    return Q, K, V, lengths, bias


@DTYPES
@pytest.mark.parametrize("scale", [0.125, float(np.float32(1.0 / 3.0))], ids=["pow2", "third"])
@pytest.mark.parametrize("B,H,Lq,Lk,d", [(2, 2, 128, 256, 64), (3, 1, 64, 384, 128), (16, 4, 1024, 128, 64)])
def test_stage1_key_bias_bit_exact_on_integer_inputs(B, H, Lq, Lk, d, dtype, scale):
    Q, K, _, lengths, bias = _padding_case(B, H, Lq, Lk, d, 6800 + Lq + d, integer=True)
    s = _shape(B, H, Lq, Lk, d, dtype)
    vals, meta = dfss.dfss_sddmm_prune_bias(_dev(Q), _dev(K), _dev(bias), s, scale)
    torch.cuda.synchronize()
    vals, meta = vals.cpu().numpy(), _meta_np(meta, s)
    assert int((lengths % 2 != 0).sum()) > 0
    for h in range(B * H) if B * H <= 8 else (0, 5, B * H - 1):
        S = oracle.add_key_bias(oracle.scores(Q[h].numpy(), K[h].numpy(), scale), bias[h // H].numpy())
        _, v, kidx = oracle.prune(S, 1, 2)
        assert np.array_equal(meta[h], oracle.encode_meta_f32(kidx, Lk)), f"metadata differs in head {h}"
        assert np.array_equal(vals[h], v), f"kept scores differ in head {h}"      # includes -inf entries


@pytest.mark.parametrize("B,H,Lq,Lk,d", [(2, 2, 128, 256, 64), (2, 2, 64, 384, 128)])
def test_attention_key_bias(B, H, Lq, Lk, d):
    """Whole path with a padding mask: one kernel, stage kernels, both full-attention baselines."""
    Q, K, V, lengths, bias = _padding_case(B, H, Lq, Lk, d, 6900 + Lq + d, integer=False)
    s = _shape(B, H, Lq, Lk, d, DFSS_F32_BF16X3)
    scale = 1.0 / math.sqrt(d)
    Qd, Kd, Vd, bd = _dev(Q), _dev(K), _dev(V), _dev(bias)
    O = dfss.dfss_attention_bias(Qd, Kd, Vd, bd, s, scale)
    Odf = dfss.dense_attention_fused_bias(Qd, Kd, Vd, bd, s, scale)
    Od = dfss.dense_attention_bias(Qd, Kd, Vd, bd, s, scale)
    O0 = dfss.dfss_attention_bias(Qd, Kd, Vd, None, s, scale)          # NULL bias = the plain call
    O1 = dfss.dfss_attention(Qd, Kd, Vd, s, scale)
    Os = dfss.dfss_attention_staged_bias(Qd, Kd, Vd, bd, s, scale)
    torch.cuda.synchronize()
    assert torch.equal(O0, O1)
    Qn, Kn, Vn = Q.numpy(), K.numpy(), V.numpy()
    ref = oracle.attention(Qn, Kn, Vn, 1, 2, scale, store_bf16=False, key_bias=bias.numpy(), heads_per_batch=H)
    refd = oracle.attention(Qn, Kn, Vn, 2, 2, scale, store_bf16=False, key_bias=bias.numpy(), heads_per_batch=H)
    for name, got in (("one kernel", O), ("staged", Os)):
        got = got.cpu().numpy()
        assert np.isfinite(got).all(), name
        assert np.abs(got - ref).max() <= 2e-2, name
    for name, got in (("dense fused", Odf), ("dense 3-stage", Od)):
        assert np.abs(got.cpu().numpy() - refd).max() <= TOL_O[DFSS_F32_BF16X3], name
    # fp32 matrix instructions: the stage kernels take the bias too (no one-kernel form there)
    s32 = _shape(B, H, Lq, Lk, d, DFSS_F32)
    O32 = dfss.dfss_attention_bias(Qd, Kd, Vd, bd, s32, scale)
    O32s = dfss.dfss_attention_staged_bias(Qd, Kd, Vd, bd, s32, scale)
    Od32 = dfss.dense_attention_bias(Qd, Kd, Vd, bd, s32, scale)
    torch.cuda.synchronize()
    assert torch.equal(O32, O32s)
    assert np.isfinite(O32.cpu().numpy()).all()
    assert np.abs(O32.cpu().numpy() - ref).max() <= 2e-2
    assert np.abs(Od32.cpu().numpy() - refd).max() <= TOL_O[DFSS_F32]
    for h in range(B * H):
        S = oracle.add_key_bias(oracle.scores(Qn[h], Kn[h], scale), bias[h // H].numpy())
        bound = _score_error_bound(Qn[h], Kn[h], scale, DFSS_F32)
        with np.errstate(invalid="ignore"):
            gap = np.abs(S[:, 0::2] - S[:, 1::2])
        safe = (np.isnan(gap) | (gap > 2 * (bound[:, 0::2] + bound[:, 1::2]))).all(-1)
        assert safe.sum() > 0
        assert np.abs(O32.cpu().numpy()[h] - ref[h])[safe].max() <= TOL_O[DFSS_F32]
    # rows with no pair inside the error window: fp32-like accuracy of the pruned path
    for h in range(B * H):
        S = oracle.add_key_bias(oracle.scores(Qn[h], Kn[h], scale), bias[h // H].numpy())
        bound = _score_error_bound(Qn[h], Kn[h], scale, DFSS_F32_BF16X3)
        with np.errstate(invalid="ignore"):
            gap = np.abs(S[:, 0::2] - S[:, 1::2])              # nan where both keys of a pair are masked
        safe = (np.isnan(gap) | (gap > 2 * (bound[:, 0::2] + bound[:, 1::2]))).all(-1)
        assert safe.sum() > 0
        assert np.abs(O.cpu().numpy()[h] - ref[h])[safe].max() <= TOL_O[DFSS_F32_BF16X3]


def test_attention_key_bias_first_blocks_fully_masked():
    """Leading key blocks that are entirely masked: the running maximum stays at its start value until the
    first real key, and nothing of the masked blocks reaches the output."""
    B, H, Lq, Lk, d = 1, 2, 64, 512, 64
    Q, K, V = synth.gaussian_qkv(B * H, Lq, Lk, d, 1.0, 6950, dtype=torch.float32)
    bias = torch.zeros(B, Lk)
    bias[:, :200] = float("-inf")
    s = _shape(B, H, Lq, Lk, d, DFSS_F32_BF16X3)
    O = dfss.dfss_attention_bias(_dev(Q), _dev(K), _dev(V), _dev(bias), s, 0.125)
    Od = dfss.dense_attention_fused_bias(_dev(Q), _dev(K), _dev(V), _dev(bias), s, 0.125)
    torch.cuda.synchronize()
    ref = oracle.attention(Q.numpy(), K.numpy(), V.numpy(), 1, 2, 0.125, store_bf16=False, key_bias=bias.numpy(),
                           heads_per_batch=H)
    refd = oracle.attention(Q.numpy(), K.numpy(), V.numpy(), 2, 2, 0.125, store_bf16=False, key_bias=bias.numpy(),
                            heads_per_batch=H)
    assert np.isfinite(O.cpu().numpy()).all()
    assert np.abs(O.cpu().numpy() - ref).max() <= 2e-2
    assert np.abs(Od.cpu().numpy() - refd).max() <= TOL_O[DFSS_F32_BF16X3]


# ----------------------------------------------------------------------------------
# hybrid block sparsity x 1:2 (64 x 64 block patterns) in the float mode: bf16x3 products only
# ----------------------------------------------------------------------------------
@pytest.mark.parametrize("BH,Lq,Lk,d", [(2, 256, 256, 64), (2, 128, 1024, 64), (1, 192, 512, 128)])
def test_attention_blocked(BH, Lq, Lk, d):
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=7000 + Lq + Lk + d, dtype=torch.float32)
    small = Lk // 64 <= 4
    bm = synth.block_pattern(Lq // 64, Lk // 64, seed=7001 + Lk, window=0 if small else 1, n_random=0 if small else 3)
    assert 0 < int(bm.sum()) < bm.numel()
    s = _shape(1, BH, Lq, Lk, d, DFSS_F32_BF16X3)
    scale = 1.0 / math.sqrt(d)
    Qd, Kd, Vd, bmd = _dev(Q), _dev(K), _dev(V), _dev(bm)
    O = dfss.dfss_attention_blocked(Qd, Kd, Vd, None, bmd, s, scale)
    Od = dfss.dense_attention_fused_blocked(Qd, Kd, Vd, None, bmd, s, scale)
    torch.cuda.synchronize()
    Qn, Kn, Vn = Q.numpy(), K.numpy(), V.numpy()
    ref = oracle.attention(Qn, Kn, Vn, 1, 2, scale, store_bf16=False, block_mask=bm.numpy(), block_size=64)
    ref_dense = oracle.attention(Qn, Kn, Vn, 2, 2, scale, store_bf16=False, block_mask=bm.numpy(), block_size=64)
    assert np.abs(O.cpu().numpy() - ref).max() <= 2e-2
    assert np.abs(Od.cpu().numpy() - ref_dense).max() <= TOL_O[DFSS_F32_BF16X3]
    # the pattern matters: full attention gives something else
    assert np.abs(ref - oracle.attention(Qn, Kn, Vn, 1, 2, scale, store_bf16=False)).max() > 0.05


def test_attention_blocked_with_key_bias_and_full_pattern():
    B, H, L, d = 2, 2, 384, 64
    Q, K, V, lengths, bias = _padding_case(B, H, L, L, d, 7100, integer=False)
    s = _shape(B, H, L, L, d, DFSS_F32_BF16X3)
    Qd, Kd, Vd, bd = _dev(Q), _dev(K), _dev(V), _dev(bias)
    # block pattern and padding mask together (row blocks keep block 0, which always holds real keys)
    bm = synth.block_pattern(L // 64, L // 64, seed=7101, n_random=1)
    O = dfss.dfss_attention_blocked(Qd, Kd, Vd, bd, _dev(bm), s, 0.125)
    torch.cuda.synchronize()
    ref = oracle.attention(Q.numpy(), K.numpy(), V.numpy(), 1, 2, 0.125, store_bf16=False, key_bias=bias.numpy(),
                           heads_per_batch=H, block_mask=bm.numpy(), block_size=64)
    assert np.abs(O.cpu().numpy() - ref).max() <= 2e-2
    # a pattern that keeps every block is the unblocked call, bit for bit
    ones = torch.ones((L // 64, L // 64), dtype=torch.uint8)
    O1 = dfss.dfss_attention_blocked(Qd, Kd, Vd, bd, _dev(ones), s, 0.125)
    O2 = dfss.dfss_attention_bias(Qd, Kd, Vd, bd, s, 0.125)
    O3 = dfss.dense_attention_fused_blocked(Qd, Kd, Vd, None, _dev(ones), s, 0.125)
    O4 = dfss.dense_attention_fused(Qd, Kd, Vd, s, 0.125)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(O3, O4)


# ----------------------------------------------------------------------------------
# backward pass through the fixed selection in the float mode (bf16x3 products)
# ----------------------------------------------------------------------------------
def _oracle_forward_f32(Qn, Kn, scale):
    """Selection, softmax weights and canonical metadata of the oracle, per head."""
    kidx, P, meta = [], [], []
    for h in range(Qn.shape[0]):
        S = oracle.scores(Qn[h], Kn[h], scale)
        _, v, ki = oracle.prune(S, 1, 2)
        kidx.append(ki)
        P.append(oracle.softmax_kept(v))
        meta.append(oracle.encode_meta_f32(ki, Kn.shape[1]))
    return np.stack(kidx), np.stack(P), np.stack(meta)


@pytest.mark.parametrize("BH,Lq,Lk,d", [(2, 128, 256, 64), (1, 192, 128, 128), (2, 64, 384, 64)])
def test_transposed_spmm(BH, Lq, Lk, d):
    Q, K, _ = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=7300 + Lq + Lk, dtype=torch.float32)
    X = torch.randn(BH, Lq, d, generator=torch.Generator().manual_seed(7301 + d))
    s = _shape(1, BH, Lq, Lk, d, DFSS_F32_BF16X3)
    kidx, P, meta_c = _oracle_forward_f32(Q.numpy(), K.numpy(), 1.0 / math.sqrt(d))
    meta = dfss.dfss_meta_from_canonical(_dev(torch.from_numpy(meta_c.view(np.int16))), s)
    out = dfss.dfss_spmm_t(_dev(torch.from_numpy(P)), meta, _dev(X), s)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    for h in range(BH):
        Pd = np.zeros((Lq, Lk))
        np.put_along_axis(Pd, kidx[h].astype(np.int64), P[h].astype(np.float64), axis=1)
        Xh = X[h].numpy().astype(np.float64)
        ref = Pd.T @ Xh
        # split products (3.01 * 2^-18 per product) + fp32 accumulation of 3 Lq terms
        bound = (3.01 * 2.0 ** -18 + 3 * Lq * U) * (np.abs(Pd).T @ np.abs(Xh))
        assert np.all(np.abs(out[h] - ref) <= bound + 1e-12)


@pytest.mark.parametrize("BH,Lq,Lk,d", [(2, 128, 256, 64), (2, 192, 384, 64), (2, 128, 128, 128)])
def test_backward_against_oracle_through_the_same_selection(BH, Lq, Lk, d):
    """The kernels are fed the oracle's forward results (weights, metadata, O), so both sides differentiate
    through exactly the same selection."""
    scale = 1.0 / math.sqrt(d)
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=7400 + Lq + d, dtype=torch.float32)
    dO = torch.randn(BH, Lq, d, generator=torch.Generator().manual_seed(7401 + Lq))
    Qn, Kn, Vn, dOn = Q.numpy(), K.numpy(), V.numpy(), dO.numpy()
    kidx, P, meta_c = _oracle_forward_f32(Qn, Kn, scale)
    O = np.stack([oracle.spmm(P[h], kidx[h], Vn[h]) for h in range(BH)])
    s = _shape(1, BH, Lq, Lk, d, DFSS_F32_BF16X3)
    meta = dfss.dfss_meta_from_canonical(_dev(torch.from_numpy(meta_c.view(np.int16))), s)
    dQ, dK, dV = dfss.dfss_attention_backward(_dev(dO), _dev(Q), _dev(K), _dev(V), _dev(torch.from_numpy(O)),
                                              _dev(torch.from_numpy(P)), meta, s, scale)
    torch.cuda.synchronize()
    worst = 0.0
    for h in range(BH):
        rQ, rK, rV = oracle.attention_backward(Qn[h], Kn[h], Vn[h], dOn[h], P[h], kidx[h], scale)
        for name, got, ref in (("dQ", dQ[h], rQ), ("dK", dK[h], rK), ("dV", dV[h], rV)):
            # split products drop at most 3.01 * 2^-18 per product; dS = P (dP - delta) cancels, so the bar is
            # relative to the largest entry of the result, not to each entry
            err = np.max(np.abs(got.cpu().numpy() - ref)) / np.max(np.abs(ref))
            worst = max(worst, err)
            assert err <= 1e-4, (name, h, err)
    print(f"largest relative error {worst:.2e}")


def test_forward_stages_then_backward_on_exact_scores():
    """GPU forward (three stage calls, integer-valued Q and K: the selection equals the oracle's exactly)
    followed by the GPU backward, against the oracle end to end."""
    BH, L, d = 2, 256, 64
    Q, K, V = synth.integer_qkv(BH, L, L, d, seed=7500, dtype=torch.float32)
    Q, K = Q * 0.25, K * 0.25                                  # keeps the softmax soft; still exact
    dO = torch.randn(BH, L, d, generator=torch.Generator().manual_seed(7501))
    s = _shape(1, BH, L, L, d, DFSS_F32_BF16X3)
    Qd, Kd, Vd, dOd = _dev(Q), _dev(K), _dev(V), _dev(dO)
    vals, meta = dfss.dfss_sddmm_prune(Qd, Kd, s, 0.125)
    dfss.dfss_sparse_softmax(vals, s)
    O = dfss.dfss_spmm(vals, meta, Vd, s)
    dQ, dK, dV = dfss.dfss_attention_backward(dOd, Qd, Kd, Vd, O, vals, meta, s, 0.125)
    torch.cuda.synchronize()
    Qn, Kn, Vn, dOn = Q.numpy(), K.numpy(), V.numpy(), dO.numpy()
    kidx, P, meta_c = _oracle_forward_f32(Qn, Kn, 0.125)
    assert np.array_equal(_meta_np(meta, s), meta_c)           # same selection on both sides
    for h in range(BH):
        rQ, rK, rV = oracle.attention_backward(Qn[h], Kn[h], Vn[h], dOn[h], P[h], kidx[h], 0.125)
        for name, got, ref in (("dQ", dQ[h], rQ), ("dK", dK[h], rK), ("dV", dV[h], rV)):
            assert np.max(np.abs(got.cpu().numpy() - ref)) <= 1e-4 * np.max(np.abs(ref)), name
