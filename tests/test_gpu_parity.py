"""Parity of the HIP path against the CPU oracle, through the C ABI (needs an MI355X).

Bars (stated by the benchmark spec for this path):
  * masks / metadata bit-exact on integer-valued Q, K (scores exact in fp32);
  * on Gaussian inputs >= 99.9 % of groups identical once groups whose N-th and (N+1)-th
    scores are closer than 1e-3 are set aside, kept values within one bf16 step;
  * output O within 2e-2 max-abs of the oracle.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2203_00091_amd as dfss
from paper_2203_00091_amd import Shape, binding, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
BF16_STEP = 2.0 ** -7  # spacing of bfloat16 relative to the value (8 significant bits)


def _dev(t):
    return t.to(DEV).contiguous()


def _np(t):
    return t.detach().to("cpu", torch.float32).numpy()


def _canon_meta(meta, s):
    canon = dfss.dfss_meta_to_canonical(meta, s)
    torch.cuda.synchronize()
    return canon.cpu().numpy().view(np.uint16)


def _oracle_head(Q, K, V, N, M, scale):
    """All intermediate results of the oracle for one head (numpy float32 inputs)."""
    S = oracle.scores(Q, K, scale)
    mask, vals, kidx = oracle.prune(S, N, M)
    meta = oracle.encode_meta(kidx, K.shape[0])
    return dict(S=S, mask=mask, vals=vals, kidx=kidx, meta=meta)


def _stage1(Qt, Kt, s, scale):
    vals, meta = dfss.dfss_sddmm_prune(_dev(Qt), _dev(Kt), s, scale)
    torch.cuda.synchronize()
    return _np(vals), _canon_meta(meta, s)


# ----------------------------------------------------------------------------------
# stage 1: bit-exact on integer inputs
# ----------------------------------------------------------------------------------
@pytest.mark.parametrize("BH,Lq,Lk,d,N,M,scale", [
    (1, 256, 256, 64, 2, 4, 0.125),     # the tiny check of the task
    (3, 128, 384, 64, 2, 4, 0.125),     # several heads, rectangular, several key tiles
    (2, 192, 256, 128, 2, 4, 0.125),    # d = 128, 16-query tiles (Lq not a multiple of 128)
    (2, 128, 256, 64, 1, 2, 0.125),     # 1:2
    (1, 64, 128, 128, 1, 2, 0.125),     # smallest legal shape
    (1, 128, 8192, 64, 2, 4, 0.125),    # longest key sequence the library accepts
    (2, 128, 256, 128, 2, 4, float(np.float32(1.0 / math.sqrt(128.0)))),   # scale applied after the product
    (2, 192, 384, 64, 1, 2, float(np.float32(1.0 / 3.0))),                  # same, 16-query tiles, 1:2
])
def test_stage1_bit_exact_on_integer_inputs(BH, Lq, Lk, d, N, M, scale):
    Q, K, _ = synth.integer_qkv(BH, Lq, Lk, d, seed=1002 + Lq + d + N)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    vals, meta = _stage1(Q, K, s, scale)
    Qn, Kn = synth.to_numpy_f32(Q), synth.to_numpy_f32(K)
    ties = 0
    for h in range(BH):
        o = _oracle_head(Qn[h], Kn[h], None, N, M, scale)
        assert np.array_equal(meta[h], o["meta"]), f"metadata differs in head {h}"
        assert np.array_equal(vals[h], oracle.round_bf16(o["vals"])), f"kept values differ in head {h}"
        g = o["S"].reshape(Lq, -1, M)
        ties += int(np.sum(np.sort(g, -1)[..., M - N - 1] == np.sort(g, -1)[..., M - N]))
    assert ties > 0  # the tie rule was exercised


def test_stage1_all_equal_scores_keep_lowest_indices():
    BH, L, d = 1, 128, 64
    Q = torch.zeros(BH, L, d, dtype=torch.bfloat16)
    K = torch.ones(BH, L, d, dtype=torch.bfloat16)
    vals, meta = _stage1(Q, K, Shape(1, BH, L, L, d, 2, 4), 0.125)
    assert np.all(meta == 0x4444) and np.all(vals == 0)
    vals, meta = _stage1(Q, K, Shape(1, BH, L, L, d, 1, 2), 0.125)
    assert np.all(meta == 0x8888)


# ----------------------------------------------------------------------------------
# stage 1: Gaussian inputs
# ----------------------------------------------------------------------------------
def _compare_stage1_gaussian(Qn, Kn, vals, meta, N, M, scale):
    """Returns (#groups, #near-tie groups, #disagreeing groups outside near ties)."""
    Lq, Lk = Qn.shape[0], Kn.shape[0]
    o = _oracle_head(Qn, Kn, None, N, M, scale)
    gsort = np.sort(o["S"].reshape(Lq, -1, M), -1)
    gap = gsort[..., M - N] - gsort[..., M - N - 1]          # N-th minus (N+1)-th largest
    # compare per run of 4 keys (one 4-bit code); a run is near-tied if any of its groups is
    near = (gap < 1e-3).reshape(Lq, Lk // 4, -1).any(-1)
    got = np.stack([(meta >> (4 * k)) & 0xF for k in range(4)], -1).reshape(Lq, -1)
    exp = np.stack([(o["meta"] >> (4 * k)) & 0xF for k in range(4)], -1).reshape(Lq, -1)
    differ = got != exp
    bad = differ & ~near
    # kept values: where the selection agrees, within one bf16 step of the oracle's value
    same = np.repeat(~differ, 2, axis=1)
    ref = oracle.round_bf16(o["vals"])
    err = np.abs(vals - ref)[same]
    tol = (BF16_STEP * np.abs(ref) + 1e-6)[same]
    assert np.all(err <= tol), f"kept value off by more than a bf16 step: {err.max()}"
    return differ.size, int(near.sum()), int(bad.sum())


@pytest.mark.parametrize("name", ["tiny_2to4"])
def test_stage1_tiny_gaussian(name):
    w = synth.WORKLOADS[name]
    Q, K, _ = synth.make(w)
    s = Shape(w.B, w.H, w.L, w.L, w.d, w.N, w.M)
    vals, meta = _stage1(Q, K, s, w.scale)
    Qn, Kn = synth.to_numpy_f32(Q), synth.to_numpy_f32(K)
    total, near, bad = _compare_stage1_gaussian(Qn[0], Kn[0], vals[0], meta[0], w.N, w.M, w.scale)
    assert bad <= 1e-3 * total, (total, near, bad)


@pytest.mark.parametrize("name,heads", [
    ("bert_base_L384_2to4", [0, 17, 95]),
    ("bert_base_L512_1to2", [0, 101, 191]),
    ("long_L4096_2to4", [5]),
    ("large_head_L2048_d128_2to4", [63]),
    ("large_head_L2048_d128_1to2", [0]),
])
def test_stage1_full_size_sampled_heads(name, heads):
    """The launch configuration the benchmark times, checked on sampled heads."""
    w = synth.WORKLOADS[name]
    Q, K, _ = synth.make(w)
    s = Shape(w.B, w.H, w.L, w.L, w.d, w.N, w.M)
    vals, meta = dfss.dfss_sddmm_prune(_dev(Q), _dev(K), s, w.scale)
    canon = dfss.dfss_meta_to_canonical(meta, s)
    torch.cuda.synchronize()
    for h in heads:
        v = _np(vals[h])
        m = canon[h].cpu().numpy().view(np.uint16)
        total, near, bad = _compare_stage1_gaussian(synth.to_numpy_f32(Q[h]), synth.to_numpy_f32(K[h]), v, m,
                                                    w.N, w.M, w.scale)
        assert bad <= 1e-3 * total, (name, h, total, near, bad)
        assert near < 0.01 * total


# ----------------------------------------------------------------------------------
# stage 2: softmax over kept entries
# ----------------------------------------------------------------------------------
@pytest.mark.parametrize("BH,Lq,Lk", [(2, 64, 128), (2, 128, 384), (1, 64, 1024), (1, 64, 4096), (1, 64, 8192)])
def test_stage2_softmax(BH, Lq, Lk):
    g = torch.Generator().manual_seed(77 + Lk)
    x = (torch.randn(BH, Lq, Lk // 2, generator=g) * 2.0).to(torch.bfloat16)
    x[0, 0, :] = 0.0            # uniform row
    x[0, 1, 3] = 60.0           # one dominant entry
    x[0, 2, :] = -80.0          # large negative offsets must not underflow the row
    s = Shape(1, BH, Lq, Lk, 64, 2, 4)
    y = dfss.dfss_sparse_softmax(_dev(x).clone(), s)
    torch.cuda.synchronize()
    y = _np(y)
    for h in range(BH):
        ref = oracle.softmax_kept(_np(x[h]))
        assert np.all(np.abs(y[h] - ref) <= 2.0 ** -8 * ref + 1e-7)
    assert np.max(np.abs(y.sum(-1) - 1.0)) < 1e-2


# ----------------------------------------------------------------------------------
# stage 3: compressed weights times V, fed with oracle-made operands
# ----------------------------------------------------------------------------------
@pytest.mark.parametrize("BH,Lq,Lk,d,N,M", [(2, 64, 128, 64, 2, 4), (2, 128, 384, 64, 2, 4), (1, 64, 256, 128, 2, 4),
                                            (2, 64, 256, 64, 1, 2)])
def test_stage3_spmm(BH, Lq, Lk, d, N, M):
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=300 + Lk + d + N)
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    s = Shape(1, BH, Lq, Lk, d, N, M)
    P = np.empty((BH, Lq, Lk // 2), np.float32)
    meta = np.empty((BH, Lq, Lk // 16), np.uint16)
    ref = np.empty((BH, Lq, d), np.float32)
    for h in range(BH):
        o = _oracle_head(Qn[h], Kn[h], None, N, M, 1 / math.sqrt(d))
        P[h] = oracle.round_bf16(oracle.softmax_kept(o["vals"]))
        meta[h] = o["meta"]
        ref[h] = oracle.spmm(P[h], o["kidx"], Vn[h])
    P_t = torch.from_numpy(P).to(torch.bfloat16)
    assert np.array_equal(_np(P_t), P)
    meta_lib = dfss.dfss_meta_from_canonical(_dev(torch.from_numpy(meta.view(np.int16))), s)
    O = dfss.dfss_spmm(_dev(P_t), meta_lib, _dev(V), s)
    torch.cuda.synchronize()
    err = np.abs(_np(O) - ref)
    assert np.all(err <= 2.0 ** -8 * np.abs(ref) + 1e-4), err.max()


def test_meta_order_round_trip():
    s = Shape(1, 3, 128, 256, 64, 2, 4)
    canon = torch.randint(-32768, 32767, (3, 128, 16), dtype=torch.int16)
    lib = dfss.dfss_meta_from_canonical(_dev(canon), s)
    back = dfss.dfss_meta_to_canonical(lib, s)
    torch.cuda.synchronize()
    assert torch.equal(back.cpu(), canon)
    # documented order: lib32[bh][r/16][v/4][r%16][slot(v%4)] = canon32[bh][r][v], slot(c) = 2*(c%2) + c/2
    lib5 = lib.cpu().view(torch.int32).view(3, 8, 2, 16, 4)          # [bh][r/16][v/4][r%16][slot]
    c32 = canon.view(torch.int32).view(3, 8, 16, 2, 4)               # [bh][r/16][r%16][v/4][c]
    for c in range(4):
        slot = 2 * (c % 2) + c // 2
        assert torch.equal(lib5[:, :, :, :, slot], c32[:, :, :, :, c].permute(0, 1, 3, 2))


# ----------------------------------------------------------------------------------
# whole path
# ----------------------------------------------------------------------------------
def _staged_attention(Qd, Kd, Vd, s, scale):
    """The stage kernels through a workspace (stage 1, then the product that applies the softmax as it reads)."""
    return dfss.dfss_attention_staged(Qd, Kd, Vd, s, scale)


def _check_attention(w, heads=None):
    Q, K, V = synth.make(w)
    s = Shape(w.B, w.H, w.L, w.L, w.d, w.N, w.M)
    Qd, Kd, Vd = _dev(Q), _dev(K), _dev(V)
    O = dfss.dfss_attention(Qd, Kd, Vd, s, w.scale)          # one fused kernel
    Os = _staged_attention(Qd, Kd, Vd, s, w.scale)           # stage kernels via the workspace
    # the three stage calls compose to the same function
    vals, meta = dfss.dfss_sddmm_prune(Qd, Kd, s, w.scale)
    dfss.dfss_sparse_softmax(vals, s)
    O3 = dfss.dfss_spmm(vals, meta, Vd, s)
    Od = dfss.dense_attention(Qd, Kd, Vd, s, w.scale)
    Odf = dfss.dense_attention_fused(Qd, Kd, Vd, s, w.scale)
    torch.cuda.synchronize()
    O, Os, O3, Od, Odf = _np(O), _np(Os), _np(O3), _np(Od), _np(Odf)
    heads = list(range(w.BH)) if heads is None else heads
    Qn, Kn, Vn = (synth.to_numpy_f32(t[heads]) for t in (Q, K, V))
    ref = oracle.attention(Qn, Kn, Vn, w.N, w.M, w.scale)
    ref_dense = oracle.attention(Qn, Kn, Vn, 1, 1, w.scale)
    assert np.max(np.abs(O[heads] - ref)) <= 2e-2
    assert np.max(np.abs(Os[heads] - ref)) <= 2e-2
    # the three stage calls store the kept scores and the weights as bfloat16: against the oracle with the same
    # two roundings only the output rounding (2^-9 relative) and an occasional weight that rounds the other way remain
    ref_stored = oracle.attention(Qn, Kn, Vn, w.N, w.M, w.scale, store_bf16=True)
    assert (np.abs(O3[heads] - ref_stored) <= 2.0 ** -8 * np.abs(ref_stored) + 2e-3).all(), \
        np.max(np.abs(O3[heads] - ref_stored))
    # same stage 1, so the same keys are kept on every head; the staged call normalises after the product (its weights
    # are exp(s - max) rounded to bfloat16, divided by their sum at the end), the three calls round the normalised
    # weights: a bfloat16 rounding of the weights and one of the output apart
    assert np.max(np.abs(Os - O3)) <= 2e-2
    # One kernel against three kernels on EVERY head (no oracle here).  The two paths round their scores
    # differently (the one-kernel path forms them relative to its softmax reference), so where the N-th and
    # (N+1)-th score of a run are a rounding error apart they may keep different keys -- both choices are the
    # function's up to rounding, but a key with a large weight then moves its row by more than 2e-2.  Such rows
    # are a handful in 10^5 (the heads checked against the oracle above have none); anything systematic is not.
    row_diff = np.abs(O - O3).max(-1)
    assert (row_diff > 2e-2).mean() <= 1e-4
    assert row_diff.max() <= 0.25
    assert np.max(np.abs(Od[heads] - ref_dense)) <= 2e-2
    assert np.max(np.abs(Odf[heads] - ref_dense)) <= 2e-2
    return O, ref


def test_attention_tiny():
    _check_attention(synth.WORKLOADS["tiny_2to4"])
    _check_attention(synth.WORKLOADS["tiny_2to4_int"])


def test_attention_bert_base_full():
    _check_attention(synth.WORKLOADS["bert_base_L384_2to4"])


@pytest.mark.parametrize("name,heads", [
    ("bert_base_L512_1to2", [0, 64, 191]),
    ("long_L1024_2to4", [3, 20]),
    ("long_L2048_2to4", [11]),
    ("long_L4096_2to4", [23]),
    ("large_head_L2048_d128_2to4", [7]),
    ("large_head_L2048_d128_1to2", [40]),
])
def test_attention_full_size_sampled_heads(name, heads):
    _check_attention(synth.WORKLOADS[name], heads)


VARIANTS = [binding.VARIANT_Q16, binding.VARIANT_Q16X2, binding.VARIANT_Q32W2, binding.VARIANT_Q32W4,
            binding.VARIANT_Q32K2]


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("BH,L,d,N,M", [(3, 256, 64, 2, 4), (2, 384, 64, 1, 2), (2, 256, 128, 2, 4)])
def test_fused_attention_every_tile_shape(variant, BH, L, d, N, M):
    """Each tiling of the fused kernel (16- or 32-query tiles, 2 or 4 waves) against the oracle."""
    Q, K, V = synth.gaussian_qkv(BH, L, L, d, 1.0, seed=900 + L + d + N)
    s = Shape(1, BH, L, L, d, N, M)
    scale = 1.0 / math.sqrt(d)
    O = binding.internal_attention_variant(_dev(Q), _dev(K), _dev(V), None, s, scale, variant)
    Od = binding.internal_attention_variant(_dev(Q), _dev(K), _dev(V), None, s, scale, variant, dense=True)
    torch.cuda.synchronize()
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    assert np.max(np.abs(_np(O) - oracle.attention(Qn, Kn, Vn, N, M, scale))) <= 2e-2
    assert np.max(np.abs(_np(Od) - oracle.attention(Qn, Kn, Vn, 1, 1, scale))) <= 2e-2


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M", [
    (2, 128, 640, 64, 2, 4),     # more keys than queries, 5 key blocks of 128
    (3, 320, 128, 64, 1, 2),     # more queries than keys, Lq a multiple of 64 only
    (1, 64, 8192, 128, 2, 4),    # longest key sequence, smallest query tile
])
def test_attention_rectangular(BH, Lq, Lk, d, N, M):
    """Lq != Lk (cross attention): fused kernel, stage kernels and both dense baselines."""
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=31 + Lq + Lk)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    scale = 1.0 / math.sqrt(d)
    Qd, Kd, Vd = _dev(Q), _dev(K), _dev(V)
    O = dfss.dfss_attention(Qd, Kd, Vd, s, scale)
    Os = _staged_attention(Qd, Kd, Vd, s, scale)
    Od = dfss.dense_attention(Qd, Kd, Vd, s, scale)
    Odf = dfss.dense_attention_fused(Qd, Kd, Vd, s, scale)
    torch.cuda.synchronize()
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    ref = oracle.attention(Qn, Kn, Vn, N, M, scale)
    ref_dense = oracle.attention(Qn, Kn, Vn, 1, 1, scale)
    assert np.max(np.abs(_np(O) - ref)) <= 2e-2
    assert np.max(np.abs(_np(Os) - ref)) <= 2e-2
    assert np.max(np.abs(_np(Od) - ref_dense)) <= 2e-2
    assert np.max(np.abs(_np(Odf) - ref_dense)) <= 2e-2


@pytest.mark.parametrize("variant", VARIANTS)
def test_fused_attention_rescales_when_late_keys_dominate(variant):
    """Scores that grow along the key axis force the online softmax to raise its reference
    value in later blocks; a constant key makes one block dominate every row."""
    BH, L, d = 2, 256, 64
    Q, K, V = synth.gaussian_qkv(BH, L, L, d, 1.0, seed=4242)
    ramp = torch.linspace(0.0, 6.0, L).view(1, L, 1)
    K = (K.float() + ramp * torch.sign(Q.float().mean(1, keepdim=True))).to(torch.bfloat16)
    Q = (Q.float() * 2.0).to(torch.bfloat16)
    s = Shape(1, BH, L, L, d, 2, 4)
    O = binding.internal_attention_variant(_dev(Q), _dev(K), _dev(V), None, s, 0.125, variant)
    Od = binding.internal_attention_variant(_dev(Q), _dev(K), _dev(V), None, s, 0.125, variant, dense=True)
    torch.cuda.synchronize()
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    S = np.einsum("hqd,hkd->hqk", Qn, Kn) * 0.125
    assert (S.max(-1) - S[:, :, :64].max(-1)).max() > 8.0   # the first block's maximum is outgrown
    assert np.max(np.abs(_np(O) - oracle.attention(Qn, Kn, Vn, 2, 4, 0.125))) <= 2e-2
    assert np.max(np.abs(_np(Od) - oracle.attention(Qn, Kn, Vn, 1, 1, 0.125))) <= 2e-2


def _poisoned(shape, dtype, fill):
    t = torch.empty(shape, dtype=dtype, device=DEV)
    t.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).fill_(-1 if fill else 0)
    return t


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu()


def test_results_are_deterministic_and_cover_every_byte():
    """Every output array is written in full and depends on nothing it held before: each call runs twice, on
    outputs pre-filled with 0x00 and with 0xFF bytes, and the two results must agree bit for bit.  Covers the
    stage outputs (kept scores, metadata, the softmax in place, O), O of every whole-path entry point and the
    gradients."""
    w = synth.WORKLOADS["bert_base_L384_2to4"]
    Q, K, V = (_dev(t) for t in synth.make(w))
    s = Shape(w.B, w.H, w.L, w.L, w.d, w.N, w.M)
    lengths = synth.padding_lengths(w.B, w.L, 4242)
    bias = _dev(synth.key_padding_bias(lengths, w.L))
    bm = _dev(synth.block_pattern(w.L // 64, w.L // 64, seed=5, window=1, n_global=1, n_random=1))
    Lr = 332
    sr = Shape(w.B, w.H, Lr, Lr, w.d, w.N, w.M)
    Qr, Kr, Vr = (t[:, :Lr].contiguous() for t in (Q, K, V))
    dO = _dev(synth.gaussian_qkv(w.BH, w.L, w.L, w.d, 1.0, seed=99)[0])
    gm = _dev(synth.relative_position_mask(Lr, Lr, seed=98))
    o_shape, bf = (s.BH, s.Lq, s.d), torch.bfloat16
    outs = []
    for fill in (0x00, 0xFF):
        got = {}
        vals = _poisoned((s.BH, s.Lq, s.Lc), bf, fill)
        meta = _poisoned((s.BH * s.Lq * (s.Lk // 16),), torch.bfloat16, fill).view(torch.int16)
        dfss.dfss_sddmm_prune(Q, K, s, w.scale, vals, meta)
        got["scores"], got["meta"] = _bits(vals), meta.cpu()
        dfss.dfss_sparse_softmax(vals, s)           # in place: reads what stage 1 wrote, writes every weight
        got["weights"] = _bits(vals)
        got["spmm"] = _bits(dfss.dfss_spmm(vals, meta, V, s, O=_poisoned(o_shape, bf, fill)))
        O = dfss.dfss_attention(Q, K, V, s, w.scale, O=_poisoned(o_shape, bf, fill))
        got["one kernel"] = _bits(O)
        ws = _poisoned((dfss.dfss_workspace_bytes(s) // 2,), bf, fill)
        got["staged"] = _bits(dfss.dfss_attention_staged(Q, K, V, s, w.scale, O=_poisoned(o_shape, bf, fill),
                                                         ws=ws.view(torch.uint8)))
        got["bias"] = _bits(dfss.dfss_attention_bias(Q, K, V, bias, s, w.scale, O=_poisoned(o_shape, bf, fill)))
        got["varlen"] = _bits(dfss.dfss_attention_varlen(Q, K, V, _dev(lengths.to(torch.int32)), s, w.scale,
                                                         O=_poisoned(o_shape, bf, fill)))
        got["blocked"] = _bits(dfss.dfss_attention_blocked(Q, K, V, None, bm, s, w.scale,
                                                           O=_poisoned(o_shape, bf, fill)))
        wsb = _poisoned((dfss.dfss_blocked_split_workspace_bytes(s) // 2,), bf, fill)
        got["blocked split"] = _bits(dfss.dfss_attention_blocked_split(Q, K, V, None, bm, s, w.scale,
                                                                       O=_poisoned(o_shape, bf, fill),
                                                                       ws=wsb.view(torch.uint8)))
        got["ragged"] = _bits(dfss.dfss_attention_ragged(Qr, Kr, Vr, None, sr, w.scale,
                                                         O=_poisoned((s.BH, Lr, s.d), bf, fill)))
        got["mask"] = _bits(dfss.dfss_attention_mask(Qr, Kr, Vr, gm, sr, w.scale,
                                                     O=_poisoned((s.BH, Lr, s.d), bf, fill)))
        ws = _poisoned((dfss.dfss_workspace_bytes(sr) // 2,), bf, fill)
        got["staged mask"] = _bits(dfss.dfss_attention_staged_mask(Qr, Kr, Vr, gm, sr, w.scale,
                                                                   O=_poisoned((s.BH, Lr, s.d), bf, fill),
                                                                   ws=ws.view(torch.uint8)))
        got["dense"] = _bits(dfss.dense_attention(Q, K, V, s, w.scale, O=_poisoned(o_shape, bf, fill)))
        got["dense one kernel"] = _bits(dfss.dense_attention_fused(Q, K, V, s, w.scale,
                                                                   O=_poisoned(o_shape, bf, fill)))
        dQ, dK, dV = dfss.dfss_attention_backward(dO, Q, K, V, O, vals, meta, s, w.scale,
                                                  dQ=_poisoned(o_shape, bf, fill), dK=_poisoned(o_shape, bf, fill),
                                                  dV=_poisoned(o_shape, bf, fill))
        got["dQ"], got["dK"], got["dV"] = _bits(dQ), _bits(dK), _bits(dV)
        torch.cuda.synchronize()
        outs.append(got)
    for name in outs[0]:
        assert torch.equal(outs[0][name], outs[1][name]), name


# ----------------------------------------------------------------------------------
# additive key bias (padding mask)
# ----------------------------------------------------------------------------------
def _padding_case(B, H, Lq, Lk, d, seed, integer):
    BH = B * H
    Q, K, V = (synth.integer_qkv if integer else
               (lambda *a, seed: synth.gaussian_qkv(*a, 1.0, seed=seed)))(BH, Lq, Lk, d, seed=seed)
    lengths = synth.padding_lengths(B, Lk, seed + 1)
    bias = synth.key_padding_bias(lengths, Lk)
    return Q, K, V, lengths, bias


@pytest.mark.parametrize("B,H,Lq,Lk,d,N,M,scale", [
    (3, 2, 128, 256, 64, 2, 4, 0.125),      # 32-query kernel, scale folded into Q
    (2, 3, 192, 384, 64, 2, 4, 0.125),      # 16-query kernel
    (2, 2, 128, 256, 128, 1, 2, 0.125),     # d = 128, 1:2
    (2, 2, 128, 256, 64, 2, 4, float(np.float32(1.0 / 3.0))),   # bias added after the scaling
    (2, 2, 64, 128, 64, 2, 4, float(np.float32(1.0 / 3.0))),
    (2, 2, 128, 256, 128, 2, 4, float(np.float32(1.0 / 3.0))),   # d = 128: the bias comes from global memory
    (2, 1, 192, 256, 128, 1, 2, float(np.float32(1.0 / 3.0))),
])
def test_stage1_key_bias_bit_exact_on_integer_inputs(B, H, Lq, Lk, d, N, M, scale):
    """Padding masks cut through groups (lengths are not multiples of 4): masks, metadata and kept
    values, including the -inf entries of groups with fewer than N real keys, must match exactly."""
    Q, K, _, lengths, bias = _padding_case(B, H, Lq, Lk, d, 7000 + Lq + d + N, integer=True)
    s = Shape(B, H, Lq, Lk, d, N, M)
    vals, meta = dfss.dfss_sddmm_prune_bias(_dev(Q), _dev(K), _dev(bias), s, scale)
    torch.cuda.synchronize()
    vals, meta = _np(vals), _canon_meta(meta, s)
    Qn, Kn = synth.to_numpy_f32(Q), synth.to_numpy_f32(K)
    assert int((lengths % 4 != 0).sum()) > 0
    for h in range(B * H):
        S = oracle.add_key_bias(oracle.scores(Qn[h], Kn[h], scale), bias[h // H].numpy())
        mask, v, kidx = oracle.prune(S, N, M)
        assert np.array_equal(meta[h], oracle.encode_meta(kidx, Lk)), f"metadata differs in head {h}"
        assert np.array_equal(vals[h], oracle.round_bf16(v)), f"kept values differ in head {h}"


@pytest.mark.parametrize("B,H,Lq,Lk,d,N,M", [
    (3, 2, 128, 384, 64, 2, 4),
    (2, 2, 320, 256, 64, 1, 2),
    (2, 2, 128, 256, 128, 2, 4),
    (8, 12, 384, 384, 64, 2, 4),       # the benchmark shape with a padded batch
    (2, 2, 64, 1280, 64, 2, 4),        # 20 key blocks: the bias row is scanned one block per lane
    (8, 12, 1024, 256, 64, 2, 4),      # enough query tiles for the 32-queries-per-wave variant with a bias
])
def test_attention_key_bias(B, H, Lq, Lk, d, N, M):
    """Whole path with a padding mask: fused kernel, stage kernels, both dense baselines."""
    Q, K, V, lengths, bias = _padding_case(B, H, Lq, Lk, d, 7100 + Lq + Lk + d, integer=False)
    s = Shape(B, H, Lq, Lk, d, N, M)
    scale = 1.0 / math.sqrt(d)
    Qd, Kd, Vd, bd = _dev(Q), _dev(K), _dev(V), _dev(bias)
    O = dfss.dfss_attention_bias(Qd, Kd, Vd, bd, s, scale)
    Os = dfss.dfss_attention_staged_bias(Qd, Kd, Vd, bd, s, scale)
    Od = dfss.dense_attention_bias(Qd, Kd, Vd, bd, s, scale)
    Odf = dfss.dense_attention_fused_bias(Qd, Kd, Vd, bd, s, scale)
    O0 = dfss.dfss_attention_bias(Qd, Kd, Vd, None, s, scale)      # NULL bias = the plain call
    O1 = dfss.dfss_attention(Qd, Kd, Vd, s, scale)
    torch.cuda.synchronize()
    heads = list(range(B * H)) if B * H <= 12 else [0, 13, 40, 95]
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    bn = bias.numpy()
    for h in heads:
        ref = oracle.attention(Qn[h], Kn[h], Vn[h], N, M, scale, key_bias=bn[h // H])
        ref_dense = oracle.attention(Qn[h], Kn[h], Vn[h], 1, 1, scale, key_bias=bn[h // H])
        assert np.max(np.abs(_np(O[h]) - ref)) <= 2e-2
        assert np.max(np.abs(_np(Os[h]) - ref)) <= 2e-2
        assert np.max(np.abs(_np(Od[h]) - ref_dense)) <= 2e-2
        assert np.max(np.abs(_np(Odf[h]) - ref_dense)) <= 2e-2
    assert torch.equal(O0, O1)
    # a padded sequence gives what the same sequence gives when cut at a multiple of the tile: the
    # function of the real keys only (checked on the oracle side in the CPU pins; here: finite output)
    assert torch.isfinite(O.float()).all() and torch.isfinite(Os.float()).all()


@pytest.mark.parametrize("B,H,Lq,L,d,N,M", [(4, 3, 512, 512, 64, 2, 4), (2, 2, 384, 384, 128, 1, 2),
                                             (3, 2, 192, 640, 64, 2, 4)])
def test_attention_varlen_equals_the_padding_bias(B, H, Lq, L, d, N, M):
    """A padded batch given by its lengths: against the oracle with the equivalent -inf bias, and against the
    key-bias call; junk in the padding rows of K (finite) must not matter."""
    Q, K, V, lengths, bias = _padding_case(B, H, Lq, L, d, seed=7300 + L, integer=False)
    s = Shape(B, H, Lq, L, d, N, M)
    scale = 1.0 / math.sqrt(d)
    Kj = K.clone()
    for b in range(B):
        Kj[b * H:(b + 1) * H, int(lengths[b]):] = 37.0
    lens = lengths.to(torch.int32)
    O = dfss.dfss_attention_varlen(_dev(Q), _dev(Kj), _dev(V), _dev(lens), s, scale)
    Ob = dfss.dfss_attention_bias(_dev(Q), _dev(K), _dev(V), _dev(bias), s, scale)
    torch.cuda.synchronize()
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    ref = oracle.attention(Qn, Kn, Vn, N, M, scale, key_bias=bias.numpy(), heads_per_batch=H)
    assert np.abs(_np(O) - ref).max() <= 2e-2
    assert (O.float() - Ob.float()).abs().max().item() <= 2e-2
    # lengths outside 1 .. Lk are clamped
    wild = lens.clone()
    wild[0], wild[-1] = L + 77, 0
    clamped = wild.clamp(1, L)
    Ow = dfss.dfss_attention_varlen(_dev(Q), _dev(Kj), _dev(V), _dev(wild), s, scale)
    Oc = dfss.dfss_attention_varlen(_dev(Q), _dev(Kj), _dev(V), _dev(clamped), s, scale)
    torch.cuda.synchronize()
    assert torch.equal(Ow.view(torch.int16), Oc.view(torch.int16))


def test_attention_key_bias_first_blocks_fully_masked():
    """Masked keys at the START of the sequence: whole leading 64-key blocks contribute nothing and
    the running softmax reference must not turn them into NaN."""
    B, H, L, d = 2, 2, 256, 64
    Q, K, V = synth.gaussian_qkv(B * H, L, L, d, 1.0, seed=7300)
    bias = torch.zeros((B, L), dtype=torch.float32)
    bias[0, :130] = float("-inf")
    bias[1, 64:192] = float("-inf")
    s = Shape(B, H, L, L, d, 2, 4)
    O = dfss.dfss_attention_bias(_dev(Q), _dev(K), _dev(V), _dev(bias), s, 0.125)
    Odf = dfss.dense_attention_fused_bias(_dev(Q), _dev(K), _dev(V), _dev(bias), s, 0.125)
    torch.cuda.synchronize()
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    ref = oracle.attention(Qn, Kn, Vn, 2, 4, 0.125, key_bias=bias.numpy(), heads_per_batch=H)
    ref_dense = oracle.attention(Qn, Kn, Vn, 1, 1, 0.125, key_bias=bias.numpy(), heads_per_batch=H)
    assert np.max(np.abs(_np(O) - ref)) <= 2e-2
    assert np.max(np.abs(_np(Odf) - ref_dense)) <= 2e-2


def test_attention_finite_key_bias():
    """A finite bias (not a mask) moves the selection; near-ties aside the result follows the oracle."""
    B, H, L, d = 2, 2, 256, 64
    Q, K, V = synth.gaussian_qkv(B * H, L, L, d, 1.0, seed=7400)
    g = torch.Generator().manual_seed(7401)
    bias = torch.randn(B, L, generator=g) * 1.5
    s = Shape(B, H, L, L, d, 2, 4)
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    for scale in (0.125, 0.11):     # accumulator-initial-value path and add-after-scaling path
        O = dfss.dfss_attention_bias(_dev(Q), _dev(K), _dev(V), _dev(bias), s, scale)
        torch.cuda.synchronize()
        ref = oracle.attention(Qn, Kn, Vn, 2, 4, scale, key_bias=bias.numpy(), heads_per_batch=H)
        assert np.max(np.abs(_np(O) - ref)) <= 2e-2
        plain = oracle.attention(Qn, Kn, Vn, 2, 4, scale)
        assert np.max(np.abs(plain - ref)) > 0.05       # the bias really changes the result


def test_attention_key_bias_skips_masked_blocks_anywhere():
    """Fully masked 64-key blocks are skipped by the fused kernel; masks at the start, across the
    64-block boundary of the block bitmap and at the end of the longest key sequence."""
    B, H, Lq, Lk, d = 2, 1, 64, 8192, 64
    Q, K, V = synth.gaussian_qkv(B * H, Lq, Lk, d, 1.0, seed=7500)
    bias = torch.zeros((B, Lk), dtype=torch.float32)
    bias[0, :70] = float("-inf")            # block 0 and a piece of block 1
    bias[0, 3800:4500] = float("-inf")      # blocks 60..69 (crosses block 64)
    bias[0, 6400:] = float("-inf")          # blocks 100..127
    bias[1, 64:8128] = float("-inf")        # only the first and the last block stay
    s = Shape(B, H, Lq, Lk, d, 2, 4)
    Qd, Kd, Vd, bd = _dev(Q), _dev(K), _dev(V), _dev(bias)
    O = dfss.dfss_attention_bias(Qd, Kd, Vd, bd, s, 0.125)
    Odf = dfss.dense_attention_fused_bias(Qd, Kd, Vd, bd, s, 0.125)
    torch.cuda.synchronize()
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    ref = oracle.attention(Qn, Kn, Vn, 2, 4, 0.125, key_bias=bias.numpy(), heads_per_batch=H)
    ref_dense = oracle.attention(Qn, Kn, Vn, 1, 1, 0.125, key_bias=bias.numpy(), heads_per_batch=H)
    assert np.max(np.abs(_np(O) - ref)) <= 2e-2
    assert np.max(np.abs(_np(Odf) - ref_dense)) <= 2e-2


# ----------------------------------------------------------------------------------
# hybrid block sparsity x N:M (blocked-ELL)
# ----------------------------------------------------------------------------------
@pytest.mark.parametrize("BH,Lq,Lk,d,N,M", [
    (3, 512, 512, 64, 2, 4),
    (2, 256, 640, 64, 1, 2),        # rectangular
    (2, 256, 256, 128, 2, 4),       # d = 128
    (1, 128, 8192, 64, 2, 4),       # longest key sequence: both halves of the block bitmap
])
def test_attention_blocked(BH, Lq, Lk, d, N, M):
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=8000 + Lq + Lk + d)
    small = Lk // 64 <= 4
    bm = synth.block_pattern(Lq // 64, Lk // 64, seed=8001 + Lk, window=0 if small else 1, n_random=0 if small else 3)
    assert 0 < int(bm.sum()) < bm.numel()
    s = Shape(1, BH, Lq, Lk, d, N, M)
    scale = 1.0 / math.sqrt(d)
    Qd, Kd, Vd, bmd = _dev(Q), _dev(K), _dev(V), _dev(bm)
    O = dfss.dfss_attention_blocked(Qd, Kd, Vd, None, bmd, s, scale)
    Od = dfss.dense_attention_fused_blocked(Qd, Kd, Vd, None, bmd, s, scale)
    torch.cuda.synchronize()
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    ref = oracle.attention(Qn, Kn, Vn, N, M, scale, block_mask=bm.numpy(), block_size=64)
    ref_dense = oracle.attention(Qn, Kn, Vn, 1, 1, scale, block_mask=bm.numpy(), block_size=64)
    assert np.max(np.abs(_np(O) - ref)) <= 2e-2
    assert np.max(np.abs(_np(Od) - ref_dense)) <= 2e-2
    # the calls with a workspace (long row blocks shared between workgroups): same function
    ws = torch.full((dfss.dfss_blocked_split_workspace_bytes(s),), 0xFF, dtype=torch.uint8, device=Qd.device)
    Os = dfss.dfss_attention_blocked_split(Qd, Kd, Vd, None, bmd, s, scale, ws=ws)
    Ods = dfss.dense_attention_fused_blocked_split(Qd, Kd, Vd, None, bmd, s, scale, ws=ws)
    torch.cuda.synchronize()
    assert np.max(np.abs(_np(Os) - ref)) <= 2e-2
    assert np.max(np.abs(_np(Ods) - ref_dense)) <= 2e-2
    # the pattern matters: full attention gives something else
    assert np.max(np.abs(ref - oracle.attention(Qn, Kn, Vn, N, M, scale))) > 0.05


@pytest.mark.parametrize("BH,H,L,d,N,M,scale", [
    (2, 1, 1024, 64, 2, 4, 0.125),      # key groups; the scale folds into Q
    (2, 2, 1024, 64, 1, 2, 0.11),       # the scale is applied to the scores
    (1, 1, 2048, 128, 2, 4, 0.0884),    # d = 128: no key groups, same pattern
    (1, 1, 2048, 64, 2, 4, 0.125),      # 32 key blocks
])
def test_attention_blocked_long_rows_of_every_weight(BH, H, L, d, N, M, scale):
    """At d = 64 rows of 1024 keys and more are cut into key groups inside the workgroup (every group takes every
    G-th visited block and the partial results are merged).  The pattern gives the row blocks 1, 2, 3, 4, 5, 7, 9
    and all blocks, at positions that leave some groups without any block or with one block fewer than the
    others; a key bias masks keys inside and across visited blocks."""
    nb = L // 64
    bm = torch.zeros((nb, nb), dtype=torch.uint8)
    g = torch.Generator(device="cpu")
    g.manual_seed(8200 + L + d)
    counts = [nb, 1, 2, 3, 4, 5, 7, 9]
    for i in range(nb):
        c = counts[i % len(counts)]
        bm[i, torch.randperm(nb, generator=g)[:c]] = 1
    bm[nb - 1] = 0
    bm[nb - 1, nb - 1] = 1     # only the very last block
    bm[nb - 2] = 1             # a second full row
    Q, K, V = synth.gaussian_qkv(BH, L, L, d, 1.0, seed=8201 + L + d)
    # scores that grow along the keys: later groups' references lie above earlier ones', so the merge rescales
    K = (K.float() * torch.linspace(0.5, 2.0, L)[None, :, None]).to(torch.bfloat16)
    bias = torch.zeros((BH // H, L), dtype=torch.float32)
    bias[0, 100:200] = float("-inf")         # block 1 partly, block 2 fully
    bias[-1, L - 64 * 3:L - 64] = -1.5       # finite bias in two blocks
    s = Shape(BH // H, H, L, L, d, N, M)
    Qd, Kd, Vd, bmd, bd = _dev(Q), _dev(K), _dev(V), _dev(bm), _dev(bias)
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    # a padded batch element: only keys 0 .. 99 are real, so a row block that keeps every block visits two, and the
    # workgroups that share it find one block, one block, none and none
    short = torch.zeros((BH // H, L), dtype=torch.float32)
    short[0, 100:] = float("-inf")
    for kb, kbd in ((None, None), (bias, bd), (short, _dev(short))):
        O = dfss.dfss_attention_blocked(Qd, Kd, Vd, kbd, bmd, s, scale)
        Od = dfss.dense_attention_fused_blocked(Qd, Kd, Vd, kbd, bmd, s, scale)
        torch.cuda.synchronize()
        kw = dict(block_mask=bm.numpy(), block_size=64)
        if kb is not None:
            kw.update(key_bias=kb.numpy(), heads_per_batch=H)
        ref = oracle.attention(Qn, Kn, Vn, N, M, scale, **kw)
        ref_dense = oracle.attention(Qn, Kn, Vn, 1, 1, scale, **kw)
        # rows whose every visited key is masked have no defined output: none here except via the bias in row
        # blocks that see only block 2 of batch element 0
        ok = np.isfinite(ref).all(-1)
        assert ok.mean() > (0.9 if kb is not short else 0.05)
        assert np.isfinite(_np(O)[ok]).all()
        assert np.max(np.abs(_np(O)[ok] - ref[ok])) <= 2e-2
        assert np.max(np.abs(_np(Od)[ok] - ref_dense[ok])) <= 2e-2
        # with a workspace: the row blocks of more than 16 blocks are shared between four workgroups and merged;
        # the workspace starts out as garbage (nothing in it needs initialising), twice in a row on the same one
        ws = torch.full((dfss.dfss_blocked_split_workspace_bytes(s),), 0xFF, dtype=torch.uint8, device=Qd.device)
        for _ in range(2):
            Os = dfss.dfss_attention_blocked_split(Qd, Kd, Vd, kbd, bmd, s, scale, ws=ws)
            Ods = dfss.dense_attention_fused_blocked_split(Qd, Kd, Vd, kbd, bmd, s, scale, ws=ws)
            torch.cuda.synchronize()
            assert np.isfinite(_np(Os)[ok]).all()
            assert np.max(np.abs(_np(Os)[ok] - ref[ok])) <= 2e-2
            assert np.max(np.abs(_np(Ods)[ok] - ref_dense[ok])) <= 2e-2
        # row blocks that are not shared are computed exactly as without the workspace (d = 128: the call without
        # workspace has no key groups, so it is the same kernel code)
        if kb is None and d == 128:
            light = torch.from_numpy((bm.sum(1) <= 16).numpy().repeat(64)).to(O.device)
            assert bool(light.any()) and not bool(light.all())
            assert torch.equal(Os[:, light], O[:, light])


def test_attention_blocked_with_key_bias_and_full_pattern():
    B, H, L, d = 2, 2, 384, 64
    Q, K, V, lengths, bias = _padding_case(B, H, L, L, d, 8100, integer=False)
    s = Shape(B, H, L, L, d, 2, 4)
    Qd, Kd, Vd, bd = _dev(Q), _dev(K), _dev(V), _dev(bias)
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    # block pattern and padding mask together (row blocks keep block 0, which always holds real keys)
    bm = synth.block_pattern(L // 64, L // 64, seed=8101, n_random=1)
    O = dfss.dfss_attention_blocked(Qd, Kd, Vd, bd, _dev(bm), s, 0.125)
    torch.cuda.synchronize()
    ref = oracle.attention(Qn, Kn, Vn, 2, 4, 0.125, key_bias=bias.numpy(), heads_per_batch=H,
                           block_mask=bm.numpy(), block_size=64)
    assert np.max(np.abs(_np(O) - ref)) <= 2e-2
    # a pattern that keeps every block is the unblocked call: bit for bit where both run the same kernel (with a
    # key bias), to rounding where the call without bias or pattern takes the 32-queries-per-wave kernel
    ones = torch.ones((L // 64, L // 64), dtype=torch.uint8)
    O1 = dfss.dfss_attention_blocked(Qd, Kd, Vd, bd, _dev(ones), s, 0.125)
    O2 = dfss.dfss_attention_bias(Qd, Kd, Vd, bd, s, 0.125)
    O3 = dfss.dfss_attention_blocked(Qd, Kd, Vd, None, _dev(ones), s, 0.125)
    O4 = dfss.dfss_attention(Qd, Kd, Vd, s, 0.125)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2)
    assert (O3.float() - O4.float()).abs().max().item() <= 2e-2


# ----------------------------------------------------------------------------------
# capture into a HIP graph (no allocation, no synchronisation, no host state inside the calls)
# ----------------------------------------------------------------------------------
def test_calls_replay_correctly_from_a_hip_graph():
    """Every entry point is enqueued into one graph; each replay (with eager work and
    synchronisations in between, and the inputs changed between replays) must reproduce the eager
    result of the same inputs."""
    w = synth.WORKLOADS["tiny_2to4"]
    s = Shape(2, 2, 256, 256, 64, 2, 4)
    Q, K, V = (_dev(t) for t in synth.gaussian_qkv(4, 256, 256, 64, 1.0, seed=9100))
    lengths = synth.padding_lengths(2, 256, 9101)
    bias = _dev(synth.key_padding_bias(lengths, 256))
    bm = _dev(synth.block_pattern(4, 4, seed=9102, window=0, n_random=0))
    ws = torch.empty(max(dfss.dfss_workspace_bytes(s), dfss.dense_workspace_bytes(s)), dtype=torch.uint8, device=DEV)
    wsb = torch.empty(dfss.dfss_blocked_split_workspace_bytes(s), dtype=torch.uint8, device=DEV)
    outs = {k: torch.empty_like(Q) for k in ("fused", "bias", "blocked", "blocked_split", "dense", "dense_fused", "stages",
                                             "mask", "staged_mask", "varlen")}
    lens = _dev(lengths.to(torch.int32))
    gm = _dev(synth.relative_position_mask(256, 256, seed=9103))
    vals = torch.empty((s.BH, s.Lq, s.Lc), dtype=torch.bfloat16, device=DEV)
    meta = torch.empty((s.BH * s.Lq * (s.Lk // 16),), dtype=torch.int16, device=DEV)

    def run_all():
        dfss.dfss_attention(Q, K, V, s, w.scale, O=outs["fused"], ws=ws)
        dfss.dfss_attention_bias(Q, K, V, bias, s, w.scale, O=outs["bias"], ws=ws)
        dfss.dfss_attention_blocked(Q, K, V, bias, bm, s, w.scale, O=outs["blocked"])
        dfss.dfss_attention_blocked_split(Q, K, V, bias, bm, s, w.scale, O=outs["blocked_split"], ws=wsb)
        dfss.dense_attention(Q, K, V, s, w.scale, O=outs["dense"], ws=ws)
        dfss.dense_attention_fused(Q, K, V, s, w.scale, O=outs["dense_fused"])
        dfss.dfss_attention_mask(Q, K, V, gm, s, w.scale, O=outs["mask"])
        dfss.dfss_attention_varlen(Q, K, V, lens, s, w.scale, O=outs["varlen"])
        dfss.dfss_attention_staged_mask(Q, K, V, gm, s, w.scale, O=outs["staged_mask"], ws=ws)
        dfss.dfss_sddmm_prune(Q, K, s, w.scale, vals=vals, meta=meta)
        dfss.dfss_sparse_softmax(vals, s)
        dfss.dfss_spmm(vals, meta, V, s, O=outs["stages"])

    run_all()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    for rep in range(3):
        Q.copy_((torch.randn(Q.shape, generator=torch.Generator().manual_seed(9200 + rep))).to(torch.bfloat16))
        run_all()                                   # eager reference on the new inputs
        torch.cuda.synchronize()
        eager = {k: v.clone() for k, v in outs.items()}
        for v in outs.values():
            v.zero_()
        g.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(outs[k], eager[k]), (rep, k)
