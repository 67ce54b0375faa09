"""The causal mask on the GPU against the CPU oracle, through the C ABI (needs an MI355X).

Query i sees keys 0 .. i + (Lk - Lq); hidden scores count as -inf before the N:M selection.
  * stage 1 bit-exact on integer inputs: metadata and kept values, the -inf entries of runs that the diagonal cuts
    and of runs that are hidden entirely included;
  * the weight matrix of the one-kernel path and of the two-kernel path, read out through identity blocks of V:
    a hidden key must weigh exactly 0;
  * O of every causal entry point within 2e-2 of the oracle on Gaussian inputs, with and without a padding mask on top;
  * the error paths.
"""
import ctypes
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2203_00091_amd as dfss
from paper_2203_00091_amd import Shape, binding, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _dev(t):
    return t.to(DEV).contiguous()


def _np(t):
    return t.detach().to("cpu", torch.float32).numpy()


@pytest.mark.parametrize("B,H,Lq,Lk,d,N,M,scale,with_bias", [
    (1, 2, 256, 256, 64, 2, 4, 0.125, False),      # square, 32-queries-per-wave stage 1
    (1, 2, 192, 384, 64, 2, 4, 0.125, False),      # 16-queries-per-wave stage 1, more keys than queries
    (1, 2, 128, 384, 128, 1, 2, 0.125, False),     # d = 128, 1:2, the diagonal starts in the third block
    (2, 1, 256, 256, 64, 2, 4, float(np.float32(1.0 / 3.0)), False),   # scale applied after the product
    (2, 2, 128, 256, 64, 2, 4, 0.125, True),       # padding mask on top
    (2, 1, 192, 256, 64, 1, 2, float(np.float32(1.0 / 3.0)), True),
])
def test_stage1_causal_bit_exact_on_integer_inputs(B, H, Lq, Lk, d, N, M, scale, with_bias):
    BH = B * H
    Q, K, _ = synth.integer_qkv(BH, Lq, Lk, d, seed=9000 + Lq + Lk + d + N)
    s = Shape(B, H, Lq, Lk, d, N, M)
    bias = synth.key_padding_bias(synth.padding_lengths(B, Lk, 9001), Lk) if with_bias else None
    vals, meta = dfss.dfss_sddmm_prune_causal(_dev(Q), _dev(K), None if bias is None else _dev(bias), s, scale)
    canon = dfss.dfss_meta_to_canonical(meta, s)
    torch.cuda.synchronize()
    vals, canon = _np(vals), canon.cpu().numpy().view(np.uint16)
    Qn, Kn = synth.to_numpy_f32(Q), synth.to_numpy_f32(K)
    cm = oracle.causal_mask(Lq, Lk)
    hidden_runs = 0
    for h in range(BH):
        S = oracle.scores(Qn[h], Kn[h], scale)
        if bias is not None:
            S = oracle.add_key_bias(S, bias[h // H].numpy())
        S = oracle.add_mask(S, cm)
        _, v, kidx = oracle.prune(S, N, M)
        assert np.array_equal(canon[h], oracle.encode_meta(kidx, Lk)), f"metadata differs in head {h}"
        assert np.array_equal(vals[h], oracle.round_bf16(v)), f"kept values differ in head {h}"
        hidden_runs += int(np.isneginf(S.reshape(Lq, Lk // M, M)).all(-1).sum())
    assert hidden_runs > 0


def _weights(run, BH, Lq, Lk, d):
    out = np.empty((BH, Lq, Lk), np.float32)
    eye = torch.eye(d, dtype=torch.bfloat16, device=DEV)
    for j0 in range(0, Lk, d):
        V = torch.zeros((BH, Lk, d), dtype=torch.bfloat16, device=DEV)
        V[:, j0:j0 + d, :] = eye
        O = run(V)
        torch.cuda.synchronize()
        out[:, :, j0:j0 + d] = _np(O)
    return out


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M", [
    (2, 256, 256, 64, 2, 4),
    (2, 128, 384, 64, 1, 2),
    (1, 256, 256, 128, 2, 4),
    (12, 1024, 1024, 64, 2, 4),      # enough workgroups for two query tiles per wave
])
def test_causal_weight_matrix(BH, Lq, Lk, d, N, M):
    """O with V = identity on d consecutive keys IS the weight of those keys: hidden keys must weigh exactly 0,
    kept visible keys carry the oracle's weight, dropped keys 0."""
    Q, K, _ = synth.integer_qkv(BH, Lq, Lk, d, seed=9100 + Lk + d + N)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    Qd, Kd = _dev(Q), _dev(K)
    heads = range(BH) if BH <= 2 else (0, BH - 1)
    Qn, Kn = synth.to_numpy_f32(Q), synth.to_numpy_f32(K)
    cm = oracle.causal_mask(Lq, Lk)
    # the two-kernel path stores the kept scores as bfloat16 between its kernels (the method's 2-byte compressed
    # matrix): its weights are the softmax of the ROUNDED scores; the one-kernel path keeps them in fp32
    ref = {"one kernel": {}, "two kernels": {}}
    for h in heads:
        S = oracle.add_mask(oracle.scores(Qn[h], Kn[h], 0.125), cm)
        _, v, kidx = oracle.prune(S, N, M)
        for name, kept_scores in (("one kernel", v), ("two kernels", oracle.round_bf16(v))):
            W = np.zeros((Lq, Lk))
            np.put_along_axis(W, kidx.astype(np.int64), oracle.softmax_kept(kept_scores).astype(np.float64), axis=1)
            ref[name][h] = W
    for name, run in (("one kernel", lambda V: dfss.dfss_attention_causal(Qd, Kd, V, None, s, 0.125)),
                      ("two kernels", lambda V: dfss.dfss_attention_staged_causal(Qd, Kd, V, None, s, 0.125))):
        if name == "two kernels" and BH > 2:
            continue
        got = _weights(run, BH, Lq, Lk, d)
        for h in heads:
            W = ref[name][h]
            g = got[h].astype(np.float64)
            assert np.abs(g[W == 0]).max(initial=0.0) == 0.0, f"{name}: a hidden or dropped key carries weight (head {h})"
            assert (np.abs(g - W) <= 2.0 ** -6 * W + 1e-6).all(), f"{name}: weight off by {np.abs(g - W).max():.3e}"


@pytest.mark.parametrize("B,H,Lq,Lk,d,N,M,with_bias", [
    (2, 2, 256, 256, 64, 2, 4, False),
    (2, 2, 192, 384, 64, 1, 2, False),
    (1, 2, 128, 256, 128, 2, 4, True),
    (1, 24, 2048, 2048, 64, 2, 4, False),     # long rows: two query tiles per wave, many skipped blocks
])
def test_causal_attention_against_oracle(B, H, Lq, Lk, d, N, M, with_bias):
    BH = B * H
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=9200 + Lq + Lk + d)
    s = Shape(B, H, Lq, Lk, d, N, M)
    scale = 1.0 / math.sqrt(d)
    bias = synth.key_padding_bias(synth.padding_lengths(B, Lk, 9201), Lk) if with_bias else None
    Qd, Kd, Vd = _dev(Q), _dev(K), _dev(V)
    bd = None if bias is None else _dev(bias)
    O = dfss.dfss_attention_causal(Qd, Kd, Vd, bd, s, scale)
    Os = dfss.dfss_attention_staged_causal(Qd, Kd, Vd, bd, s, scale)
    Od = dfss.dense_attention_causal(Qd, Kd, Vd, bd, s, scale)
    Odf = dfss.dense_attention_fused_causal(Qd, Kd, Vd, bd, s, scale)
    torch.cuda.synchronize()
    heads = list(range(BH)) if BH <= 4 else [0, BH // 2, BH - 1]
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    for h in heads:
        kb = None if bias is None else bias[h // H].numpy()
        ref = oracle.attention(Qn[h], Kn[h], Vn[h], N, M, scale, key_bias=kb, causal=True)
        ref_dense = oracle.attention(Qn[h], Kn[h], Vn[h], 1, 1, scale, key_bias=kb, causal=True)
        assert np.max(np.abs(_np(O[h]) - ref)) <= 2e-2
        assert np.max(np.abs(_np(Os[h]) - ref)) <= 2e-2
        assert np.max(np.abs(_np(Od[h]) - ref_dense)) <= 2e-2
        assert np.max(np.abs(_np(Odf[h]) - ref_dense)) <= 2e-2
    for t in (O, Os, Od, Odf):
        assert torch.isfinite(t.float()).all()
    # the first query of a square problem sees key 0 only: its output is V[0]
    if Lq == Lk and bias is None:
        assert np.max(np.abs(_np(O[:, 0]) - _np(V[:, 0]))) <= 1e-2


def test_causal_error_paths():
    lib = binding.load_library()
    x = torch.zeros(1 << 16, dtype=torch.bfloat16, device=DEV)
    p = ctypes.c_void_p(x.data_ptr())
    more_queries = Shape(1, 1, 256, 128, 64, 2, 4)
    assert lib.dfss_attention_causal(p, p, p, None, ctypes.byref(more_queries.c()), 0.125, p, None) == 2   # shape
    assert lib.dfss_sddmm_prune_causal(p, p, None, ctypes.byref(more_queries.c()), 0.125, p, p, None) == 2
    f32 = Shape(1, 1, 128, 128, 64, 1, 2, dfss.DFSS_F32_BF16X3)
    assert lib.dfss_attention_causal(p, p, p, None, ctypes.byref(f32.c()), 0.125, p, None) == 3            # unsupported
    ok = Shape(1, 1, 128, 128, 64, 2, 4)
    assert lib.dfss_attention_causal(None, p, p, None, ctypes.byref(ok.c()), 0.125, p, None) == 1           # null
