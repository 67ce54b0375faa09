"""The general additive mask [Lq, Lk] of the stage calls on the GPU against the CPU oracle, through the C ABI
(needs an MI355X).  mask[i][j] is added to the scaled score before the N:M selection; -inf hides a key from a query.
  * stage 1 bit-exact on integer inputs with a mask of quarter-integers and -inf entries, tile multiples and
    unpadded lengths, both scale paths;
  * the special cases: a causal mask gives the causal call's kept values and metadata bit for bit, a mask whose rows
    all equal a key bias gives the key-bias call's;
  * O of the staged call, of the one-kernel calls (dfss_attention_mask, dense_attention_fused_mask) and of the
    three-kernel baseline within 2e-2 of the oracle on Gaussian inputs (the one-kernel call's selection is checked
    weight by weight in test_gpu_fused_weights.py).
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


def _mask(Lq, Lk, seed):
    """Quarter-integer terms on a third of the entries, -inf on a sixth, whole runs of four hidden here and there;
    every query keeps key 0."""
    g = torch.Generator().manual_seed(seed)
    m = torch.zeros((Lq, Lk), dtype=torch.float32)
    r = torch.rand((Lq, Lk), generator=g)
    m[r < 1 / 3] = (torch.randint(-8, 9, (Lq, Lk), generator=g).float() / 4)[r < 1 / 3]
    m[r > 5 / 6] = float("-inf")
    runs = torch.rand((Lq, Lk // 4), generator=g) < 0.1
    m[runs.repeat_interleave(4, dim=1)] = float("-inf")
    m[:, 0] = 0.0
    return m


def _canon(meta, s):
    return dfss.dfss_meta_to_canonical(meta, s).cpu().numpy().view(np.uint16).reshape(s.BH, s.LqP, s.meta_words)


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M,scale", [
    (2, 256, 384, 64, 2, 4, 0.125),                               # the mask is the initial value of the accumulators
    (2, 128, 256, 64, 1, 2, float(np.float32(1.0 / 3.0))),        # the mask is added after the scaling
    (2, 128, 256, 128, 2, 4, 0.125),                              # d = 128
    (2, 192, 128, 64, 2, 4, 0.125),                               # Lq = 64 mod 128: half a workgroup stores nothing
    (2, 100, 132, 64, 2, 4, 0.125),                               # unpadded lengths
    (1, 250, 516, 128, 1, 2, 0.25),
])
def test_stage1_mask_bit_exact_on_integer_inputs(BH, Lq, Lk, d, N, M, scale):
    Q, K, _ = synth.integer_qkv(BH, Lq, Lk, d, seed=9900 + Lq + Lk)
    mask = _mask(Lq, Lk, 9901 + Lq)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    vals, meta = dfss.dfss_sddmm_prune_mask(_dev(Q), _dev(K), _dev(mask), s, scale)
    torch.cuda.synchronize()
    v, mc = vals.float().cpu().numpy(), _canon(meta, s)
    Qn, Kn = synth.to_numpy_f32(Q), synth.to_numpy_f32(K)
    for h in range(BH):
        S = oracle.add_mask(oracle.scores(Qn[h], Kn[h], scale), mask.numpy())
        Sp = np.full((Lq, s.LkP), -np.inf, dtype=np.float32)
        Sp[:, :Lk] = S
        _, vref, kidx = oracle.prune(Sp, N, M)
        assert np.array_equal(mc[h, :Lq], oracle.encode_meta(kidx, s.LkP)), f"metadata differs in head {h}"
        assert np.array_equal(v[h, :Lq], oracle.round_bf16(vref)), f"kept scores differ in head {h}"


def test_mask_special_cases_equal_the_dedicated_calls():
    BH, Lq, Lk, d = 3, 256, 384, 64
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=9910)
    s = Shape(1, BH, Lq, Lk, d, 2, 4)
    Qd, Kd, Vd = _dev(Q), _dev(K), _dev(V)
    for scale in (0.125, float(np.float32(1.0 / 3.0))):
        # causal
        cm = torch.from_numpy(oracle.causal_mask(Lq, Lk))
        v1, m1 = dfss.dfss_sddmm_prune_mask(Qd, Kd, _dev(cm), s, scale)
        v2, m2 = dfss.dfss_sddmm_prune_causal(Qd, Kd, None, s, scale)
        O1 = dfss.dfss_attention_staged_mask(Qd, Kd, Vd, _dev(cm), s, scale)
        O2 = dfss.dfss_attention_staged_causal(Qd, Kd, Vd, None, s, scale)
        torch.cuda.synchronize()
        assert torch.equal(v1.view(torch.int16), v2.view(torch.int16)) and torch.equal(m1, m2)
        assert torch.equal(O1.view(torch.int16), O2.view(torch.int16))
        # key bias (one batch element): every row of the mask is the bias
        bias = synth.key_padding_bias(synth.padding_lengths(1, Lk, 9911), Lk)
        bias[0, 3:40:5] = -0.75
        bm = bias.expand(Lq, Lk).contiguous()
        v1, m1 = dfss.dfss_sddmm_prune_mask(Qd, Kd, _dev(bm), s, scale)
        v2, m2 = dfss.dfss_sddmm_prune_bias(Qd, Kd, _dev(bias), s, scale)
        torch.cuda.synchronize()
        assert torch.equal(v1.view(torch.int16), v2.view(torch.int16)) and torch.equal(m1, m2)


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M", [
    (2, 256, 512, 64, 2, 4),
    (2, 128, 384, 128, 1, 2),
    (2, 300, 1000, 64, 2, 4),      # unpadded lengths
])
def test_attention_with_a_mask(BH, Lq, Lk, d, N, M):
    Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=9920 + Lq)
    # a relative-position term (finite everywhere) plus a band of hidden keys per query
    i, j = torch.arange(Lq)[:, None], torch.arange(Lk)[None, :]
    mask = -0.01 * (i * Lk // Lq - j).abs().float()
    mask[(j > i * Lk // Lq + 64) & (j % 7 != 0)] = float("-inf")
    mask[:, 0] = 0.0
    s = Shape(1, BH, Lq, Lk, d, N, M)
    scale = 1.0 / math.sqrt(d)
    Qd, Kd, Vd, md = _dev(Q), _dev(K), _dev(V), _dev(mask)
    O = dfss.dfss_attention_staged_mask(Qd, Kd, Vd, md, s, scale)
    Od = dfss.dense_attention_mask(Qd, Kd, Vd, md, s, scale)
    vals, meta = dfss.dfss_sddmm_prune_mask(Qd, Kd, md, s, scale)
    dfss.dfss_sparse_softmax(vals, s)
    O3 = dfss.dfss_spmm(vals, meta, Vd, s)
    O1 = dfss.dfss_attention_mask(Qd, Kd, Vd, md, s, scale)
    O1p = dfss.dfss_attention_mask(Qd, Kd, Vd, md, s, 0.125)       # a power of two: the other scale path
    Od1 = dfss.dense_attention_fused_mask(Qd, Kd, Vd, md, s, scale)
    torch.cuda.synchronize()
    Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
    ref = oracle.attention(Qn, Kn, Vn, N, M, scale, mask=mask.numpy())
    refd = oracle.attention(Qn, Kn, Vn, 1, 1, scale, mask=mask.numpy())
    assert np.abs(ref - oracle.attention(Qn, Kn, Vn, N, M, scale)).max() > 0.05      # the mask matters
    refp = oracle.attention(Qn, Kn, Vn, N, M, 0.125, mask=mask.numpy())
    for name, got, r in (("staged", O, ref), ("three stages", O3, ref), ("dense", Od, refd), ("one kernel", O1, ref),
                         ("one kernel, scale 1/8", O1p, refp), ("dense, one kernel", Od1, refd)):
        got = _np(got)
        assert np.isfinite(got).all(), name
        assert np.abs(got - r).max() <= 2e-2, name


def test_one_kernel_mask_special_cases():
    """A causal mask gives the causal call's result, a zero mask the plain call's (to the rounding of different
    tilings); unpadded lengths included."""
    for BH, Lq, Lk, d in ((3, 256, 384, 64), (2, 200, 328, 128)):
        Q, K, V = synth.gaussian_qkv(BH, Lq, Lk, d, 1.0, seed=9930 + Lq)
        s = Shape(1, BH, Lq, Lk, d, 2, 4)
        Qd, Kd, Vd = _dev(Q), _dev(K), _dev(V)
        scale = 1.0 / math.sqrt(d)
        cm = torch.from_numpy(oracle.causal_mask(Lq, Lk))
        O1 = dfss.dfss_attention_mask(Qd, Kd, Vd, _dev(cm), s, scale)
        O2 = dfss.dfss_attention_staged_causal(Qd, Kd, Vd, None, s, scale) if Lq % 64 == 0 else O1
        O3 = dfss.dfss_attention_mask(Qd, Kd, Vd, torch.zeros((Lq, Lk), device=DEV), s, scale)
        O4 = dfss.dfss_attention_ragged(Qd, Kd, Vd, None, s, scale)
        torch.cuda.synchronize()
        assert (O1.float() - O2.float()).abs().max().item() <= 2e-2
        assert (O3.float() - O4.float()).abs().max().item() <= 2e-2
        Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Q, K, V))
        ref = oracle.attention(Qn, Kn, Vn, 2, 4, scale, mask=cm.numpy())
        assert np.abs(_np(O1) - ref).max() <= 2e-2


def test_mask_calls_refuse_what_they_cannot_run():
    s = Shape(1, 1, 128, 128, 64, 1, 2, dfss.DFSS_F32_BF16X3)
    Q = torch.zeros(1, 128, 64, device=DEV)
    with pytest.raises(dfss.DfssError):       # 2-byte dtype only
        dfss.dfss_attention_staged_mask(Q, Q, Q, torch.zeros(128, 128, device=DEV), s, 0.125)
    with pytest.raises(dfss.DfssError):
        dfss.dfss_attention_mask(Q, Q, Q, torch.zeros(128, 128, device=DEV), s, 0.125)
    s2 = Shape(1, 1, 128, 128, 64)
    with pytest.raises(ValueError):           # the mask is [Lq, Lk]
        dfss.dfss_sddmm_prune_mask(Q.bfloat16(), Q.bfloat16(), torch.zeros(128, 64, device=DEV), s2, 0.125)
    torch.cuda.synchronize()
