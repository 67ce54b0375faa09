"""Element-wise check of the one-kernel paths (needs an MI355X).

The one-kernel forward pass writes neither kept scores nor metadata, so its selection cannot be read
back directly.  It can be made visible: with V = the identity on d consecutive keys j0 .. j0+d-1 and zero
elsewhere, O[i, c] IS the softmax weight of key j0 + c in row i.  Sweeping j0 over the key axis shows the
whole weight matrix, which is compared with the oracle entry by entry:

  * a key the oracle drops must have weight exactly 0 (a wrong pick, or two swapped position codes inside a
    run of four, puts a weight on a dropped key);
  * a kept key must carry the oracle's weight up to the bfloat16 roundings of weight, row sum and output.

Q and K hold small integers, so every score is exact in fp32 on both sides and equal scores (ties) abound:
the selection must then agree with the oracle's rank rule exactly, ties included.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2203_00091_amd as dfss
from paper_2203_00091_amd import DFSS_BF16, DFSS_F32_BF16X3, Shape, binding, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
# Three bfloat16 roundings stack up in a weight: the weight itself, the dominant weight of its row (through the
# row sum) and the output.  Each is at most 2^-8 relative (half the spacing at the bottom of a binade):
# 3 * 2^-8 in the worst case, so 2^-6.  A wrong pick is off by 100 %.
REL, ABS = 2.0 ** -6, 1e-6


def _dense_weights(Qn, Kn, N, M, scale, key_bias=None, block_mask=None, mask=None):
    """The oracle's weight matrix of one head, dense [Lq, Lk] (0 at dropped keys), and the kept mask."""
    S = oracle.scores(Qn, Kn, scale)
    if key_bias is not None:
        S = oracle.add_key_bias(S, key_bias)
    if mask is not None:
        S = oracle.add_mask(S, mask)
    if block_mask is not None:
        S = oracle.apply_block_mask(S, block_mask, 64)
    mask, vals, kidx = oracle.prune(S, N, M)
    P = oracle.softmax_kept(vals)
    W = np.zeros(S.shape, np.float64)
    np.put_along_axis(W, kidx.astype(np.int64), P.astype(np.float64), axis=1)
    kept = np.zeros(S.shape, bool)
    np.put_along_axis(kept, kidx.astype(np.int64), True, axis=1)
    assert kept.sum() == kidx.size and np.array_equal(kept, mask.astype(bool))
    return W, kept, S


def _weights_through_identity_v(run, BH, Lq, Lk, d, tdtype):
    """Run `run(V)` once per block of d keys with V = identity on that block; returns [BH, Lq, Lk] weights."""
    out = np.empty((BH, Lq, Lk), np.float32)
    eye = torch.eye(d, dtype=tdtype, device=DEV)
    for j0 in range(0, Lk, d):
        V = torch.zeros((BH, Lk, d), dtype=tdtype, device=DEV)
        n = min(d, Lk - j0)
        V[:, j0:j0 + n, :] = eye[:n]
        O = run(V)
        torch.cuda.synchronize()
        out[:, :, j0:j0 + n] = O.float().cpu().numpy()[:, :, :n]
    return out


def _compare(Wgpu, Qn, Kn, N, M, scale, key_bias=None, H=1, block_mask=None, rel=REL, mask=None):
    ties = 0
    for h in range(Qn.shape[0]):
        kb = None if key_bias is None else key_bias[h // H]
        W, kept, S = _dense_weights(Qn[h], Kn[h], N, M, scale, kb, block_mask, mask)
        got = Wgpu[h].astype(np.float64)
        dropped_weight = np.abs(got[~kept])
        assert dropped_weight.max(initial=0.0) == 0.0, \
            f"head {h}: {int((dropped_weight > 0).sum())} dropped keys carry weight (largest {dropped_weight.max():.3e})"
        err = np.abs(got - W)
        assert (err <= rel * W + ABS).all(), f"head {h}: weight off by {err.max():.3e}"
        G = S.reshape(S.shape[0], -1, M)
        srt = np.sort(G, axis=-1)
        ties += int((srt[..., M - N] == srt[..., M - N - 1]).sum())   # N-th and (N+1)-th largest equal
    return ties


def _int_qk(BH, Lq, Lk, d, seed, tdtype=torch.bfloat16):
    Q, K, _ = synth.integer_qkv(BH, Lq, Lk, d, seed=seed, dtype=tdtype)
    return Q, K, synth.to_numpy_f32(Q), synth.to_numpy_f32(K)


VARIANTS = [binding.VARIANT_Q16, binding.VARIANT_Q16X2, binding.VARIANT_Q32W2, binding.VARIANT_Q32W4,
            binding.VARIANT_Q32K2]


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("BH,Lq,Lk,d,N,M,scale", [
    (2, 128, 512, 64, 2, 4, 0.125),
    (2, 128, 384, 64, 1, 2, 0.125),
    (1, 128, 512, 128, 2, 4, 0.125),
    (1, 256, 256, 128, 1, 2, float(np.float32(1.0 / math.sqrt(128.0)))),   # scale that is not a power of two
    (2, 256, 384, 64, 2, 4, float(np.float32(1.0 / 3.0))),
])
def test_every_tiling_selects_and_weighs_like_the_oracle(variant, BH, Lq, Lk, d, N, M, scale):
    Q, K, Qn, Kn = _int_qk(BH, Lq, Lk, d, seed=8100 + Lk + d + N)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    Qd, Kd = Q.to(DEV), K.to(DEV)
    W = _weights_through_identity_v(
        lambda V: binding.internal_attention_variant(Qd, Kd, V, None, s, scale, variant), BH, Lq, Lk, d, torch.bfloat16)
    ties = _compare(W, Qn, Kn, N, M, scale)
    assert ties > 100          # the tie rule was exercised


@pytest.mark.parametrize("variant", VARIANTS)
def test_weights_when_late_keys_raise_the_reference(variant):
    """Scores that grow along the key axis: the running reference of the softmax is raised in later blocks
    (the partial sums are rescaled, the block's scores re-centred) and the selection must not notice."""
    BH, L, d = 2, 384, 64
    Q, K, Qn, Kn = _int_qk(BH, L, L, d, seed=8242)
    ramp = (torch.arange(L) // 24).view(1, L, 1).float()                       # 0 .. 15 in steps
    K = (K.float() + ramp * torch.sign(Q.float().sum(1, keepdim=True))).to(torch.bfloat16)   # still integers
    Kn = synth.to_numpy_f32(K)
    s = Shape(1, BH, L, L, d, 2, 4)
    S = np.einsum("hqd,hkd->hqk", Qn, Kn) * 0.125
    assert (S.max(-1) - S[:, :, :64].max(-1)).max() > 16.0      # far above what the first block saw
    Qd, Kd = Q.to(DEV), K.to(DEV)
    W = _weights_through_identity_v(
        lambda V: binding.internal_attention_variant(Qd, Kd, V, None, s, 0.125, variant), BH, L, L, d, torch.bfloat16)
    _compare(W, Qn, Kn, 2, 4, 0.125)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 2)])
def test_default_call_ragged_call_and_blocked_call(N, M):
    """The public one-kernel entry points: dfss_attention (whatever tiling it picks), dfss_attention_bias with
    a padding mask, dfss_attention_ragged on lengths that are no tile multiples, dfss_attention_blocked."""
    B, H, Lq, Lk, d = 2, 2, 192, 384, 64
    BH = B * H
    Q, K, Qn, Kn = _int_qk(BH, Lq, Lk, d, seed=8300 + N)
    s = Shape(B, H, Lq, Lk, d, N, M)
    Qd, Kd = Q.to(DEV), K.to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention(Qd, Kd, V, s, 0.125), BH, Lq, Lk, d, torch.bfloat16)
    _compare(W, Qn, Kn, N, M, 0.125)
    # the two-kernel path (stage 1, then the product that applies the softmax on the way); 192 queries take the
    # 16-queries-per-wave stage 1, 128 of them the 32-queries-per-wave one
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_staged(Qd, Kd, V, s, 0.125), BH, Lq, Lk, d,
                                    torch.bfloat16)
    _compare(W, Qn, Kn, N, M, 0.125)
    s128 = Shape(B, H, 128, Lk, d, N, M)
    Q128 = Q[:, :128].contiguous().to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_staged(Q128, Kd, V, s128, 0.125), BH, 128, Lk, d,
                                    torch.bfloat16)
    _compare(W, Qn[:, :128], Kn, N, M, 0.125)
    # padding mask whose ends cut through runs of four
    lengths = torch.tensor([Lk, 203])
    bias = synth.key_padding_bias(lengths, Lk)
    bd = bias.to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_bias(Qd, Kd, V, bd, s, 0.125), BH, Lq, Lk, d,
                                    torch.bfloat16)
    _compare(W, Qn, Kn, N, M, 0.125, key_bias=bias.numpy(), H=H)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_staged_bias(Qd, Kd, V, bd, s, 0.125), BH, Lq, Lk, d,
                                    torch.bfloat16)
    _compare(W, Qn, Kn, N, M, 0.125, key_bias=bias.numpy(), H=H)
    # unpadded lengths: 100 queries, 332 keys
    Lqr, Lkr = 100, 332
    sr = Shape(B, H, Lqr, Lkr, d, N, M)
    Qr, Kr = Q[:, :Lqr].contiguous().to(DEV), K[:, :Lkr].contiguous().to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_ragged(Qr, Kr, V, None, sr, 0.125), BH, Lqr, Lkr, d,
                                    torch.bfloat16)
    _compare(W, Qn[:, :Lqr], Kn[:, :Lkr], N, M, 0.125)
    # block pattern (window + global + random blocks)
    bm = synth.block_pattern(Lq // 64, Lk // 64, seed=77, window=1, n_global=1, n_random=1)
    bmd = bm.to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_blocked(Qd, Kd, V, None, bmd, s, 0.125), BH, Lq, Lk, d,
                                    torch.bfloat16)
    _compare(W, Qn, Kn, N, M, 0.125, block_mask=bm.numpy())


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M,scale", [
    (2, 128, 384, 64, 2, 4, 0.125),                              # the mask is the initial value of the accumulators
    (2, 192, 256, 64, 1, 2, float(np.float32(1.0 / 3.0))),       # the mask is added after the scaling
    (1, 128, 256, 128, 2, 4, 0.125),
    (2, 100, 332, 64, 2, 4, 0.125),                              # unpadded lengths
    (1, 70, 140, 128, 1, 2, float(np.float32(1.0 / 3.0))),
    (96, 1024, 192, 64, 2, 4, 0.125),                            # many heads and row blocks: several launch tiles
    (96, 1000, 132, 64, 1, 2, float(np.float32(1.0 / 3.0))),     # the same on unpadded lengths
])
def test_general_mask_in_the_one_kernel_call(BH, Lq, Lk, d, N, M, scale):
    """dfss_attention_mask: quarter-integer terms and -inf entries (whole runs of four and whole 64-key blocks of a
    query hidden); with integer Q, K every biased score is exact on both sides, so the selection must agree with the
    oracle's, ties included."""
    Q, K, Qn, Kn = _int_qk(BH, Lq, Lk, d, seed=8500 + Lq + Lk)
    g = torch.Generator().manual_seed(8501 + Lq)
    mask = torch.zeros((Lq, Lk), dtype=torch.float32)
    r = torch.rand((Lq, Lk), generator=g)
    mask[r < 1 / 3] = (torch.randint(-8, 9, (Lq, Lk), generator=g).float() / 4)[r < 1 / 3]
    mask[r > 5 / 6] = float("-inf")
    mask[(torch.rand((Lq, Lk // 4), generator=g) < 0.1).repeat_interleave(4, dim=1)] = float("-inf")
    mask[Lq // 2:, :64] = float("-inf")            # the first block hidden from half of the queries
    mask[: Lq // 3, 64:128] = float("-inf")        # the second from a third
    mask[:, 130] = 0.0                             # every query sees a key
    s = Shape(1, BH, Lq, Lk, d, N, M)
    Qd, Kd, md = Q.to(DEV), K.to(DEV), mask.to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_mask(Qd, Kd, V, md, s, scale), BH, Lq, Lk, d,
                                    torch.bfloat16)
    ties = _compare(W, Qn, Kn, N, M, scale, mask=mask.numpy())
    assert ties > 100
    # the baseline: nothing is dropped
    W = _weights_through_identity_v(lambda V: dfss.dense_attention_fused_mask(Qd, Kd, V, md, s, scale), BH, Lq, Lk, d,
                                    torch.bfloat16)
    for h in range(BH):
        S = oracle.add_mask(oracle.scores(Qn[h], Kn[h], scale), mask.numpy()).astype(np.float64)
        P = np.exp(S - S.max(-1, keepdims=True))
        P /= P.sum(-1, keepdims=True)
        assert (np.abs(W[h] - P) <= REL * P + ABS).all()


@pytest.mark.parametrize("B,H,Lq,Lk,d,N,M,scale,lengths", [
    (3, 2, 128, 384, 64, 2, 4, 0.125, (384, 203, 1)),                       # 128-query workgroups; one key only
    (2, 2, 192, 256, 64, 1, 2, float(np.float32(1.0 / 3.0)), (64, 130)),    # 64-query workgroups; an end on a block edge
    (2, 1, 128, 256, 128, 2, 4, 0.125, (255, 66)),
])
def test_padded_batch_given_by_its_lengths(B, H, Lq, Lk, d, N, M, scale, lengths):
    """dfss_attention_varlen: the padding keys must carry weight exactly 0 and the selection among the real keys (runs
    of four that the end of a sequence cuts included) must be the oracle's with the equivalent -inf bias."""
    BH = B * H
    Q, K, Qn, Kn = _int_qk(BH, Lq, Lk, d, seed=8600 + Lk + d)
    s = Shape(B, H, Lq, Lk, d, N, M)
    lens = torch.tensor(lengths, dtype=torch.int32)
    bias = synth.key_padding_bias(lens, Lk)
    Qd, Kd, ld = Q.to(DEV), K.to(DEV), lens.to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_varlen(Qd, Kd, V, ld, s, scale), BH, Lq, Lk, d,
                                    torch.bfloat16)
    _compare(W, Qn, Kn, N, M, scale, key_bias=bias.numpy(), H=H)
    for b in range(B):
        assert (W[b * H:(b + 1) * H, :, lengths[b]:] == 0).all()


def test_ragged_call_on_a_grid_that_fills_the_chip():
    """dfss_attention_ragged on many heads runs the 32-queries-per-wave kernel: weight by weight, with a last
    query tile of 8 rows and a last key block of 4 keys."""
    BH, Lq, Lk, d, N, M = 64, 904, 260, 64, 2, 4
    Q, K, Qn, Kn = _int_qk(BH, Lq, Lk, d, seed=8700)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    Qd, Kd = Q.to(DEV), K.to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention_ragged(Qd, Kd, V, None, s, 0.125), BH, Lq, Lk, d,
                                    torch.bfloat16)
    ties = _compare(W[::8], Qn[::8], Kn[::8], N, M, 0.125)
    assert ties > 100


@pytest.mark.parametrize("BH,Lq,Lk,d,N,M,scale", [
    (200, 192, 256, 64, 2, 4, 0.125),
    (200, 192, 128, 128, 1, 2, 0.0625),
])
def test_default_call_with_half_a_workgroup_left_over_on_a_large_grid(BH, Lq, Lk, d, N, M, scale):
    """Lq an odd multiple of 64 on more than 384 workgroups: dfss_attention runs 128-query workgroups whose last
    one per head is half empty.  Weight by weight against the oracle, every eighth head."""
    Q, K, Qn, Kn = _int_qk(BH, Lq, Lk, d, seed=8800 + d)
    s = Shape(1, BH, Lq, Lk, d, N, M)
    Qd, Kd = Q.to(DEV), K.to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention(Qd, Kd, V, s, scale), BH, Lq, Lk, d, torch.bfloat16)
    ties = _compare(W[::8], Qn[::8], Kn[::8], N, M, scale)
    assert ties > 100


def test_float_one_kernel_path():
    """The 4-byte mode's one-kernel path (split products; integer inputs are exact in its bfloat16 pieces)."""
    BH, Lq, Lk, d = 2, 128, 256, 64
    Q, K, Qn, Kn = _int_qk(BH, Lq, Lk, d, seed=8400, tdtype=torch.float32)
    s = Shape(1, BH, Lq, Lk, d, 1, 2, DFSS_F32_BF16X3)
    Qd, Kd = Q.to(DEV), K.to(DEV)
    W = _weights_through_identity_v(lambda V: dfss.dfss_attention(Qd, Kd, V, s, 0.125), BH, Lq, Lk, d, torch.float32)
    # weights are split into two bfloat16 pieces (2^-17) and the output is fp32: far tighter than the 2-byte mode
    ties = _compare(W, Qn, Kn, 1, 2, 0.125, rel=2.0 ** -14)
    assert ties > 100
