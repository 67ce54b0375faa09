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
