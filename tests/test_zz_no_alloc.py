"""The staged forward pass with the library's fixed scratch array (for callers that cannot allocate)
against the same pass with a caller workspace, through the C ABI."""
import ctypes
import math

import pytest
import torch

import paper_2203_00091_amd as dfss
from paper_2203_00091_amd import Shape, binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run_both(B, H, L, d, N, M, seed, with_bias):
    Q, K, V = (t.to(DEV) for t in synth.gaussian_qkv(B * H, L, L, d, 1.0, seed=seed))
    s = Shape(B, H, L, L, d, N, M)
    scale = 1.0 / math.sqrt(d)
    bias = None
    if with_bias:
        lengths = synth.padding_lengths(B, L, seed + 1)
        bias = synth.key_padding_bias(lengths, L).to(DEV)
    ref = dfss.dfss_attention_staged_bias(Q, K, V, bias, s, scale)
    O = torch.full((B * H, L, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    lib = dfss.load_library()
    st = lib.dfss_attention_staged_static(Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                                          None if bias is None else bias.data_ptr(), ctypes.byref(s.c()),
                                          scale, O.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == 0, st
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(O.view(torch.int16), ref.view(torch.int16))


def test_static_scratch_matches_the_workspace_call_twice_in_a_row():
    assert dfss.dfss_static_scratch_bytes() == 32 << 20
    _run_both(8, 12, 384, 64, 2, 4, 515, with_bias=False)    # 17.7 MB of the 32 MiB
    _run_both(2, 3, 128, 128, 1, 2, 516, with_bias=True)     # smaller second call on the same array
    _run_both(8, 12, 384, 64, 2, 4, 517, with_bias=True)


def test_static_scratch_rejects_what_does_not_fit():
    lib = dfss.load_library()
    s = Shape(16, 12, 512, 512, 64, 1, 2)        # 56.6 MB of kept scores and metadata
    assert dfss.dfss_workspace_bytes(s) > dfss.dfss_static_scratch_bytes()
    x = torch.zeros(16, dtype=torch.bfloat16, device=DEV)
    p = x.data_ptr()
    assert lib.dfss_attention_staged_static(p, p, p, None, ctypes.byref(s.c()), 0.125, p, None) == 4   # workspace
    bad = Shape(1, 1, 100, 128, 64)
    assert lib.dfss_attention_staged_static(p, p, p, None, ctypes.byref(bad.c()), 0.125, p, None) == 2
    assert lib.dfss_attention_staged_static(None, p, p, None, ctypes.byref(s.c()), 0.125, p, None) == 1
