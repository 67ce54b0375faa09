"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, sizes follow the paper's footprint, and invalid arguments
are turned into status codes before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2203_00091_amd as dfss
from paper_2203_00091_amd import Shape
from paper_2203_00091_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "dfss.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:dfss|dense)_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = dfss.load_library()
    names = _declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/dfss.h but not exported"
    assert set(names) == set(binding.EXPORTS)
    for n in binding.INTERNAL_EXPORTS:      # test hooks, declared in csrc/dfss_internal.h
        assert hasattr(lib, n), n


def test_sizes_follow_the_compressed_footprint():
    s = Shape(8, 12, 384, 384, 64, 2, 4)
    dense = 96 * 384 * 384 * 2
    assert dfss.dfss_vals_bytes(s) == dense // 2           # N/M of the dense matrix (Sec. 2.3)
    assert dfss.dfss_meta_bytes(s) == dense // 16          # 1/16 of the dense bits (Sec. 2.3)
    assert dfss.dense_workspace_bytes(s) >= dense
    assert dfss.dfss_workspace_bytes(s) >= dense // 2 + dense // 16
    assert dfss.dfss_backward_workspace_bytes(s) >= dense // 2      # dS in the layout of the kept values
    s12 = Shape(16, 12, 512, 512, 64, 1, 2)
    assert dfss.dfss_vals_bytes(s12) == 192 * 512 * 512
    assert dfss.dfss_meta_bytes(s12) == 192 * 512 * 512 // 8
    # the 4-byte mode: half of the dense floats, metadata again 1/16 of the dense bits
    f32 = Shape(16, 12, 512, 512, 64, 1, 2, dfss.DFSS_F32)
    dense32 = 192 * 512 * 512 * 4
    assert dfss.dfss_vals_bytes(f32) == dense32 // 2
    assert dfss.dfss_meta_bytes(f32) == dense32 // 16
    assert dfss.dense_workspace_bytes(f32) >= dense32
    assert dfss.dfss_backward_workspace_bytes(f32) == 0     # no backward pass on the fp32 matrix instruction
    # the same arrays whichever way the fp32 products are formed
    x3 = Shape(16, 12, 512, 512, 64, 1, 2, dfss.DFSS_F32_BF16X3)
    for fn in (dfss.dfss_vals_bytes, dfss.dfss_meta_bytes, dfss.dfss_workspace_bytes, dfss.dense_workspace_bytes):
        assert fn(x3) == fn(f32)
    assert dfss.dfss_backward_workspace_bytes(x3) >= dense32 // 2     # the backward pass takes split products
    assert x3.meta_words == f32.meta_words == 512 // 8 and x3.torch_dtype == f32.torch_dtype


@pytest.mark.parametrize("shape", [
    Shape(1, 1, 100, 250, 64),       # Lk not a multiple of 4 (whole runs of M keys)
    Shape(1, 1, 100, 256, 64, 1, 2, 2),  # lengths that are not tile multiples: 2-byte dtype only
    Shape(1, 1, 128, 192, 64, 1, 2, 1),
    Shape(0, 1, 128, 128, 64),
    Shape(1, 1, 128, 128, 64, 3, 4),  # N:M not implemented
    Shape(1, 1, 128, 128, 96),       # head size not implemented
    Shape(1, 1, 128, 128, 64, 2, 4, 1),  # 2:4 on float data: not a mode of the method (Sec. 2.3)
    Shape(1, 1, 128, 128, 64, 2, 4, 2),  # ... whichever way its products are formed
    Shape(1, 1, 128, 128, 64, 1, 2, 3),  # dtype not implemented
    Shape(300, 300, 128, 128, 64),   # too many heads for one launch
    Shape(1, 1, 128, 16384, 64),     # rows longer than the softmax kernel holds
])
def test_invalid_shapes_have_zero_size(shape):
    assert dfss.dfss_vals_bytes(shape) == 0
    assert dfss.dfss_workspace_bytes(shape) == 0


def odd_early(aligned):
    return ctypes.c_void_p(aligned.value + 2)


def test_unpadded_lengths_take_the_layout_of_the_padded_ones():
    """Stage calls on lengths that are not tile multiples (2-byte dtype): the compressed arrays are laid out for Lq
    rounded up to a multiple of 64 and Lk to a multiple of 128."""
    s, p = Shape(2, 3, 100, 260, 64), Shape(2, 3, 128, 384, 64)
    for f in (dfss.dfss_vals_bytes, dfss.dfss_meta_bytes, dfss.dfss_workspace_bytes, dfss.dense_workspace_bytes):
        assert f(s) == f(p) > 0
    assert (s.LqP, s.LkP, s.Lc, s.meta_words) == (128, 384, 192, 24)
    assert (p.LqP, p.LkP) == (128, 384)


def test_errors_are_reported_before_any_launch():
    lib = dfss.load_library()
    ok = Shape(1, 1, 128, 128, 64).c()
    buf = ctypes.create_string_buffer(64)          # host memory: never dereferenced on these paths
    p = ctypes.cast(buf, ctypes.c_void_p)
    aligned = ctypes.c_void_p((p.value + 15) // 16 * 16)
    E_NULL, E_SHAPE, E_UNSUP, E_WS = 1, 2, 3, 4
    assert lib.dfss_sddmm_prune(None, aligned, ctypes.byref(ok), 0.125, aligned, aligned, None) == E_NULL
    assert lib.dfss_sddmm_prune(aligned, aligned, None, 0.125, aligned, aligned, None) == E_NULL
    bad = Shape(1, 1, 100, 130, 64).c()    # (Lq = 100 alone is fine: unpadded lengths; Lk must hold whole runs of 4)
    assert lib.dfss_sddmm_prune(aligned, aligned, ctypes.byref(bad), 0.125, aligned, aligned, None) == E_SHAPE
    unp = Shape(1, 1, 100, 132, 64).c()    # unpadded lengths: the stage calls take them, with the same checks
    assert lib.dfss_sddmm_prune(aligned, odd_early(aligned), ctypes.byref(unp), 0.125, aligned, aligned, None) == E_SHAPE
    assert lib.dfss_sddmm_prune_causal(aligned, aligned, None, ctypes.byref(unp), 0.125, aligned, aligned, None) == E_UNSUP
    assert lib.dfss_attention(aligned, aligned, aligned, ctypes.byref(unp), 0.125, aligned, None, 0, None) == E_SHAPE
    bad = Shape(1, 1, 128, 128, 64, 4, 8).c()
    assert lib.dfss_sddmm_prune(aligned, aligned, ctypes.byref(bad), 0.125, aligned, aligned, None) == E_UNSUP
    for scale in (0.0, -1.0, float("inf"), float("nan")):
        assert lib.dfss_sddmm_prune(aligned, aligned, ctypes.byref(ok), scale, aligned, aligned, None) == E_UNSUP
    odd = ctypes.c_void_p(aligned.value + 2)
    assert lib.dfss_sddmm_prune(odd, aligned, ctypes.byref(ok), 0.125, aligned, aligned, None) == E_SHAPE
    assert lib.dfss_sparse_softmax(None, ctypes.byref(ok), None) == E_NULL
    assert lib.dfss_spmm(aligned, aligned, aligned, ctypes.byref(ok), None, None) == E_NULL
    ws = ctypes.c_void_p((p.value + 255) // 256 * 256)
    assert lib.dfss_attention_staged(aligned, aligned, aligned, ctypes.byref(ok), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dfss_attention_staged(aligned, aligned, aligned, ctypes.byref(ok), 0.125, aligned, None, 1 << 30, None) == E_NULL
    assert lib.dfss_attention_staged(aligned, aligned, aligned, ctypes.byref(ok), 0.125, aligned,
                                     ctypes.c_void_p(ws.value + 16), 1 << 30, None) == E_SHAPE   # workspace not 256-byte aligned
    assert lib.dfss_attention(None, aligned, aligned, ctypes.byref(ok), 0.125, aligned, None, 0, None) == E_NULL
    assert lib.dfss_attention(aligned, aligned, aligned, ctypes.byref(ok), -0.125, aligned, None, 0, None) == E_UNSUP
    assert lib.dense_attention(aligned, aligned, aligned, ctypes.byref(ok), 0.125, aligned, ws, 16, None) == E_WS
    # the key-bias entry points validate the same way, and reject a misaligned bias pointer
    assert lib.dfss_sddmm_prune_bias(None, aligned, aligned, ctypes.byref(ok), 0.125, aligned, aligned, None) == E_NULL
    assert lib.dfss_sddmm_prune_bias(aligned, aligned, odd, ctypes.byref(ok), 0.125, aligned, aligned, None) == E_SHAPE
    assert lib.dfss_attention_staged_bias(aligned, aligned, aligned, aligned, ctypes.byref(ok), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dfss_attention_bias(aligned, aligned, aligned, odd, ctypes.byref(ok), 0.125, aligned, None, 0, None) == E_SHAPE
    assert lib.dense_attention_bias(aligned, aligned, aligned, aligned, ctypes.byref(ok), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dense_attention_fused_bias(aligned, aligned, aligned, odd, ctypes.byref(ok), 0.125, aligned, None) == E_SHAPE
    assert lib.dense_attention_fused_bias(aligned, aligned, aligned, aligned, ctypes.byref(ok), -1.0, aligned, None) == E_UNSUP
    assert lib.dfss_attention_blocked(aligned, aligned, aligned, None, None, ctypes.byref(ok), 0.125, aligned, None) == E_NULL
    assert lib.dfss_attention_blocked(aligned, aligned, aligned, None, aligned, ctypes.byref(bad), 0.125, aligned, None) == E_UNSUP
    assert lib.dense_attention_fused_blocked(aligned, aligned, aligned, odd, aligned, ctypes.byref(ok), 0.125, aligned, None) == E_SHAPE
    assert lib.dfss_attention_blocked_split(aligned, aligned, aligned, None, aligned, ctypes.byref(ok), 0.125, aligned, None, 1 << 30, None) == E_NULL
    assert lib.dfss_attention_blocked_split(aligned, aligned, aligned, None, aligned, ctypes.byref(ok), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dense_attention_fused_blocked_split(aligned, aligned, aligned, None, None, ctypes.byref(ok), 0.125, aligned, ws, 1 << 30, None) == E_NULL
    assert lib.dense_attention_fused_blocked_split(aligned, aligned, aligned, odd, aligned, ctypes.byref(ok), 0.125, aligned, ws, 1 << 30, None) == E_SHAPE
    assert lib.dfss_blocked_split_workspace_bytes(ctypes.byref(ok)) > 0
    assert lib.dfss_blocked_split_workspace_bytes(ctypes.byref(Shape(1, 1, 100, 128, 64).c())) == 0
    # the general additive mask: same checks, 2-byte dtype only
    assert lib.dfss_sddmm_prune_mask(aligned, aligned, None, ctypes.byref(ok), 0.125, aligned, aligned, None) == E_NULL
    assert lib.dfss_sddmm_prune_mask(aligned, aligned, odd, ctypes.byref(ok), 0.125, aligned, aligned, None) == E_SHAPE
    assert lib.dfss_attention_staged_mask(aligned, aligned, aligned, aligned, ctypes.byref(ok), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dfss_attention_staged_mask(aligned, aligned, aligned, aligned, ctypes.byref(ok), 0.0, aligned, ws, 1 << 30, None) == E_UNSUP
    assert lib.dense_attention_mask(aligned, aligned, None, aligned, ctypes.byref(ok), 0.125, aligned, ws, 1 << 30, None) == E_NULL
    assert lib.dense_attention_mask(aligned, aligned, aligned, aligned, ctypes.byref(ok), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dfss_attention_mask(aligned, aligned, aligned, None, ctypes.byref(ok), 0.125, aligned, None) == E_NULL
    assert lib.dfss_attention_mask(aligned, aligned, aligned, odd, ctypes.byref(unp), 0.125, aligned, None) == E_SHAPE
    assert lib.dfss_attention_mask(aligned, aligned, aligned, aligned, ctypes.byref(Shape(1, 1, 100, 130, 64).c()), 0.125, aligned, None) == E_SHAPE
    assert lib.dense_attention_fused_mask(aligned, aligned, aligned, aligned, ctypes.byref(ok), float("nan"), aligned, None) == E_UNSUP
    assert lib.dense_attention_fused_mask(aligned, aligned, aligned, aligned, ctypes.byref(ok), 0.125, None, None) == E_NULL
    assert lib.dfss_attention_varlen(aligned, aligned, aligned, None, ctypes.byref(ok), 0.125, aligned, None) == E_NULL
    assert lib.dfss_attention_varlen(aligned, aligned, aligned, odd, ctypes.byref(ok), 0.125, aligned, None) == E_SHAPE
    assert lib.dfss_attention_varlen(aligned, aligned, aligned, aligned, ctypes.byref(unp), 0.125, aligned, None) == E_SHAPE
    assert lib.dfss_attention_varlen(aligned, aligned, aligned, aligned, ctypes.byref(ok), 0.0, aligned, None) == E_UNSUP
    assert lib.dfss_spmm_t(aligned, aligned, None, ctypes.byref(ok), aligned, None) == E_NULL
    assert lib.dfss_attention_backward(aligned, aligned, aligned, aligned, aligned, aligned, aligned, ctypes.byref(ok),
                                       0.125, aligned, aligned, aligned, ws, 16, None) == E_WS
    assert lib.dfss_attention_backward(aligned, aligned, aligned, aligned, aligned, aligned, aligned, ctypes.byref(ok),
                                       0.0, aligned, aligned, aligned, ws, 1 << 30, None) == E_UNSUP
    # the 4-byte mode: calls without a float path refuse it, the others validate as usual
    f32 = Shape(1, 1, 128, 128, 64, 1, 2, dfss.DFSS_F32).c()
    assert lib.dense_attention_fused(aligned, aligned, aligned, ctypes.byref(f32), 0.125, aligned, None) == E_UNSUP
    assert lib.dfss_sddmm_prune_bias(aligned, aligned, odd, ctypes.byref(f32), 0.125, aligned, aligned, None) == E_SHAPE
    assert lib.dfss_attention_bias(aligned, aligned, aligned, aligned, ctypes.byref(f32), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dense_attention_bias(aligned, aligned, aligned, aligned, ctypes.byref(f32), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dfss_attention_blocked(aligned, aligned, aligned, None, aligned, ctypes.byref(f32), 0.125, aligned, None) == E_UNSUP
    assert lib.dfss_attention_blocked_split(aligned, aligned, aligned, None, aligned, ctypes.byref(f32), 0.125, aligned, ws, 1 << 30, None) == E_UNSUP
    assert lib.dfss_blocked_split_workspace_bytes(ctypes.byref(f32)) == 0
    assert lib.dfss_sddmm_prune_mask(aligned, aligned, aligned, ctypes.byref(f32), 0.125, aligned, aligned, None) == E_UNSUP
    assert lib.dfss_attention_mask(aligned, aligned, aligned, aligned, ctypes.byref(f32), 0.125, aligned, None) == E_UNSUP
    x3 = Shape(1, 1, 128, 128, 64, 1, 2, dfss.DFSS_F32_BF16X3).c()
    assert lib.dfss_attention_mask(aligned, aligned, aligned, aligned, ctypes.byref(x3), 0.125, aligned, None) == E_UNSUP
    assert lib.dense_attention_fused_mask(aligned, aligned, aligned, aligned, ctypes.byref(x3), 0.125, aligned, None) == E_UNSUP
    assert lib.dfss_attention_varlen(aligned, aligned, aligned, aligned, ctypes.byref(f32), 0.125, aligned, None) == E_UNSUP
    assert lib.dfss_spmm_t(aligned, aligned, aligned, ctypes.byref(f32), aligned, None) == E_UNSUP
    assert lib.dfss_attention_backward(aligned, aligned, aligned, aligned, aligned, aligned, aligned, ctypes.byref(f32),
                                       0.125, aligned, aligned, aligned, ws, 1 << 30, None) == E_UNSUP
    assert lib.dfss_attention(aligned, aligned, aligned, ctypes.byref(f32), 0.125, aligned, ws, 16, None) == E_WS
    assert lib.dense_attention(aligned, aligned, aligned, ctypes.byref(f32), 0.125, aligned, ws, 16, None) == E_WS
    # unpadded lengths: any Lq, Lk a multiple of 4; bfloat16 or split-product float data only
    rag = Shape(1, 1, 100, 132, 64).c()
    assert lib.dfss_attention_ragged(aligned, aligned, None, None, ctypes.byref(rag), 0.125, aligned, None) == E_NULL
    assert lib.dfss_attention_ragged(aligned, aligned, aligned, odd, ctypes.byref(rag), 0.125, aligned, None) == E_SHAPE
    assert lib.dfss_attention_ragged(aligned, aligned, aligned, None, ctypes.byref(rag), 0.0, aligned, None) == E_UNSUP
    for bad_rag in (Shape(1, 1, 100, 130, 64), Shape(1, 1, 100, 8196, 64), Shape(1, 1, 0, 128, 64)):
        assert lib.dfss_attention_ragged(aligned, aligned, aligned, None, ctypes.byref(bad_rag.c()), 0.125, aligned, None) == E_SHAPE
        assert lib.dense_attention_fused_ragged(aligned, aligned, aligned, None, ctypes.byref(bad_rag.c()), 0.125, aligned, None) == E_SHAPE
    for unsup in (Shape(1, 1, 100, 132, 64, 1, 2, dfss.DFSS_F32), Shape(1, 1, 100, 132, 64, 2, 4, dfss.DFSS_F32_BF16X3),
                  Shape(1, 1, 100, 132, 96), Shape(1, 1, 100, 132, 64, 3, 4)):
        assert lib.dfss_attention_ragged(aligned, aligned, aligned, None, ctypes.byref(unsup.c()), 0.125, aligned, None) == E_UNSUP
    assert lib.dfss_status_string(0) == b"ok"
    assert lib.dfss_status_string(E_WS) == b"workspace too small"


def test_causal_calls_validate_before_any_launch():
    """More queries than keys is a shape error (the queries are the last Lq positions); 4-byte dtypes are not
    implemented; everything else is validated as in the calls without the suffix."""
    lib = dfss.load_library()
    buf = ctypes.create_string_buffer(1024)
    a = ctypes.c_void_p((ctypes.cast(buf, ctypes.c_void_p).value + 255) // 256 * 256)
    E_NULL, E_SHAPE, E_UNSUP, E_WS = 1, 2, 3, 4
    ok = Shape(1, 1, 128, 256, 64).c()
    more_queries = Shape(1, 1, 256, 128, 64).c()
    f32 = Shape(1, 1, 128, 128, 64, 1, 2, dfss.DFSS_F32_BF16X3).c()
    for shape, want in ((more_queries, E_SHAPE), (f32, E_UNSUP)):
        r = ctypes.byref(shape)
        assert lib.dfss_sddmm_prune_causal(a, a, None, r, 0.125, a, a, None) == want
        assert lib.dfss_attention_causal(a, a, a, None, r, 0.125, a, None) == want
        assert lib.dfss_attention_staged_causal(a, a, a, None, r, 0.125, a, a, 1 << 40, None) == want
        assert lib.dense_attention_causal(a, a, a, None, r, 0.125, a, a, 1 << 40, None) == want
        assert lib.dense_attention_fused_causal(a, a, a, None, r, 0.125, a, None) == want
    r = ctypes.byref(ok)
    assert lib.dfss_attention_causal(None, a, a, None, r, 0.125, a, None) == E_NULL
    assert lib.dfss_attention_causal(a, a, a, None, r, float("nan"), a, None) == E_UNSUP
    assert lib.dfss_attention_causal(a, a, a, ctypes.c_void_p(a.value + 4), r, 0.125, a, None) == E_SHAPE   # bias alignment
    assert lib.dfss_attention_staged_causal(a, a, a, None, r, 0.125, a, a, 16, None) == E_WS
    assert lib.dense_attention_causal(a, a, a, None, r, 0.125, a, a, 16, None) == E_WS
    assert lib.dfss_sddmm_prune_causal(a, a, None, r, 0.125, None, a, None) == E_NULL


def test_binding_refuses_host_tensors():
    import torch
    s = Shape(1, 1, 128, 128, 64)
    q = torch.zeros(1, 128, 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        dfss.dfss_sddmm_prune(q, q, s, 0.125, vals=q, meta=q)
    with pytest.raises(ValueError):   # element type that does not match dfss_shape.dtype (checked before the device check)
        dfss.dfss_sddmm_prune(q.float(), q.float(), s, 0.125, vals=q, meta=q)
    with pytest.raises(ValueError):   # key bias of the wrong shape or type
        dfss.dfss_attention_bias(q, q, q, torch.zeros(2, 128), s, 0.125, O=q, ws=q)
