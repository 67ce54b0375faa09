"""ctypes binding of the C ABI declared in include/dfss.h.

Each function has the name of the C entry point it calls and only marshals
arguments: tensors are passed as raw device pointers, the current PyTorch HIP
stream as the stream handle.  There is no fallback: if ``libdfss.so`` is
missing or a call reports an error, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdfss.so")

EXPORTS = (
    "dfss_vals_bytes", "dfss_meta_bytes", "dfss_workspace_bytes", "dense_workspace_bytes",
    "dfss_sddmm_prune", "dfss_sparse_softmax", "dfss_spmm", "dfss_attention", "dense_attention",
    "dense_attention_fused", "dfss_meta_to_canonical", "dfss_meta_from_canonical", "dfss_status_string",
    "dfss_sddmm_prune_bias", "dfss_attention_bias", "dense_attention_bias", "dense_attention_fused_bias",
    "dfss_attention_blocked", "dense_attention_fused_blocked", "dfss_spmm_t",
    "dfss_backward_workspace_bytes", "dfss_attention_backward",
    "dfss_attention_ragged", "dense_attention_fused_ragged",
    "dfss_attention_staged", "dfss_attention_staged_bias",
    "dfss_static_scratch_bytes", "dfss_attention_staged_static",
    "dfss_sddmm_prune_causal", "dfss_attention_causal", "dfss_attention_staged_causal", "dense_attention_causal",
    "dense_attention_fused_causal",
    "dfss_blocked_split_workspace_bytes", "dfss_attention_blocked_split", "dense_attention_fused_blocked_split",
    "dfss_sddmm_prune_mask", "dfss_attention_staged_mask", "dense_attention_mask",
    "dfss_attention_mask", "dense_attention_fused_mask",
    "dfss_attention_varlen",
)
# exported for the library's own tests only (csrc/dfss_internal.h)
INTERNAL_EXPORTS = ("dfss_internal_attention_variant",)
VARIANT_AUTO, VARIANT_Q16, VARIANT_Q16X2, VARIANT_Q32W2, VARIANT_Q32W4, VARIANT_Q32K2 = range(6)


DFSS_BF16, DFSS_F32, DFSS_F32_BF16X3 = 0, 1, 2


class DfssError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__(f"{fn} failed: status {status} ({text})")
        self.status = status


class _CShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "H", "Lq", "Lk", "d", "N", "M", "dtype")]


@dataclass(frozen=True)
class Shape:
    """Mirror of ``dfss_shape``: B*H heads, Lq queries, Lk keys, head size d, keep N of M."""
    B: int
    H: int
    Lq: int
    Lk: int
    d: int
    N: int = 2
    M: int = 4
    dtype: int = 0  # DFSS_BF16 = 0; DFSS_F32 = 1, DFSS_F32_BF16X3 = 2 (the 4-byte mode: 1:2 only)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == DFSS_BF16 else torch.float32

    @property
    def LqP(self) -> int:
        """Rows of the compressed arrays (vals, meta, the dense workspace): Lq, rounded up to a multiple of 64 where
        the stage calls take an unpadded length (2-byte dtype)."""
        return (self.Lq + 63) // 64 * 64

    @property
    def LkP(self) -> int:
        """Keys of the compressed arrays: Lk, rounded up to a multiple of 128 where the stage calls take an unpadded
        length."""
        return (self.Lk + 127) // 128 * 128

    @property
    def meta_words(self) -> int:
        """uint16 metadata words per row: one 4-bit code per 8 bytes of dense data."""
        return self.LkP // (16 if self.dtype == DFSS_BF16 else 8)

    def c(self) -> _CShape:
        return _CShape(self.B, self.H, self.Lq, self.Lk, self.d, self.N, self.M, self.dtype)

    @property
    def BH(self) -> int:
        return self.B * self.H

    @property
    def Lc(self) -> int:
        """Kept entries per row of the compressed arrays."""
        return self.LkP * self.N // self.M


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libdfss.so (built in-tree by ``paper_2203_00091_amd.build``); raise if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} not built: run `python -m paper_2203_00091_amd.build` (needs hipcc)")
        L = ctypes.CDLL(_LIB_PATH)
        sp = ctypes.POINTER(_CShape)
        vp, sz, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
        for name in ("dfss_vals_bytes", "dfss_meta_bytes", "dfss_workspace_bytes", "dense_workspace_bytes",
                     "dfss_backward_workspace_bytes", "dfss_blocked_split_workspace_bytes"):
            getattr(L, name).argtypes = [sp]
            getattr(L, name).restype = sz
        L.dfss_sddmm_prune.argtypes = [vp, vp, sp, f32, vp, vp, vp]
        L.dfss_sparse_softmax.argtypes = [vp, sp, vp]
        L.dfss_spmm.argtypes = [vp, vp, vp, sp, vp, vp]
        L.dfss_attention.argtypes = [vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dense_attention.argtypes = [vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dense_attention_fused.argtypes = [vp, vp, vp, sp, f32, vp, vp]
        L.dfss_sddmm_prune_bias.argtypes = [vp, vp, vp, sp, f32, vp, vp, vp]
        L.dfss_attention_bias.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dense_attention_bias.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dense_attention_fused_bias.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_attention_blocked.argtypes = [vp, vp, vp, vp, vp, sp, f32, vp, vp]
        L.dense_attention_fused_blocked.argtypes = [vp, vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_attention_blocked_split.argtypes = [vp, vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dense_attention_fused_blocked_split.argtypes = [vp, vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dfss_sddmm_prune_mask.argtypes = [vp, vp, vp, sp, f32, vp, vp, vp]
        L.dfss_attention_staged_mask.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dense_attention_mask.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dfss_attention_mask.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_attention_varlen.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dense_attention_fused_mask.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_attention_ragged.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_attention_staged.argtypes = [vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dfss_attention_staged_bias.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dfss_attention_staged_static.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_sddmm_prune_causal.argtypes = [vp, vp, vp, sp, f32, vp, vp, vp]
        L.dfss_attention_causal.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_attention_staged_causal.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dense_attention_causal.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp, sz, vp]
        L.dense_attention_fused_causal.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_attention_staged_static.restype = ctypes.c_int
        L.dfss_static_scratch_bytes.argtypes = []
        L.dfss_static_scratch_bytes.restype = sz
        L.dfss_internal_attention_variant.argtypes = [vp, vp, vp, vp, sp, f32, vp, ctypes.c_int, ctypes.c_int, vp]
        L.dense_attention_fused_ragged.argtypes = [vp, vp, vp, vp, sp, f32, vp, vp]
        L.dfss_spmm_t.argtypes = [vp, vp, vp, sp, vp, vp]
        L.dfss_attention_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, sp, f32, vp, vp, vp, vp, sz, vp]
        L.dfss_meta_to_canonical.argtypes = [vp, sp, vp, vp]
        L.dfss_meta_from_canonical.argtypes = [vp, sp, vp, vp]
        for name in ("dfss_sddmm_prune", "dfss_sparse_softmax", "dfss_spmm", "dfss_attention",
                     "dense_attention", "dense_attention_fused", "dfss_meta_to_canonical", "dfss_meta_from_canonical",
                     "dfss_sddmm_prune_bias", "dfss_attention_bias", "dense_attention_bias",
                     "dense_attention_fused_bias", "dfss_attention_blocked", "dense_attention_fused_blocked",
                     "dfss_attention_ragged", "dense_attention_fused_ragged", "dfss_spmm_t",
                     "dfss_attention_backward", "dfss_attention_staged", "dfss_attention_staged_bias",
                     "dfss_internal_attention_variant", "dfss_sddmm_prune_causal", "dfss_attention_causal",
                     "dfss_attention_staged_causal", "dense_attention_causal", "dense_attention_fused_causal",
                     "dfss_attention_blocked_split", "dense_attention_fused_blocked_split",
                     "dfss_sddmm_prune_mask", "dfss_attention_staged_mask", "dense_attention_mask",
                     "dfss_attention_mask", "dense_attention_fused_mask",
                     "dfss_attention_varlen"):
            getattr(L, name).restype = ctypes.c_int
        L.dfss_status_string.argtypes = [ctypes.c_int]
        L.dfss_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(fn: str, status: int):
    if status != 0:
        raise DfssError(fn, status, load_library().dfss_status_string(status).decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: torch.Tensor | None) -> int | None:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def _data(t: torch.Tensor | None, s: Shape, *shape) -> int | None:
    """Pointer of a Q/K/V/O/vals-like tensor after checking that its element type is the one the shape
    declares and its size the one the call will touch (the C side sees raw pointers only)."""
    if t is None:
        return None
    if t.dtype != s.torch_dtype:
        raise ValueError(f"expected a {s.torch_dtype} tensor for dfss_shape.dtype = {s.dtype}, got {t.dtype}")
    n = 1
    for k in shape:
        n *= k
    if t.numel() != n:
        raise ValueError(f"expected {n} elements {shape}, got {t.numel()}")
    return _ptr(t)


def _q(t, s: Shape):      # Q, O and their gradients: [BH, Lq, d]
    return _data(t, s, s.BH, s.Lq, s.d)


def _kv(t, s: Shape):     # K, V and their gradients: [BH, Lk, d]
    return _data(t, s, s.BH, s.Lk, s.d)


def _kept(t, s: Shape):   # kept scores / weights: [BH, Lq, Lk*N/M]
    return _data(t, s, s.BH, s.LqP, s.Lc)


def _meta(t: torch.Tensor, s: Shape) -> int:
    if t.element_size() != 2 or t.numel() != s.BH * s.LqP * s.meta_words:
        raise ValueError(f"metadata must hold {s.BH * s.LqP * s.meta_words} 16-bit words")
    return _ptr(t)


def dfss_vals_bytes(s: Shape) -> int:
    return int(load_library().dfss_vals_bytes(ctypes.byref(s.c())))


def dfss_meta_bytes(s: Shape) -> int:
    return int(load_library().dfss_meta_bytes(ctypes.byref(s.c())))


def dfss_workspace_bytes(s: Shape) -> int:
    return int(load_library().dfss_workspace_bytes(ctypes.byref(s.c())))


def dense_workspace_bytes(s: Shape) -> int:
    return int(load_library().dense_workspace_bytes(ctypes.byref(s.c())))


def _alloc_bytes(n: int, device) -> torch.Tensor:
    return torch.empty(max(n, 1), dtype=torch.uint8, device=device)


def dfss_sddmm_prune(Q, K, s: Shape, scale: float, vals=None, meta=None):
    """Stage 1.  Returns (vals [BH, Lq, Lk*N/M] in the shape's dtype, meta: 16-bit words in library order)."""
    if vals is None:
        vals = torch.empty((s.BH, s.LqP, s.Lc), dtype=s.torch_dtype, device=Q.device)
    if meta is None:
        meta = torch.empty((s.BH * s.LqP * s.meta_words,), dtype=torch.int16, device=Q.device)
    st = load_library().dfss_sddmm_prune(_q(Q, s), _kv(K, s), ctypes.byref(s.c()), scale,
                                         _kept(vals, s), _meta(meta, s), _stream())
    _check("dfss_sddmm_prune", st)
    return vals, meta


def dfss_sparse_softmax(vals, s: Shape):
    """Stage 2, in place on vals."""
    _check("dfss_sparse_softmax", load_library().dfss_sparse_softmax(_kept(vals, s), ctypes.byref(s.c()), _stream()))
    return vals


def dfss_spmm(vals, meta, V, s: Shape, O=None):
    """Stage 3.  Returns O [BH, Lq, d]."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=V.device)
    st = load_library().dfss_spmm(_kept(vals, s), _meta(meta, s), _kv(V, s),
                                  ctypes.byref(s.c()), _q(O, s), _stream())
    _check("dfss_spmm", st)
    return O


def _needs_workspace(s: Shape) -> bool:
    """Only the exact-product float mode runs dfss_attention through a workspace."""
    return s.dtype == DFSS_F32


def dfss_attention(Q, K, V, s: Shape, scale: float, O=None, ws=None):
    """Whole DFSS forward in one kernel.  ``ws`` is passed on if given (the library uses it with DFSS_F32 only,
    where it is allocated here if absent)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None and _needs_workspace(s):
        ws = _alloc_bytes(dfss_workspace_bytes(s), Q.device)
    st = load_library().dfss_attention(_q(Q, s), _kv(K, s), _kv(V, s),
                                       ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                       0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check("dfss_attention", st)
    return O


def dfss_attention_staged(Q, K, V, s: Shape, scale: float, O=None, ws=None):
    """Whole DFSS forward through ``ws`` (allocated if not given): stage 1, then the product that applies the
    softmax as it reads the kept scores (4-byte dtypes: the three stage kernels)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dfss_workspace_bytes(s), Q.device)
    st = load_library().dfss_attention_staged(_q(Q, s), _kv(K, s), _kv(V, s),
                                              ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                              ws.numel() * ws.element_size(), _stream())
    _check("dfss_attention_staged", st)
    return O


def dfss_attention_staged_bias(Q, K, V, key_bias, s: Shape, scale: float, O=None, ws=None):
    """dfss_attention_staged with an additive key bias (may be None)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dfss_workspace_bytes(s), Q.device)
    st = load_library().dfss_attention_staged_bias(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                   ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                                   ws.numel() * ws.element_size(), _stream())
    _check("dfss_attention_staged_bias", st)
    return O


def dfss_static_scratch_bytes() -> int:
    return int(load_library().dfss_static_scratch_bytes())


def dfss_attention_staged_static(Q, K, V, key_bias, s: Shape, scale: float, O):
    """The staged forward pass with the library's own fixed scratch array; allocates nothing (O is the caller's)."""
    st = load_library().dfss_attention_staged_static(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                     ctypes.byref(s.c()), scale, _q(O, s), _stream())
    _check("dfss_attention_staged_static", st)
    return O


def internal_attention_variant(Q, K, V, key_bias, s: Shape, scale: float, variant: int, dense: bool = False, O=None):
    """Test hook: the one-kernel forward pass (DFSS, or full attention if ``dense``) with a named tiling."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dfss_internal_attention_variant(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                        ctypes.byref(s.c()), scale, _q(O, s), int(variant),
                                                        int(bool(dense)), _stream())
    _check("dfss_internal_attention_variant", st)
    return O


def dense_attention(Q, K, V, s: Shape, scale: float, O=None, ws=None):
    """Full attention baseline on the same GPU."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dense_workspace_bytes(s), Q.device)
    st = load_library().dense_attention(_q(Q, s), _kv(K, s), _kv(V, s),
                                        ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                        ws.numel() * ws.element_size(), _stream())
    _check("dense_attention", st)
    return O


def dense_attention_fused(Q, K, V, s: Shape, scale: float, O=None):
    """Full attention in one kernel (the stronger baseline)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dense_attention_fused(_q(Q, s), _kv(K, s), _kv(V, s),
                                              ctypes.byref(s.c()), scale, _q(O, s),
                                              _stream())
    _check("dense_attention_fused", st)
    return O


def _bias_ptr(key_bias, s: Shape):
    if key_bias is None:
        return None
    if key_bias.dtype != torch.float32 or tuple(key_bias.shape) != (s.B, s.Lk):
        raise ValueError(f"key_bias must be float32 [B, Lk] = [{s.B}, {s.Lk}]")
    return _ptr(key_bias)


def dfss_sddmm_prune_bias(Q, K, key_bias, s: Shape, scale: float, vals=None, meta=None):
    """Stage 1 with an additive key bias (float32 [B, Lk] device tensor, -inf masks a key)."""
    if vals is None:
        vals = torch.empty((s.BH, s.LqP, s.Lc), dtype=s.torch_dtype, device=Q.device)
    if meta is None:
        meta = torch.empty((s.BH * s.LqP * s.meta_words,), dtype=torch.int16, device=Q.device)
    st = load_library().dfss_sddmm_prune_bias(_q(Q, s), _kv(K, s), _bias_ptr(key_bias, s),
                                              ctypes.byref(s.c()), scale, _kept(vals, s), _meta(meta, s), _stream())
    _check("dfss_sddmm_prune_bias", st)
    return vals, meta


def dfss_attention_bias(Q, K, V, key_bias, s: Shape, scale: float, O=None, ws=None):
    """Whole DFSS forward (one kernel) with an additive key bias."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None and _needs_workspace(s):
        ws = _alloc_bytes(dfss_workspace_bytes(s), Q.device)
    st = load_library().dfss_attention_bias(_q(Q, s), _kv(K, s), _kv(V, s),
                                            _bias_ptr(key_bias, s), ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                            0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check("dfss_attention_bias", st)
    return O


def dense_attention_bias(Q, K, V, key_bias, s: Shape, scale: float, O=None, ws=None):
    """Full attention (three stages) with an additive key bias."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dense_workspace_bytes(s), Q.device)
    st = load_library().dense_attention_bias(_q(Q, s), _kv(K, s), _kv(V, s),
                                             _bias_ptr(key_bias, s), ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                            ws.numel() * ws.element_size(), _stream())
    _check("dense_attention_bias", st)
    return O


def dense_attention_fused_bias(Q, K, V, key_bias, s: Shape, scale: float, O=None):
    """Full attention in one kernel with an additive key bias."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dense_attention_fused_bias(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                   ctypes.byref(s.c()), scale, _q(O, s), _stream())
    _check("dense_attention_fused_bias", st)
    return O


def dfss_sddmm_prune_causal(Q, K, key_bias, s: Shape, scale: float, vals=None, meta=None):
    """Stage 1 under the causal mask (query i sees keys 0 .. i + Lk - Lq); key_bias may be None."""
    if vals is None:
        vals = torch.empty((s.BH, s.LqP, s.Lc), dtype=s.torch_dtype, device=Q.device)
    if meta is None:
        meta = torch.empty((s.BH * s.LqP * s.meta_words,), dtype=torch.int16, device=Q.device)
    st = load_library().dfss_sddmm_prune_causal(_q(Q, s), _kv(K, s), _bias_ptr(key_bias, s),
                                                ctypes.byref(s.c()), scale, _kept(vals, s), _meta(meta, s), _stream())
    _check("dfss_sddmm_prune_causal", st)
    return vals, meta


def dfss_attention_causal(Q, K, V, key_bias, s: Shape, scale: float, O=None):
    """Whole DFSS forward in one kernel under the causal mask; key_bias may be None."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dfss_attention_causal(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                              ctypes.byref(s.c()), scale, _q(O, s), _stream())
    _check("dfss_attention_causal", st)
    return O


def dfss_attention_staged_causal(Q, K, V, key_bias, s: Shape, scale: float, O=None, ws=None):
    """dfss_attention_staged under the causal mask; key_bias may be None."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dfss_workspace_bytes(s), Q.device)
    st = load_library().dfss_attention_staged_causal(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                     ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                                     ws.numel() * ws.element_size(), _stream())
    _check("dfss_attention_staged_causal", st)
    return O


def dense_attention_causal(Q, K, V, key_bias, s: Shape, scale: float, O=None, ws=None):
    """Full attention (three stages) under the causal mask; key_bias may be None."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dense_workspace_bytes(s), Q.device)
    st = load_library().dense_attention_causal(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                               ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                               ws.numel() * ws.element_size(), _stream())
    _check("dense_attention_causal", st)
    return O


def dense_attention_fused_causal(Q, K, V, key_bias, s: Shape, scale: float, O=None):
    """Full attention in one kernel under the causal mask; key_bias may be None."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dense_attention_fused_causal(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                     ctypes.byref(s.c()), scale, _q(O, s), _stream())
    _check("dense_attention_fused_causal", st)
    return O


def dfss_attention_ragged(Q, K, V, key_bias, s: Shape, scale: float, O=None):
    """DFSS forward in one kernel on unpadded arrays: any Lq, Lk a multiple of 4; key_bias may be None."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dfss_attention_ragged(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                              ctypes.byref(s.c()), scale, _q(O, s), _stream())
    _check("dfss_attention_ragged", st)
    return O


def dense_attention_fused_ragged(Q, K, V, key_bias, s: Shape, scale: float, O=None):
    """Full attention in one kernel on unpadded arrays (the baseline of dfss_attention_ragged)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dense_attention_fused_ragged(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                     ctypes.byref(s.c()), scale, _q(O, s), _stream())
    _check("dense_attention_fused_ragged", st)
    return O


def _block_mask_ptr(block_mask, s: Shape):
    if block_mask.dtype != torch.uint8 or tuple(block_mask.shape) != (s.Lq // 64, s.Lk // 64):
        raise ValueError(f"block_mask must be uint8 [Lq/64, Lk/64] = [{s.Lq // 64}, {s.Lk // 64}]")
    return _ptr(block_mask)


def dfss_attention_blocked(Q, K, V, key_bias, block_mask, s: Shape, scale: float, O=None):
    """DFSS forward restricted to the 64 x 64 score blocks with a non-zero entry in block_mask."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dfss_attention_blocked(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                               _block_mask_ptr(block_mask, s), ctypes.byref(s.c()), scale, _q(O, s),
                                               _stream())
    _check("dfss_attention_blocked", st)
    return O


def dense_attention_fused_blocked(Q, K, V, key_bias, block_mask, s: Shape, scale: float, O=None):
    """Block-sparse full attention (same block pattern, no N:M pruning)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dense_attention_fused_blocked(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                      _block_mask_ptr(block_mask, s), ctypes.byref(s.c()), scale,
                                                      _q(O, s), _stream())
    _check("dense_attention_fused_blocked", st)
    return O


def _mask_ptr(mask: torch.Tensor, s: Shape) -> int:
    if mask.dtype != torch.float32 or mask.numel() != s.Lq * s.Lk:
        raise ValueError(f"the mask must be float32 [{s.Lq}, {s.Lk}]")
    return _ptr(mask)


def dfss_sddmm_prune_mask(Q, K, mask, s: Shape, scale: float, vals=None, meta=None):
    """Stage 1 with an additive mask [Lq, Lk] shared by all heads."""
    if vals is None:
        vals = torch.empty((s.BH, s.LqP, s.Lc), dtype=s.torch_dtype, device=Q.device)
    if meta is None:
        meta = torch.empty((s.BH * s.LqP * s.meta_words,), dtype=torch.int16, device=Q.device)
    st = load_library().dfss_sddmm_prune_mask(_q(Q, s), _kv(K, s), _mask_ptr(mask, s), ctypes.byref(s.c()), scale,
                                              _kept(vals, s), _meta(meta, s), _stream())
    _check("dfss_sddmm_prune_mask", st)
    return vals, meta


def dfss_attention_staged_mask(Q, K, V, mask, s: Shape, scale: float, O=None, ws=None):
    """dfss_attention_staged with an additive mask [Lq, Lk] shared by all heads."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dfss_workspace_bytes(s), Q.device)
    st = load_library().dfss_attention_staged_mask(_q(Q, s), _kv(K, s), _kv(V, s), _mask_ptr(mask, s),
                                                   ctypes.byref(s.c()), scale, _q(O, s), _ptr(ws),
                                                   ws.numel() * ws.element_size(), _stream())
    _check("dfss_attention_staged_mask", st)
    return O


def dense_attention_mask(Q, K, V, mask, s: Shape, scale: float, O=None, ws=None):
    """Full attention (three kernels) with the same mask."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dense_workspace_bytes(s), Q.device)
    st = load_library().dense_attention_mask(_q(Q, s), _kv(K, s), _kv(V, s), _mask_ptr(mask, s), ctypes.byref(s.c()),
                                             scale, _q(O, s), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check("dense_attention_mask", st)
    return O


def _len_ptr(key_len: torch.Tensor, s: Shape) -> int:
    if key_len.dtype != torch.int32 or key_len.numel() != s.B:
        raise ValueError(f"key_len must be int32 [B] = [{s.B}]")
    return _ptr(key_len)


def dfss_attention_varlen(Q, K, V, key_len, s: Shape, scale: float, O=None):
    """DFSS forward in one kernel on a padded batch: keys key_len[b] .. Lk - 1 of batch element b are padding."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dfss_attention_varlen(_q(Q, s), _kv(K, s), _kv(V, s), _len_ptr(key_len, s), ctypes.byref(s.c()),
                                              scale, _q(O, s), _stream())
    _check("dfss_attention_varlen", st)
    return O


def dfss_attention_mask(Q, K, V, mask, s: Shape, scale: float, O=None):
    """DFSS forward in one kernel with an additive mask fp32 [Lq, Lk] (any Lq, Lk a multiple of 4; arrays unpadded)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dfss_attention_mask(_q(Q, s), _kv(K, s), _kv(V, s), _mask_ptr(mask, s), ctypes.byref(s.c()),
                                            scale, _q(O, s), _stream())
    _check("dfss_attention_mask", st)
    return O


def dense_attention_fused_mask(Q, K, V, mask, s: Shape, scale: float, O=None):
    """Full attention in one kernel with the same mask (the baseline of dfss_attention_mask)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    st = load_library().dense_attention_fused_mask(_q(Q, s), _kv(K, s), _kv(V, s), _mask_ptr(mask, s),
                                                   ctypes.byref(s.c()), scale, _q(O, s), _stream())
    _check("dense_attention_fused_mask", st)
    return O


def dfss_blocked_split_workspace_bytes(s: Shape) -> int:
    return int(load_library().dfss_blocked_split_workspace_bytes(ctypes.byref(s.c())))


def dfss_attention_blocked_split(Q, K, V, key_bias, block_mask, s: Shape, scale: float, O=None, ws=None):
    """dfss_attention_blocked with a workspace: long row blocks are shared between several workgroups."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dfss_blocked_split_workspace_bytes(s), Q.device)
    st = load_library().dfss_attention_blocked_split(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                     _block_mask_ptr(block_mask, s), ctypes.byref(s.c()), scale,
                                                     _q(O, s), ws.data_ptr(), ws.numel() * ws.element_size(), _stream())
    _check("dfss_attention_blocked_split", st)
    return O


def dense_attention_fused_blocked_split(Q, K, V, key_bias, block_mask, s: Shape, scale: float, O=None, ws=None):
    """Block-sparse full attention with the same workspace (the baseline of dfss_attention_blocked_split)."""
    if O is None:
        O = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dfss_blocked_split_workspace_bytes(s), Q.device)
    st = load_library().dense_attention_fused_blocked_split(_q(Q, s), _kv(K, s), _kv(V, s), _bias_ptr(key_bias, s),
                                                            _block_mask_ptr(block_mask, s), ctypes.byref(s.c()), scale,
                                                            _q(O, s), ws.data_ptr(), ws.numel() * ws.element_size(),
                                                            _stream())
    _check("dense_attention_fused_blocked_split", st)
    return O


def dfss_spmm_t(vals, meta, X, s: Shape, out=None):
    """Transposed sparse product A^T X -> bf16 [BH, Lk, d] (dV = P^T dO, dK = dS^T Q)."""
    if out is None:
        out = torch.empty((s.BH, s.Lk, s.d), dtype=s.torch_dtype, device=X.device)
    st = load_library().dfss_spmm_t(_kept(vals, s), _meta(meta, s), _q(X, s),
                                    ctypes.byref(s.c()), _kv(out, s), _stream())
    _check("dfss_spmm_t", st)
    return out


def dfss_backward_workspace_bytes(s: Shape) -> int:
    return int(load_library().dfss_backward_workspace_bytes(ctypes.byref(s.c())))


def dfss_attention_backward(dO, Q, K, V, O, P, meta, s: Shape, scale: float, dQ=None, dK=None, dV=None, ws=None):
    """Gradients through the fixed selection.  P, meta: weights and metadata kept from the forward stages."""
    if dQ is None:
        dQ = torch.empty((s.BH, s.Lq, s.d), dtype=s.torch_dtype, device=Q.device)
    if dK is None:
        dK = torch.empty((s.BH, s.Lk, s.d), dtype=s.torch_dtype, device=Q.device)
    if dV is None:
        dV = torch.empty((s.BH, s.Lk, s.d), dtype=s.torch_dtype, device=Q.device)
    if ws is None:
        ws = _alloc_bytes(dfss_backward_workspace_bytes(s), Q.device)
    st = load_library().dfss_attention_backward(_q(dO, s), _q(Q, s), _kv(K, s), _kv(V, s), _q(O, s),
                                                _kept(P, s), _meta(meta, s), ctypes.byref(s.c()), scale,
                                                _q(dQ, s), _kv(dK, s),
                                                _kv(dV, s), _ptr(ws),
                                                ws.numel() * ws.element_size(), _stream())
    _check("dfss_attention_backward", st)
    return dQ, dK, dV


def dfss_meta_to_canonical(meta, s: Shape, canon=None):
    """Library word order -> canonical uint16 [BH, Lq, Lk/16] (held as int16 bits)."""
    if canon is None:
        canon = torch.empty((s.BH, s.LqP, s.meta_words), dtype=torch.int16, device=meta.device)
    st = load_library().dfss_meta_to_canonical(_meta(meta, s), ctypes.byref(s.c()), _meta(canon, s), _stream())
    _check("dfss_meta_to_canonical", st)
    return canon


def dfss_meta_from_canonical(canon, s: Shape, meta=None):
    if meta is None:
        meta = torch.empty((s.BH * s.LqP * s.meta_words,), dtype=torch.int16, device=canon.device)
    st = load_library().dfss_meta_from_canonical(_meta(canon, s), ctypes.byref(s.c()), _meta(meta, s), _stream())
    _check("dfss_meta_from_canonical", st)
    return meta
