"""CPU oracle for the DFSS attention forward pass -- TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the CPU-baseline leg of the benchmark
may import this package.  It wraps ``dfss_oracle.c`` (plain C, built with gcc)
through ctypes and numpy; it shares nothing with the HIP library.

Passages followed (arXiv 2203.00091): Eq. 1 (Sec. 2.1), the N:M selection
(Sec. 2.3, App. A.1.1), the metadata words (App. A.1.1, A.1.2), the softmax
over kept entries (Sec. 3.1, App. A.1.3), the L^p quality (Def. 4.1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dfss_oracle.c")
# An instrumented build for the test-suite's sanitizer pass: extra gcc flags and a library name of its own, so that
# it never replaces the plain build.  Test infrastructure only (the HIP library reads no environment).
_EXTRA_CFLAGS = os.environ.get("DFSS_ORACLE_EXTRA_CFLAGS", "").split()
_LIB = os.path.join(_HERE, "liboracle" + ("_instrumented" if _EXTRA_CFLAGS else "") + ".so")

_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(dtype=np.uint16, flags="C_CONTIGUOUS")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps the fp32 dot
    product a plain multiply-then-add sequence, as the oracle's header states."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=native", "-ffp-contract=off", "-fopenmp", "-fPIC",
               "-shared", "-std=c11", "-Wall", "-Wextra", *_EXTRA_CFLAGS, "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c_int, c_float, c_double = ctypes.c_int, ctypes.c_float, ctypes.c_double
        L.oracle_scores.argtypes = [_f32p, _f32p, c_int, c_int, c_int, c_float, _f32p]
        L.oracle_scores.restype = None
        L.oracle_prune.argtypes = [_f32p, c_int, c_int, c_int, c_int, _u8p, _f32p, _i32p]
        L.oracle_prune.restype = c_int
        L.oracle_encode_meta.argtypes = [_i32p, c_int, c_int, _u16p]
        L.oracle_encode_meta.restype = c_int
        L.oracle_decode_meta.argtypes = [_u16p, c_int, c_int, _i32p]
        L.oracle_decode_meta.restype = c_int
        L.oracle_encode_meta_f32.argtypes = [_i32p, c_int, c_int, _u16p]
        L.oracle_encode_meta_f32.restype = c_int
        L.oracle_decode_meta_f32.argtypes = [_u16p, c_int, c_int, _i32p]
        L.oracle_decode_meta_f32.restype = c_int
        L.oracle_softmax_kept.argtypes = [_f32p, c_int, c_int, _f32p]
        L.oracle_softmax_kept.restype = None
        L.oracle_spmm.argtypes = [_f32p, _i32p, _f32p, c_int, c_int, c_int, _f32p]
        L.oracle_spmm.restype = None
        L.oracle_round_bf16_array.argtypes = [_f32p, ctypes.c_size_t, _f32p]
        L.oracle_round_bf16_array.restype = None
        L.oracle_attention_batched.argtypes = [_f32p, _f32p, _f32p, c_int, c_int, c_int, c_int,
                                               c_int, c_int, c_float, c_int, _f32p]
        L.oracle_attention_batched.restype = c_int
        L.oracle_attention_bias_batched.argtypes = [_f32p, _f32p, _f32p, _f32p, c_int, c_int, c_int, c_int,
                                                    c_int, c_int, c_int, c_float, c_int, _f32p]
        L.oracle_attention_bias_batched.restype = c_int
        L.oracle_attention_masked_batched.argtypes = [_f32p, _f32p, _f32p, ctypes.c_void_p, c_int, ctypes.c_void_p,
                                                      ctypes.c_void_p, c_int, c_int, c_int, c_int, c_int, c_int,
                                                      c_int, c_float, c_int, _f32p]
        L.oracle_attention_masked_batched.restype = c_int
        L.oracle_apply_block_mask.argtypes = [_f32p, c_int, c_int, _u8p, c_int]
        L.oracle_apply_block_mask.restype = c_int
        L.oracle_add_key_bias.argtypes = [_f32p, c_int, c_int, _f32p]
        L.oracle_add_key_bias.restype = None
        L.oracle_add_mask.argtypes = [_f32p, c_int, c_int, _f32p]
        L.oracle_add_mask.restype = None
        L.oracle_causal_mask.argtypes = [c_int, c_int, _f32p]
        L.oracle_causal_mask.restype = c_int
        L.oracle_attention_backward.argtypes = [_f32p, _f32p, _f32p, _f32p, _f32p, _i32p, c_int, c_int, c_int, c_int,
                                                c_float, _f32p, _f32p, _f32p, ctypes.c_void_p]
        L.oracle_attention_backward.restype = None
        L.oracle_num_threads.argtypes = []
        L.oracle_num_threads.restype = c_int
        L.oracle_quality_p.argtypes = [_f32p, _u8p, c_int, c_int, c_double]
        L.oracle_quality_p.restype = c_double
        _lib = L
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def scores(Q, K, scale):
    """S = scale * Q K^T for one head, fp32 sequential accumulation (Eq. 1)."""
    Q, K = _f32(Q), _f32(K)
    Lq, d = Q.shape
    Lk, d2 = K.shape
    assert d == d2
    S = np.empty((Lq, Lk), np.float32)
    _load().oracle_scores(Q, K, Lq, Lk, d, float(scale), S)
    return S


def add_key_bias(S, bias):
    """S + bias[None, :] in fp32 (additive key mask applied before the N:M comparison)."""
    S = _f32(S).copy()
    bias = _f32(bias)
    Lq, Lk = S.shape
    assert bias.shape == (Lk,)
    _load().oracle_add_key_bias(S, Lq, Lk, bias)
    return S


def add_mask(S, mask):
    """S + mask, both [Lq, Lk] (fp32 add; -inf hides a key from a query)."""
    S = _f32(S).copy()
    mask = _f32(mask)
    assert mask.shape == S.shape, mask.shape
    _load().oracle_add_mask(S, S.shape[0], S.shape[1], mask)
    return S


def causal_mask(Lq, Lk):
    """[Lq, Lk] additive mask: 0 where key j <= i + (Lk - Lq) (the queries are the last Lq positions), else -inf."""
    mask = np.empty((Lq, Lk), np.float32)
    if _load().oracle_causal_mask(Lq, Lk, mask) != 0:
        raise ValueError("causal mask needs Lk >= Lq >= 1")
    return mask


def apply_block_mask(S, block_mask, block_size):
    """Scores of blocks the block pattern prunes (block_mask == 0) become -inf (blocked-ELL, App. A.1.2)."""
    S = _f32(S).copy()
    bm = np.ascontiguousarray(block_mask, dtype=np.uint8)
    Lq, Lk = S.shape
    assert bm.shape == (Lq // block_size, Lk // block_size)
    rc = _load().oracle_apply_block_mask(S, Lq, Lk, bm, int(block_size))
    if rc != 0:
        raise ValueError(f"oracle_apply_block_mask failed rc={rc}")
    return S


def prune(S, N, M):
    """N:M selection on one head's scores -> (mask u8 [Lq,Lk], vals f32 [Lq,Lc], kidx i32 [Lq,Lc])."""
    S = _f32(S)
    Lq, Lk = S.shape
    Lc = Lk // M * N
    mask = np.empty((Lq, Lk), np.uint8)
    vals = np.empty((Lq, Lc), np.float32)
    kidx = np.empty((Lq, Lc), np.int32)
    rc = _load().oracle_prune(S, Lq, Lk, N, M, mask, vals, kidx)
    if rc != 0:
        raise ValueError(f"oracle_prune failed rc={rc}")
    return mask, vals, kidx


def encode_meta(kidx, Lk):
    """Key indices of kept entries (2 per run of 4 keys) -> canonical uint16 words [Lq, Lk/16]."""
    kidx = np.ascontiguousarray(kidx, dtype=np.int32)
    Lq = kidx.shape[0]
    meta = np.empty((Lq, Lk // 16), np.uint16)
    rc = _load().oracle_encode_meta(kidx, Lq, Lk, meta)
    if rc != 0:
        raise ValueError(f"oracle_encode_meta failed rc={rc}")
    return meta


def decode_meta(meta, Lk):
    meta = np.ascontiguousarray(meta, dtype=np.uint16)
    Lq = meta.shape[0]
    kidx = np.empty((Lq, Lk // 2), np.int32)
    rc = _load().oracle_decode_meta(meta, Lq, Lk, kidx)
    if rc != 0:
        raise ValueError(f"oracle_decode_meta failed rc={rc}")
    return kidx


def encode_meta_f32(kidx, Lk):
    """4-byte mode (1:2 on float data): one kept key per aligned pair -> uint16 words [Lq, Lk/8]."""
    kidx = np.ascontiguousarray(kidx, dtype=np.int32)
    Lq = kidx.shape[0]
    meta = np.empty((Lq, Lk // 8), np.uint16)
    rc = _load().oracle_encode_meta_f32(kidx, Lq, Lk, meta)
    if rc != 0:
        raise ValueError(f"oracle_encode_meta_f32 failed rc={rc}")
    return meta


def decode_meta_f32(meta, Lk):
    meta = np.ascontiguousarray(meta, dtype=np.uint16)
    Lq = meta.shape[0]
    kidx = np.empty((Lq, Lk // 2), np.int32)
    rc = _load().oracle_decode_meta_f32(meta, Lq, Lk, kidx)
    if rc != 0:
        raise ValueError(f"oracle_decode_meta_f32 failed rc={rc}")
    return kidx


def softmax_kept(x):
    x = _f32(x)
    Lq, Lc = x.shape
    P = np.empty_like(x)
    _load().oracle_softmax_kept(x, Lq, Lc, P)
    return P


def spmm(P, kidx, V):
    P, V = _f32(P), _f32(V)
    kidx = np.ascontiguousarray(kidx, dtype=np.int32)
    Lq, Lc = P.shape
    Lk, d = V.shape
    O = np.empty((Lq, d), np.float32)
    _load().oracle_spmm(P, kidx, V, Lq, Lc, d, O)
    return O


def round_bf16(x):
    x = _f32(x)
    y = np.empty_like(x)
    _load().oracle_round_bf16_array(x.reshape(-1), x.size, y.reshape(-1))
    return y


def attention(Q, K, V, N, M, scale, store_bf16=False, key_bias=None, heads_per_batch=1,
              block_mask=None, block_size=64, mask=None, causal=False):
    """Whole forward for [BH, L, d] (or [L, d]) inputs; heads run on host threads.

    key_bias: optional float32 [BH // heads_per_batch, Lk] (or [Lk] for a single head), added to
    the scaled scores before the N:M selection; -inf masks a key.
    block_mask: optional uint8 [Lq // block_size, Lk // block_size] shared by all heads; blocks with a
    zero entry are not part of the attention (their scores count as -inf).
    mask: optional float32 [Lq, Lk] shared by all heads, added like the key bias.  causal=True adds
    causal_mask(Lq, Lk) (on top of ``mask`` if both are given).
    """
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    squeeze = Q.ndim == 2
    if squeeze:
        Q, K, V = Q[None], K[None], V[None]
    BH, Lq, d = Q.shape
    Lk = K.shape[1]
    O = np.empty((BH, Lq, d), np.float32)
    if causal:
        cm = causal_mask(Lq, Lk)
        mask = cm if mask is None else (_f32(mask) + cm).astype(np.float32)
    if key_bias is None and block_mask is None and mask is None:
        rc = _load().oracle_attention_batched(Q, K, V, BH, Lq, Lk, d, N, M, float(scale),
                                              int(bool(store_bf16)), O)
    else:
        kb = bm = m2 = None
        if mask is not None:
            m2 = _f32(mask)
            assert m2.shape == (Lq, Lk), m2.shape
        if key_bias is not None:
            kb = _f32(key_bias)
            if kb.ndim == 1:
                kb = kb[None]
            assert BH % heads_per_batch == 0 and kb.shape == (BH // heads_per_batch, Lk), kb.shape
        if block_mask is not None:
            bm = np.ascontiguousarray(block_mask, dtype=np.uint8)
            assert bm.shape == (Lq // block_size, Lk // block_size), bm.shape
        rc = _load().oracle_attention_masked_batched(
            Q, K, V, kb.ctypes.data if kb is not None else None, int(heads_per_batch),
            m2.ctypes.data if m2 is not None else None,
            bm.ctypes.data if bm is not None else None, int(block_size),
            BH, Lq, Lk, d, N, M, float(scale), int(bool(store_bf16)), O)
    if rc != 0:
        raise ValueError(f"oracle_attention failed rc={rc}")
    return O[0] if squeeze else O


def attention_backward(Q, K, V, dO, P, kidx, scale, return_dS=False):
    """Gradients of one head through the fixed selection: (dQ, dK, dV[, dS]).

    P [Lq, Lc] are the softmax weights of the kept entries and kidx [Lq, Lc] their key indices, both
    from the forward pass (prune + softmax_kept)."""
    Q, K, V, dO, P = _f32(Q), _f32(K), _f32(V), _f32(dO), _f32(P)
    kidx = np.ascontiguousarray(kidx, dtype=np.int32)
    Lq, d = Q.shape
    Lk = K.shape[0]
    Lc = P.shape[1]
    dQ = np.empty((Lq, d), np.float32)
    dK = np.empty((Lk, d), np.float32)
    dV = np.empty((Lk, d), np.float32)
    dS = np.empty((Lq, Lc), np.float32) if return_dS else None
    _load().oracle_attention_backward(Q, K, V, dO, P, kidx, Lq, Lk, Lc, d, float(scale), dQ, dK, dV,
                                      dS.ctypes.data if dS is not None else None)
    return (dQ, dK, dV, dS) if return_dS else (dQ, dK, dV)


def num_threads():
    return int(_load().oracle_num_threads())


def quality_p(S, mask, p):
    """L^p quality of a mask on one head's score matrix (Def. 4.1)."""
    S = _f32(S)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    Lq, Lk = S.shape
    return float(_load().oracle_quality_p(S, mask, Lq, Lk, float(p)))
