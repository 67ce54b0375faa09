"""Pins of the oracle's 4-byte mode (float data, 1:2 selection; Sec. 2.3, App. A.1.1) against
things other than itself: the two codes the paper prints, the metadata size it states, the
relation to the 2-byte format (a float is two 2-byte slots, so the float-mode words must equal
the 2-byte words of the "both slots of the kept element" selection), brute force, and planted
mistakes.  None of these needs a GPU.
"""
import numpy as np
import pytest

import oracle
from conftest import read_golden


def _rng(seed):
    return np.random.default_rng(seed)


def test_only_the_two_printed_codes_occur():
    gold = read_golden("meta_codes.txt")
    c4 = int(gold["keep_slots_0_1"], 16)
    ce = int(gold["keep_slots_2_3"], 16)
    # keep the first element of every pair / the second of every pair
    first = np.arange(0, 32, 2, dtype=np.int32)[None]
    second = first + 1
    assert np.all(oracle.encode_meta_f32(first, 32) == c4 * 0x1111)
    assert np.all(oracle.encode_meta_f32(second, 32) == ce * 0x1111)
    r = _rng(3)
    S = r.standard_normal((32, 256)).astype(np.float32)
    _, _, kidx = oracle.prune(S, 1, 2)
    meta = oracle.encode_meta_f32(kidx, 256)
    codes = {int((w >> (4 * k)) & 0xF) for w in meta.reshape(-1) for k in range(4)}
    assert codes == {c4, ce}


def test_code_of_pair_k_sits_at_bits_4k():
    """App. A.1.2: the k-th of four consecutive codes occupies bits [4k, 4k+3]."""
    gold = read_golden("meta_codes.txt")
    c4 = int(gold["keep_slots_0_1"], 16)
    ce = int(gold["keep_slots_2_3"], 16)
    for pair in range(8):
        kidx = np.arange(0, 16, 2, dtype=np.int32)[None].copy()
        kidx[0, pair] += 1
        meta = oracle.encode_meta_f32(kidx, 16)[0]
        for p in range(8):
            code = (int(meta[p // 4]) >> (4 * (p % 4))) & 0xF
            assert code == (ce if p == pair else c4)


def test_size_is_one_sixteenth_of_the_dense_bits():
    gold = read_golden("meta_codes.txt")
    Lq, Lk = 16, 128
    r = _rng(4)
    S = r.standard_normal((Lq, Lk)).astype(np.float32)
    _, vals, kidx = oracle.prune(S, 1, 2)
    meta = oracle.encode_meta_f32(kidx, Lk)
    dense_bits = Lq * Lk * 32
    assert meta.nbytes * 8 / dense_bits == float(gold["meta_fraction_of_dense_bits"])
    # Sec. 3.4: n^2 * 32 bit -> n^2/2 * 32 bit of values + n^2/16 * 32 bit of metadata
    assert (vals.nbytes * 8 + meta.nbytes * 8) / dense_bits == float(gold["footprint_fraction"])


def test_equals_the_two_byte_format_on_the_slot_view():
    """A float occupies two 2-byte slots: viewing a row of Lk floats as 2*Lk slots and keeping both
    slots of every kept float is a 2:4 selection on slots, whose 2-byte words must be the same."""
    r = _rng(5)
    Lq, Lk = 8, 64
    S = r.standard_normal((Lq, Lk)).astype(np.float32)
    _, _, kidx = oracle.prune(S, 1, 2)
    slots = np.stack([2 * kidx, 2 * kidx + 1], axis=-1).reshape(Lq, Lk).astype(np.int32)
    assert np.array_equal(oracle.encode_meta_f32(kidx, Lk), oracle.encode_meta(slots, 2 * Lk))


def test_round_trip_and_brute_force():
    r = _rng(6)
    Lq, Lk = 12, 40
    S = r.integers(-3, 4, size=(Lq, Lk)).astype(np.float32)     # many ties
    mask, vals, kidx = oracle.prune(S, 1, 2)
    # brute force: the larger of each aligned pair, the first on a tie
    for i in range(Lq):
        for p in range(Lk // 2):
            a, b = S[i, 2 * p], S[i, 2 * p + 1]
            want = 2 * p + (1 if b > a else 0)
            assert kidx[i, p] == want
            assert vals[i, p] == max(a, b)
    meta = oracle.encode_meta_f32(kidx, Lk)
    back = oracle.decode_meta_f32(meta, Lk)
    assert np.array_equal(back, kidx)
    dense = np.zeros_like(S)
    np.put_along_axis(dense, back, vals, axis=1)
    assert np.array_equal(dense, S * mask)


def test_bad_inputs_are_rejected():
    kidx = np.arange(0, 16, 2, dtype=np.int32)[None].copy()
    kidx[0, 3] = 9                        # a key of another pair
    with pytest.raises(ValueError):
        oracle.encode_meta_f32(kidx, 16)
    with pytest.raises(ValueError):       # 0x8 = slots {0, 2}: not one element
        oracle.decode_meta_f32(np.array([[0x4448, 0x4444]], np.uint16), 16)
    with pytest.raises(ValueError):
        oracle.encode_meta_f32(np.zeros((1, 6), np.int32), 12)


def test_planted_mistakes_fail_the_pins():
    """A swapped element order (code of element 0 <-> element 1) or a reversed nibble order must
    differ from the pinned words."""
    gold = read_golden("meta_codes.txt")
    c4 = int(gold["keep_slots_0_1"], 16)
    ce = int(gold["keep_slots_2_3"], 16)
    kidx = np.array([[0, 2, 4, 7]], np.int32)
    good = int(oracle.encode_meta_f32(kidx, 8)[0, 0])
    assert good == (c4 | c4 << 4 | c4 << 8 | ce << 12)
    swapped = ce | ce << 4 | ce << 8 | c4 << 12
    reversed_ = ce | c4 << 4 | c4 << 8 | c4 << 12
    assert good != swapped and good != reversed_


def test_whole_path_keeps_fp32_scores():
    """In the 4-byte mode nothing is rounded to bfloat16: the path on float inputs equals
    softmax over the larger of each pair, in double precision, to fp32 accuracy."""
    r = _rng(8)
    Lq, Lk, d = 16, 48, 32
    Q = r.standard_normal((Lq, d)).astype(np.float32)
    K = r.standard_normal((Lk, d)).astype(np.float32)
    V = r.standard_normal((Lk, d)).astype(np.float32)
    scale = 1 / np.sqrt(d)
    O = oracle.attention(Q, K, V, 1, 2, scale, store_bf16=False)
    S = (Q.astype(np.float64) @ K.astype(np.float64).T) * scale
    Sp = S.reshape(Lq, Lk // 2, 2)
    sel = Sp.argmax(-1)
    kept = np.take_along_axis(Sp, sel[..., None], -1)[..., 0]
    P = np.exp(kept - kept.max(-1, keepdims=True))
    P /= P.sum(-1, keepdims=True)
    Vsel = V.astype(np.float64).reshape(Lk // 2, 2, d)[np.arange(Lk // 2)[None, :], sel]   # [Lq, Lk/2, d]
    want = np.einsum("qp,qpd->qd", P, Vsel)
    assert np.abs(O - want).max() < 2e-6
