"""Pins for the oracle's per-step path (Section 3.1 "Inference", Figure 1;
Section 2.2 logit masking): special masks, popcount identities, end-to-end
losslessness against validity computed token by token, bit-preservation of
allowed logits, idempotence, and the token -> representative map."""

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from synthetic_inputs.configs import f32_to_bf16_bits, words_for


def _bits_to_bool(words, n):
    u = np.ascontiguousarray(words).view(np.uint32)
    return np.unpackbits(u.view(np.uint8), bitorder="little").reshape(u.shape[0], -1)[:, :n].astype(bool)


def _bool_to_bits(b):
    B, n = b.shape
    pad = np.zeros((B, words_for(n) * 32), dtype=bool)
    pad[:, :n] = b
    return np.packbits(pad, axis=1, bitorder="little").view(np.uint32).reshape(B, -1).view(np.int32)


@pytest.fixture(scope="module")
def built(cfg2_small):
    v, table = cfg2_small["vocab"], cfg2_small["table"]
    sig = oracle.signatures(v.tok_bytes, v.tok_off, table)
    c, r = oracle.build_classes(sig, v.tok_off)
    return v, table, sig, c, r


def test_all_ones_and_all_zero_masks(built):
    v, _, _, c, r = built
    C, V = len(r), v.V
    ones = np.full((2, words_for(C)), -1, dtype=np.int32)
    out = oracle.expand_mask(ones, c, C)
    assert _bits_to_bool(out, V).all()
    full = _bits_to_bool(out, words_for(V) * 32)
    assert not full[:, V:].any()  # pad bits are zero
    zeros = np.zeros((2, words_for(C)), dtype=np.int32)
    assert (oracle.expand_mask(zeros, c, C) == 0).all()


def test_identity_class_map_copies_mask():
    V = 77
    c = np.arange(V, dtype=np.int32)
    rng = np.random.default_rng(0)
    m = rng.random((3, V)) < 0.5
    out = oracle.expand_mask(_bool_to_bits(m), c, V)
    assert (_bits_to_bool(out, V) == m).all()


def test_pad_bits_of_input_are_ignored(built):
    v, _, _, c, r = built
    C = len(r)
    rng = np.random.default_rng(1)
    m = rng.random((4, C)) < 0.5
    a = _bool_to_bits(m)
    b = a.copy()
    if C % 32:
        b[:, -1] = (b[:, -1].view(np.uint32) | (np.uint32(0xFFFFFFFF) << np.uint32(C % 32))).view(np.int32)
    assert (oracle.expand_mask(a, c, C) == oracle.expand_mask(b, c, C)).all()


def test_popcount_identities(built):
    v, _, _, c, r = built
    C, V = len(r), v.V
    sizes = np.bincount(c, minlength=C)
    rng = np.random.default_rng(2)
    for k in rng.integers(0, C, size=5):
        m = np.zeros((1, C), dtype=bool)
        m[0, k] = True
        out = _bits_to_bool(oracle.expand_mask(_bool_to_bits(m), c, C), V)
        assert out.sum() == sizes[k] and out[0, c == k].all()
    m = rng.random((6, C)) < 0.5
    out = _bits_to_bool(oracle.expand_mask(_bool_to_bits(m), c, C), V)
    assert (out.sum(axis=1) == (m * sizes[None, :]).sum(axis=1)).all()


def test_lossless_end_to_end(built):
    """For automaton state q: the mask computed on the representatives only and
    then expanded equals the mask computed token by token (Figure 1(b))."""
    v, table, sig, c, r = built
    C, V = len(r), v.V
    rng = np.random.default_rng(3)
    states = rng.integers(0, table.shape[0], size=16)
    cls_valid = np.stack([sig[r, q] != 0 for q in states])      # engine checks one token per class
    tok_valid = np.stack([sig[:, q] != 0 for q in states])      # naive: every token
    out = oracle.expand_mask(_bool_to_bits(cls_valid), c, C)
    assert (_bits_to_bool(out, V) == tok_valid).all()


SPECIAL_F32 = np.array([0x7FC00001, 0xFFC12345, 0x80000000, 0x00000000, 0x7F800000, 0xFF800000,
                        0x00000001, 0x807FFFFF, 0x7F7FFFFF, 0xFF7FFFFF], dtype=np.uint32)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_apply_mask_preserves_allowed_bits_and_is_idempotent(dtype):
    rng = np.random.default_rng(4)
    B, V = 5, 203
    x = rng.standard_normal((B, V)).astype(np.float32)
    raw = x.view(np.uint32).copy()
    raw[:, :len(SPECIAL_F32)] = SPECIAL_F32  # NaN payloads, -0, +-inf, subnormals, max finite
    raw[:, 100:100 + len(SPECIAL_F32)] = SPECIAL_F32
    allow = rng.random((B, V)) < 0.5
    allow[:, :len(SPECIAL_F32)] = True
    allow[:, 100:100 + len(SPECIAL_F32)] = False
    bits = _bool_to_bits(allow)
    if dtype == "f32":
        logits, ninf = raw, np.uint32(0xFF800000)
    else:
        logits, ninf = (raw >> 16).astype(np.uint16), np.uint16(0xFF80)
    out = oracle.apply_mask(logits, bits, dtype)
    assert (out[allow] == logits[allow]).all()
    assert (out[~allow] == ninf).all()
    assert (oracle.apply_mask(out, bits, dtype) == out).all()
    # as floats: the pattern really is minus infinity
    if dtype == "f32":
        assert np.isneginf(out.view(np.float32)[~allow]).all()
    else:
        assert np.isneginf((out.astype(np.uint32) << 16).view(np.float32)[~allow]).all()


def test_apply_mask_respects_row_stride():
    rng = np.random.default_rng(5)
    B, V, stride = 3, 50, 64
    logits = f32_to_bf16_bits(rng.standard_normal((B, stride)).astype(np.float32)).reshape(B, stride)
    allow = rng.random((B, V)) < 0.3
    out = oracle.apply_mask(logits, _bool_to_bits(allow), "bf16", V=V)
    assert (out[:, V:] == logits[:, V:]).all()
    assert (out[:, :V][~allow] == 0xFF80).all() and (out[:, :V][allow] == logits[:, :V][allow]).all()


def test_map_to_rep(built):
    v, _, _, c, r = built
    rng = np.random.default_rng(6)
    tok = rng.integers(0, v.V, size=300).astype(np.int32)
    out = oracle.map_to_rep(tok, c, r)
    assert (out == r[c[tok]]).all()
    assert (oracle.map_to_rep(out, c, r) == out).all()   # idempotent
    assert (c[out] == c[tok]).all()
    bad = np.array([-1, v.V, 5], dtype=np.int32)
    assert list(oracle.map_to_rep(bad, c, r)[:2]) == [-1, -1]


def test_bf16_rounding_of_generator():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38], dtype=np.float32)
    got = f32_to_bf16_bits(x)
    # 1.00390625 = 0x3F808000 is a tie -> even (0x3F80); 1.01171875 = 0x3F818000 tie -> 0x3F82
    assert list(got[:4]) == [0x3F80, 0x3F80, 0x3F82, 0xC020]


def test_adjust_class_count_hits_target(built):
    _, _, _, c, _ = built
    for target in (len(np.unique(c)) // 2, len(np.unique(c)) + 37):
        c2, r2 = si.adjust_class_count(c, target)
        assert len(r2) == target and len(np.unique(c2)) == target
        assert (c2[r2] == np.arange(target)).all()
