"""Pins of the oracle's engine-side functions for a deterministic byte automaton (paper
Section 2.2: a token is allowed iff the extended sequence is still a prefix of the language;
Section 3.1 "Inference": the engine works on the representatives only).  Everything here is
checked against the definitions by brute force or against closed forms, on the CPU."""

import itertools

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from synthetic_inputs.vocab import vocab_from_tokens


def _bit(row, k):
    return (int(np.uint32(row[k >> 5])) >> (k & 31)) & 1


def _run(table, q, bs):
    for b in bs:
        q = int(table[q, b])
    return q


def test_live_states_closed_forms():
    S = 6
    table = np.zeros((S, 256), dtype=np.uint16)
    # 1 -a-> 2 -a-> 3 (accepting), 4 -a-> 4 (a loop that never accepts), everything else -> 0
    table[1, 97], table[2, 97], table[4, 97] = 2, 3, 4
    table[5, :] = 5
    accept = np.zeros(S, dtype=np.uint8)
    accept[3] = 1
    assert list(oracle.live_states(table, accept)) == [0, 1, 1, 1, 0, 0]
    assert oracle.live_states(table, np.ones(S, dtype=np.uint8)).all()
    assert not oracle.live_states(table, np.zeros(S, dtype=np.uint8)).any()


@pytest.mark.parametrize("seed", range(5))
def test_live_states_by_enumeration(seed):
    """live[q] <=> some byte string of length < S over the used alphabet reaches F."""
    rng = np.random.default_rng(seed)
    S, alphabet = 5, [0, 1]
    table = np.zeros((S, 256), dtype=np.uint16)
    table[:, alphabet] = rng.integers(0, S, size=(S, 2))
    table[:, 2:] = table[:, [0]]  # the other bytes behave like byte 0: no new targets
    accept = (rng.random(S) < 0.3).astype(np.uint8)
    live = oracle.live_states(table, accept)
    for q in range(S):
        reach = any(accept[_run(table, q, w)] for n in range(S) for w in itertools.product(alphabet, repeat=n))
        assert bool(live[q]) == reach


def _tiny_setup(seed, S=7, n_tokens=40, alphabet=(97, 98, 99)):
    rng = np.random.default_rng(seed)
    table = np.zeros((S, 256), dtype=np.uint16)
    for b in alphabet:
        table[1:, b] = rng.integers(0, S, size=S - 1)  # state 0 absorbs
    toks = [bytes(rng.choice(alphabet, size=int(rng.integers(1, 4)))) for _ in range(n_tokens)]
    vocab = vocab_from_tokens(toks)
    accept = (rng.random(S) < 0.35).astype(np.uint8)
    accept[0] = 0
    sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    c, r = oracle.build_classes(sig, vocab.tok_off)
    return table, vocab, toks, accept, sig, c, r


@pytest.mark.parametrize("seed", range(6))
def test_class_mask_matches_the_definition_of_logit_masking(seed):
    """Section 2.2 by brute force: token t is allowed after a prefix that left the automaton
    in state q iff q.t.z is accepted for some continuation z - and the class-level mask,
    expanded through c, says exactly that for every token."""
    table, vocab, toks, accept, sig, c, r = _tiny_setup(seed)
    S, C = table.shape[0], len(r)
    alphabet = (97, 98, 99)
    live = oracle.live_states(table, accept)
    sm = oracle.state_masks(sig[r], live)
    for q in range(S):
        cls = oracle.class_masks(sm, C, np.array([q], dtype=np.int32))
        tokbits = oracle.expand_mask(cls, c, C)[0]
        for t, bs in enumerate(toks):
            after = _run(table, q, bs)
            extendable = any(accept[_run(table, after, z)] for n in range(S)
                             for z in itertools.product(alphabet, repeat=n))
            assert _bit(tokbits, t) == int(extendable), (q, t)


def test_state_masks_closed_forms():
    S, C = 9, 70
    live = (np.arange(S) % 2).astype(np.uint8)
    ident = np.tile(np.arange(S, dtype=np.uint16), (C, 1))  # every representative maps q -> q
    sm = oracle.state_masks(ident, live)
    assert sm.shape == (S, 3)
    for q in range(S):
        bits = [_bit(sm[q], k) for k in range(96)]
        assert bits[:C] == [int(live[q])] * C and bits[C:] == [0] * (96 - C)  # pad bits are 0
    const = np.full((C, S), 3, dtype=np.uint16)
    const[5] = 4  # class 5 always ends in a dead state
    sm = oracle.state_masks(const, live)
    assert all(_bit(sm[q], k) == (0 if k == 5 else 1) for q in range(S) for k in range(C))


def test_class_masks_rows_and_bad_states():
    sm = np.arange(12, dtype=np.int32).reshape(4, 3) + 100
    out = oracle.class_masks(sm, 70, np.array([2, 0, -1, 4, 3], dtype=np.int32))
    assert (out[0] == sm[2]).all() and (out[1] == sm[0]).all() and (out[4] == sm[3]).all()
    assert not out[2].any() and not out[3].any()


def test_engine_on_representatives_follows_the_token_sequence(cfg1):
    """Theorem 1 in action on the tiny configuration: feeding the engine r[c[t]] instead of t
    leaves it in the same automaton state after every step, and its expanded mask equals the
    mask computed token by token on the full vocabulary."""
    v, table = cfg1["vocab"], cfg1["table"]
    S = table.shape[0]
    sig = oracle.signatures(v.tok_bytes, v.tok_off, table)
    c, r = oracle.build_classes(sig, v.tok_off)
    C = len(r)
    rng = np.random.default_rng(3)
    accept = (rng.random(S) < 0.4).astype(np.uint8)
    accept[0] = 0
    live = oracle.live_states(table, accept)
    sig_rep = sig[r]
    sm = oracle.state_masks(sig_rep, live)
    B, steps = 8, 12
    states = rng.integers(1, S, size=B).astype(np.int32)
    direct = states.copy()
    for _ in range(steps):
        cls = oracle.class_masks(sm, C, states)
        tokbits = oracle.expand_mask(cls, c, C)
        for b in range(B):
            want = live[sig[:, direct[b]]]  # token-level mask straight from the definition
            got = np.unpackbits(tokbits[b].view(np.uint8), bitorder="little")[:v.V]
            assert (got == want).all()
        tok = rng.integers(0, v.V, size=B).astype(np.int32)
        states = oracle.advance_states(sig_rep, c, tok, states)
        direct = np.array([_run(table, int(direct[b]), v.token(int(tok[b]))) for b in range(B)],
                          dtype=np.int32)
        assert (states == direct).all()


def test_advance_states_range_checks():
    sig_rep = np.array([[0, 2, 1], [0, 0, 2]], dtype=np.uint16)  # C=2, S=3
    c = np.array([0, 1, 1, 0], dtype=np.int32)
    tok = np.array([0, 1, 4, -1, 3, 2], dtype=np.int32)
    states = np.array([1, 2, 1, 1, 3, -1], dtype=np.int32)
    assert list(oracle.advance_states(sig_rep, c, tok, states)) == [2, 2, -1, -1, -1, -1]


def test_representative_vocabulary_is_the_list_of_their_byte_strings(cfg1):
    """The vocabulary E the engine is given: token r[k]'s bytes for every class k, in class order."""
    from synthetic_inputs.vocab import vocab_from_tokens
    vocab = cfg1["vocab"]
    sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, cfg1["table"])
    _c, r = oracle.build_classes(sig, vocab.tok_off)
    rep_bytes, rep_off = oracle.representative_vocabulary(vocab.tok_bytes, vocab.tok_off, r)
    want = vocab_from_tokens([vocab.token(int(t)) for t in r])
    assert (rep_off == want.tok_off).all() and (rep_bytes == want.tok_bytes).all()
    # ids may repeat, be out of range (an empty string), or select nothing
    ids = np.array([5, 5, -1, vocab.V, 0, 7], dtype=np.int32)
    b, o = oracle.representative_vocabulary(vocab.tok_bytes, vocab.tok_off, ids)
    toks = [vocab.token(5), vocab.token(5), b"", b"", vocab.token(0), vocab.token(7)]
    assert o.tolist() == np.cumsum([0] + [len(t) for t in toks]).tolist() and b.tobytes() == b"".join(toks)
