"""Pins for the oracle's engine side over a non-deterministic byte automaton (Section 2.2: a token
may follow iff the extended sequence can still be completed; Section 3.1 "Inference": the engine
sees representatives only).  The engine's state is a set of automaton states."""

import numpy as np
import pytest

import oracle
from synthetic_inputs.nfa import add_transitions, nfa_from_dfa
from synthetic_inputs.vocab import vocab_from_tokens


def _random_nfa(rng, S, n_sym, per_row):
    W = (S + 31) // 32
    nfa = np.zeros((256, S, W), np.uint32)
    for b in range(n_sym):
        for q in range(S):
            for x in rng.integers(0, S, size=rng.poisson(per_row)):
                nfa[b, q, x >> 5] |= np.uint32(1 << (int(x) & 31))
    return nfa


def _unpack(rows, S):
    """[..., W] words -> [..., S] booleans"""
    bits = np.unpackbits(np.ascontiguousarray(rows).view(np.uint8), axis=-1, bitorder="little")
    return bits[..., :S].astype(bool)


def _pack(flags):
    n = flags.shape[-1]
    pad = (-n) % 32
    f = np.concatenate([flags, np.zeros(flags.shape[:-1] + (pad,), bool)], axis=-1)
    return np.packbits(f, axis=-1, bitorder="little").view(np.uint32)


@pytest.mark.parametrize("seed", range(4))
def test_live_states_by_reachability_closure(seed):
    """live = accepting states closed under "has a successor that is live": compared with the
    transitive closure of the one-step relation computed by boolean matrix powers."""
    rng = np.random.default_rng(seed)
    S = int(rng.integers(2, 40))
    nfa = _random_nfa(rng, S, 3, 0.7)
    accept = (rng.random(S) < 0.2).astype(np.uint8)
    step = _unpack(nfa[:3], S).any(axis=0)                      # [S, S]: q -> q' on some byte
    reach = np.eye(S, dtype=bool) | step
    for _ in range(S):
        reach = reach | (reach.astype(np.int32) @ reach.astype(np.int32) > 0)
    want = (reach & accept.astype(bool)[None, :]).any(axis=1)
    assert (oracle.nfa_live_states(nfa, accept).astype(bool) == want).all()


def test_deterministic_automaton_gives_the_deterministic_engine(cfg1):
    """One-state sets over a deterministic automaton: masks and advances are those of the
    deterministic engine (the reject state corresponds to the empty set)."""
    table, vocab = cfg1["table"], cfg1["vocab"]
    S = table.shape[0]
    rng = np.random.default_rng(5)
    accept = (rng.random(S) < 0.4).astype(np.uint8)
    accept[0] = 0
    sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    c, r = oracle.build_classes(sig, vocab.tok_off)
    C = len(r)
    nfa = nfa_from_dfa(table)
    rel = oracle.nfa_signatures(vocab.tok_bytes, vocab.tok_off, nfa)
    live_d = oracle.live_states(table, accept)
    live_n = oracle.nfa_live_states(nfa, accept)
    assert (live_d[1:] == live_n[1:]).all()
    sm_d = oracle.state_masks(sig[r], live_d)
    sm_n = oracle.nfa_state_masks(rel[r], live_n)
    assert (sm_d[1:] == sm_n[1:]).all() and not sm_n[0].any()
    B = 50
    states = rng.integers(1, S, size=B).astype(np.int32)
    sets = np.zeros((B, 1), np.uint32)
    sets[np.arange(B), 0] = np.uint32(1) << states.astype(np.uint32)
    assert (oracle.nfa_class_masks(sm_n, C, sets) == oracle.class_masks(sm_d, C, states)).all()
    tok = rng.integers(0, vocab.V, size=B).astype(np.int32)
    nxt_d = oracle.advance_states(sig[r], c, tok, states)
    nxt_n = oracle.nfa_advance_states(rel[r], c, tok, sets)
    want = np.where(nxt_d > 0, np.uint32(1) << np.maximum(nxt_d, 0).astype(np.uint32), 0).astype(np.uint32)
    assert (nxt_n[:, 0] == want).all()


@pytest.mark.parametrize("seed", range(5))
def test_masks_and_advances_equal_the_definition_on_every_token(seed):
    """Losslessness (Theorem 1) for state sets, by brute force over the whole vocabulary: the
    class mask expanded to tokens is the token-level mask computed from each token's own relation
    (allowed iff some state of the set reaches a live state on the token's bytes), and advancing
    on the representative equals advancing on the token itself."""
    rng = np.random.default_rng(100 + seed)
    S = int(rng.choice([3, 17, 33, 70]))
    nfa = _random_nfa(rng, S, 4, 0.9)
    toks = [bytes(rng.integers(0, 4, size=int(n)).astype(np.uint8)) for n in rng.integers(0, 6, size=400)]
    vocab = vocab_from_tokens(toks)
    W = (S + 31) // 32
    rel = oracle.nfa_signatures(vocab.tok_bytes, vocab.tok_off, nfa)          # [V, S, W]
    c, r = oracle.build_classes(np.ascontiguousarray(rel).view(np.uint16).reshape(vocab.V, -1), vocab.tok_off)
    C = len(r)
    accept = (rng.random(S) < 0.3).astype(np.uint8)
    live = oracle.nfa_live_states(nfa, accept).astype(bool)
    sm = oracle.nfa_state_masks(rel[r], live.astype(np.uint8))
    B = 40
    members = rng.random((B, S)) < rng.choice([0.05, 0.3, 0.9], size=(B, 1))
    members[0] = False                                                       # an empty set
    sets = _pack(members)
    cls = oracle.nfa_class_masks(sm, C, sets)
    got_tok = _unpack(oracle.expand_mask(cls, c, C).view(np.uint32), vocab.V)
    R = _unpack(rel, S)                                                      # [V, S, S]
    reach_live = (R & live[None, None, :]).any(axis=2)                        # [V, S]: from q, t reaches a live state
    want_tok = (members[:, None, :] & reach_live[None, :, :]).any(axis=2)    # [B, V]
    assert (got_tok == want_tok).all()
    tok = rng.integers(0, vocab.V, size=B).astype(np.int32)
    tok[3] = -1
    tok[4] = vocab.V
    nxt = _unpack(oracle.nfa_advance_states(rel[r], c, tok, sets), S)
    for b in range(B):
        if 0 <= tok[b] < vocab.V:
            want = (members[b][:, None] & R[tok[b]]).any(axis=0)
        else:
            want = np.zeros(S, bool)
        assert (nxt[b] == want).all(), b
    assert _pack(nxt[:, :S]).shape == (B, W)
