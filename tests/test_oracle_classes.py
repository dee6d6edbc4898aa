"""Pins for the oracle's grouping (Section 3.1 "Pre-Computation"): brute force
over all token pairs, partition invariants, closed-form automata, the
representative rule, Theorem 1's consequence, and Definition 1 (syntactic
congruence) by brute force on tiny automata."""

import itertools

import numpy as np
import pytest

import oracle
from synthetic_inputs.vocab import vocab_from_tokens


def _build(vocab, table):
    sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    c, r = oracle.build_classes(sig, vocab.tok_off)
    return sig, c, r


def check_partition_invariants(c, r, lengths):
    V, C = len(c), len(r)
    assert c.min() == 0 and c.max() == C - 1
    assert len(np.unique(c)) == C                       # every id used
    assert (c[r] == np.arange(C)).all()                 # representative lies in its class
    first = np.full(C, V, dtype=np.int64)
    np.minimum.at(first, c, np.arange(V))
    assert (np.diff(first) > 0).all() and first[0] == 0  # numbered by first appearance
    for k in range(C):
        members = np.flatnonzero(c == k)
        lmin = lengths[members].min()
        assert lengths[r[k]] == lmin                     # byte-wise shortest
        assert r[k] == members[lengths[members] == lmin].min()  # tie: smallest id


def test_pairwise_brute_force_config1(cfg1):
    v, table = cfg1["vocab"], cfg1["table"]
    sig, c, r = _build(v, table)
    V = v.V
    for lo in range(0, V, 256):  # all V^2 pairs, in strips
        eq_sig = (sig[lo:lo + 256, None, :] == sig[None, :, :]).all(axis=2)
        eq_cls = c[lo:lo + 256, None] == c[None, :]
        assert (eq_sig == eq_cls).all()
    check_partition_invariants(c, r, v.lengths)


def test_partition_invariants_lexer(cfg2_small):
    v, table = cfg2_small["vocab"], cfg2_small["table"]
    sig, c, r = _build(v, table)
    check_partition_invariants(c, r, v.lengths)
    # equal class <=> equal signature, checked against each class's first member
    first = {}
    for t in range(v.V):
        k = int(c[t])
        if k in first:
            assert (sig[t] == sig[first[k]]).all()
        else:
            first[k] = t
    heads = sig[[first[k] for k in range(len(r))]]
    assert len(np.unique(heads, axis=0)) == len(r)       # distinct classes differ


def test_identity_automaton_one_class():
    S = 9
    table = np.repeat(np.arange(S, dtype=np.uint16)[:, None], 256, axis=1)
    v = vocab_from_tokens([b"abc", b"d", b"", b"zzzz", b"q"])
    _, c, r = _build(v, table)
    assert (c == 0).all() and list(r) == [2]  # the empty token is the shortest


def test_counter_automaton_classes_are_length_residues():
    S = 6
    table = np.zeros((S, 256), dtype=np.uint16)
    for q in range(1, S):
        table[q, :] = 1 + (q % (S - 1))
    rng = np.random.default_rng(0)
    toks = [rng.integers(0, 256, size=int(rng.integers(1, 30)), dtype=np.uint8).tobytes()
            for _ in range(300)]
    v = vocab_from_tokens(toks)
    _, c, r = _build(v, table)
    res = np.array([len(t) % (S - 1) for t in toks])
    assert len(r) == len(set(res))
    for a, b in itertools.combinations(range(60), 2):
        assert (c[a] == c[b]) == (res[a] == res[b])


def test_trie_automaton_classes_are_distinct_strings():
    """States are the prefixes of the vocabulary: two tokens share a class iff
    they are the same byte string."""
    rng = np.random.default_rng(1)
    toks = [bytes(rng.choice([97, 98, 99], size=int(rng.integers(1, 5))).astype(np.uint8))
            for _ in range(120)]
    prefixes = sorted({t[:k] for t in toks for k in range(1, len(t) + 1)})
    state = {b"": 1}
    for p in prefixes:
        state[p] = len(state) + 1
    S = len(state) + 1
    table = np.zeros((S, 256), dtype=np.uint16)
    for p, q in state.items():
        if p:
            table[state[p[:-1]], p[-1]] = q
    v = vocab_from_tokens(toks)
    _, c, r = _build(v, table)
    assert len(r) == len(set(toks))
    for a, b in itertools.combinations(range(len(toks)), 2):
        assert (c[a] == c[b]) == (toks[a] == toks[b])


def test_duplicates_and_empty_tokens(cfg1):
    table = cfg1["table"]
    v = vocab_from_tokens([b"ab", b"", b"ab", b"{", b"", b"ab"])
    _, c, r = _build(v, table)
    assert c[0] == c[2] == c[5] and c[1] == c[4]
    assert r[c[0]] == 0 and r[c[1]] == 1


def test_theorem1_consequence_token_behaves_like_representative(cfg2_small):
    """From every automaton state a token and its representative reach the same
    state, hence have the same validity (the losslessness claim)."""
    v, table = cfg2_small["vocab"], cfg2_small["table"]
    sig, c, r = _build(v, table)
    assert (sig == sig[r[c]]).all()
    assert ((sig != 0) == (sig[r[c]] != 0)).all()


# ---- Definition 1 (syntactic congruence) by brute force ----------------------

ALPHA = (97, 98, 99)


def _accepts(table, F, word, start=1):
    s = start
    for ch in word:
        s = int(table[s][ch])
    return s in F


def _words(max_len):
    for n in range(max_len + 1):
        for w in itertools.product(ALPHA, repeat=n):
            yield bytes(w)


def _random_small_dfa(rng, S):
    table = np.zeros((S, 256), dtype=np.uint16)
    for q in range(1, S):
        for a in ALPHA:
            table[q, a] = rng.integers(0, S)
    F = {int(q) for q in range(1, S) if rng.random() < 0.5} or {S - 1}
    return table, F


def _is_trim_and_minimal(table, F, S, ctx):
    reach = {1}
    frontier = [1]
    while frontier:
        q = frontier.pop()
        for a in ALPHA:
            n = int(table[q][a])
            if n not in reach:
                reach.add(n)
                frontier.append(n)
    if reach != set(range(S)):
        return False
    for p, q in itertools.combinations(range(S), 2):
        if not any(_accepts(table, F, z, p) != _accepts(table, F, z, q) for z in ctx):
            return False
    return True


@pytest.mark.parametrize("seed", range(6))
def test_equal_class_implies_syntactic_congruence(seed):
    """c[t] == c[u]  =>  for all w, z (bounded): w t z in L  <=>  w u z in L."""
    rng = np.random.default_rng(100 + seed)
    S = int(rng.integers(3, 7))
    table, F = _random_small_dfa(rng, S)
    toks = [w for w in _words(3)]
    v = vocab_from_tokens(toks)
    _, c, _ = _build(v, table)
    ctx = list(_words(3))
    member = {}
    for k in range(int(c.max()) + 1):
        ids = np.flatnonzero(c == k)
        prof = None
        for t in ids:
            p = tuple(_accepts(table, F, w + toks[t] + z) for w in ctx for z in ctx)
            if prof is None:
                prof = p
            assert p == prof
        member[k] = prof


def test_minimal_trim_dfa_classes_equal_syntactic_congruence():
    """For a minimal automaton whose states are all reachable the transition
    monoid is the syntactic monoid: the converse of the above holds too."""
    rng = np.random.default_rng(7)
    found = 0
    ctx = list(_words(4))
    while found < 3:
        S = 4
        table, F = _random_small_dfa(rng, S)
        if not _is_trim_and_minimal(table, F, S, ctx):
            continue
        found += 1
        toks = list(_words(3))
        v = vocab_from_tokens(toks)
        _, c, _ = _build(v, table)
        prof = [tuple(_accepts(table, F, w + t + z) for w in ctx for z in ctx) for t in toks]
        for a, b in itertools.combinations(range(len(toks)), 2):
            assert (c[a] == c[b]) == (prof[a] == prof[b])
