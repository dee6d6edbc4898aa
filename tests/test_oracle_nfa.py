"""Pins for the oracle's non-deterministic byte walk (the relation form of the displacement of
a right-linear grammar that is not deterministic)."""

import itertools

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from oracle import displacement as D
from synthetic_inputs.nfa import add_transitions, make_lexer_nfa, nfa_from_dfa
from synthetic_inputs.vocab import vocab_from_tokens


def _bits_to_sets(rows):
    """[S][W] words -> list of sets"""
    S, W = rows.shape
    return [{w * 32 + j for w in range(W) for j in range(32) if (int(rows[q, w]) >> j) & 1}
            for q in range(S)]


def _random_nfa(rng, S, n_sym, density):
    W = (S + 31) // 32
    nfa = np.zeros((256, S, W), np.uint32)
    for b in range(n_sym):
        for q in range(S):
            for x in range(S):
                if rng.random() < density:
                    nfa[b, q, x >> 5] |= np.uint32(1 << (x & 31))
    return nfa


def test_deterministic_automaton_gives_the_byte_walk(cfg1):
    table, vocab = cfg1["table"], cfg1["vocab"]
    S = table.shape[0]
    sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    rel = oracle.nfa_signatures(vocab.tok_bytes, vocab.tok_off, nfa_from_dfa(table))
    assert rel.shape == (vocab.V, S, 1)
    want = np.where((sig != 0) & (np.arange(S)[None, :] != 0), np.uint32(1) << sig.astype(np.uint32), 0)
    assert (rel[:, :, 0] == want).all()


@pytest.mark.parametrize("seed", range(5))
def test_paths_by_brute_force(seed):
    rng = np.random.default_rng(seed)
    S, n_sym = int(rng.integers(2, 7)), 3
    nfa = _random_nfa(rng, S, n_sym, 0.3)
    succ = {(b, q): _bits_to_sets(nfa[b])[q] for b in range(n_sym) for q in range(S)}
    toks = [bytes(w) for n in range(0, 5) for w in itertools.product(range(n_sym), repeat=n)]
    v = vocab_from_tokens(toks)
    rel = oracle.nfa_signatures(v.tok_bytes, v.tok_off, nfa)
    for t, tok in enumerate(toks):
        for q in range(S):
            # every path q = x0 -b1-> x1 ... -bn-> xn, enumerated one by one
            ends = set()
            for path in itertools.product(range(S), repeat=len(tok)):
                prev, ok = q, True
                for b, x in zip(tok, path):
                    if x not in succ[(b, prev)]:
                        ok = False
                        break
                    prev = x
                if ok:
                    ends.add(prev)
            assert _bits_to_sets(rel[t])[q] == ends, (tok, q)


def test_concatenation_is_the_boolean_matrix_product():
    rng = np.random.default_rng(7)
    S = 40   # two words per row
    nfa = _random_nfa(rng, S, 4, 0.05)
    toks = [bytes(rng.integers(0, 4, size=int(rng.integers(0, 5))).astype(np.uint8)) for _ in range(60)]
    pairs = [(toks[i], toks[j]) for i in range(0, 60, 3) for j in range(1, 60, 7)]
    v = vocab_from_tokens(toks + [a + b for a, b in pairs])
    rel = oracle.nfa_signatures(v.tok_bytes, v.tok_off, nfa)

    def dense(r):
        return np.array([[(int(r[q, x >> 5]) >> (x & 31)) & 1 for x in range(S)] for q in range(S)], dtype=np.int64)

    index = {}
    for i, t in enumerate(toks):
        index.setdefault(t, i)
    for k, (a, b) in enumerate(pairs):
        prod = (dense(rel[index[a]]) @ dense(rel[index[b]])) > 0
        assert (dense(rel[len(toks) + k]).astype(bool) == prod).all()
    # pad bits stay clear
    assert (rel[:, :, 1] >> (S - 32) == 0).all()


@pytest.mark.parametrize("seed", range(3))
def test_relation_equals_algorithm_1_on_the_right_linear_grammar(seed):
    """q -> a q' for every q' in nfa[a][q], q -> a where q' is accepting: the displacement of t
    is {((q), (q'))} over the relation plus {((q), ())} where an accepting state is reached."""
    rng = np.random.default_rng(50 + seed)
    S, n_sym = 5, 2
    nfa = _random_nfa(rng, S, n_sym, 0.35)
    accepting = {int(q) for q in range(S) if rng.random() < 0.4}
    prods = []
    for b in range(n_sym):
        for q, succ in enumerate(_bits_to_sets(nfa[b])):
            for x in succ:
                prods.append((q, b, (x,)))
                if x in accepting:
                    prods.append((q, b, ()))
    assert D.stack_adjacency(prods) == set()
    toks = [bytes(w) for n in range(1, 5) for w in itertools.product(range(n_sym), repeat=n)]
    v = vocab_from_tokens(toks)
    rel = oracle.nfa_signatures(v.tok_bytes, v.tok_off, nfa)
    for t, tok in enumerate(toks):
        want = set()
        for q, ends in enumerate(_bits_to_sets(rel[t])):
            for x in ends:
                want.add(((q,), (x,)))
                if x in accepting:
                    want.add(((q,), ()))
        assert D.displacement(tuple(tok), prods) == frozenset(want)


def test_generators():
    table, _ = si.make_lexer_dfa(3, 128)
    base = nfa_from_dfa(table)
    assert base.shape == (256, 128, 4) and base.dtype == np.uint32
    per_pair = np.array([[sum(bin(int(x)).count("1") for x in base[b, q]) for q in range(128)]
                         for b in range(256)])
    assert per_pair.max() == 1 and per_pair[:, 0].sum() == 0
    more = add_transitions(base, 5, 0.25)
    assert ((more & base) == base).all()
    grown = sum(bin(int(x)).count("1") for x in (more ^ base).reshape(-1))
    assert 0.15 * per_pair.sum() < grown < 0.30 * per_pair.sum()
    assert (make_lexer_nfa(9, 128) == make_lexer_nfa(9, 128)).all()
