"""Pins for the general displacement computation (Algorithm 1, Appendix B,
Appendix C) and for the reading that, on right-linear grammars, displacement
equivalence is equality of byte-walk signatures."""

import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import displacement as D
from synthetic_inputs.vocab import vocab_from_tokens

from golden_fixtures import read_fig3 as _read_fig3


def test_figure3_worked_example():
    token, prods, steps, res_i, res_o = _read_fig3()
    assert D.displacement(token, prods) == frozenset({(res_i, res_o)})
    # every prefix of the token reproduces the sub-figure's stacks
    for n, (ch, si, so) in enumerate(steps, start=1):
        assert token[n - 1] == ch
        assert D.displacement(token[:n], prods) == frozenset({(si, so)})


def test_figure3_backtrack_needs_stack_adjacency():
    token, prods, _, res_i, res_o = _read_fig3()
    adj = D.stack_adjacency(prods)
    assert ("C", "X") in adj and ("B", "C") in adj and ("Z", "J") in adj and ("J", "K") in adj
    assert ("A", "X") not in adj  # A has no unary production
    without_s = [p for p in prods if p[0] != "S"]
    assert D.displacement(token, without_s) == frozenset()          # backtrack pruned
    assert D.displacement(token, without_s, adjacency="all") == frozenset({(res_i, res_o)})


def _random_gnf(rng, n_nt, n_term, n_prod, max_rhs):
    nts = list(range(n_nt))
    prods = set()
    while len(prods) < n_prod:
        A = int(rng.integers(n_nt))
        a = int(rng.integers(n_term))
        k = int(rng.integers(0, max_rhs + 1))
        prods.add((A, a, tuple(int(x) for x in rng.integers(0, n_nt, size=k))))
    return nts, sorted(prods)


@pytest.mark.parametrize("seed", range(8))
def test_unrestricted_algorithm1_equals_equation3(seed):
    """With every pair allowed as stack-adjacent, Algorithm 1 enumerates exactly
    D'_G(t) of Appendix B (Equation 3), computed here by brute force."""
    rng = np.random.default_rng(seed)
    nts, prods = _random_gnf(rng, n_nt=3, n_term=2, n_prod=9, max_rhs=2)
    for n in range(0, 5):
        for tok in itertools.product(range(2), repeat=n):
            got = D.displacement(tok, prods, adjacency="all")
            want = D.restricted_pre_displacement(tok, prods, nts)
            assert got == want, (tok, prods)


@pytest.mark.parametrize("seed", range(8))
def test_single_symbol_slice_equals_equation2(seed):
    """Pairs whose input stack is one symbol never backtrack twice, so the
    adjacency relation cannot prune them: they equal pi(t, (A)) of Equation 2."""
    rng = np.random.default_rng(50 + seed)
    nts, prods = _random_gnf(rng, n_nt=4, n_term=2, n_prod=12, max_rhs=2)
    d = D.delta(prods)
    for n in range(1, 5):
        for tok in itertools.product(range(2), repeat=n):
            got = {(a, b) for (a, b) in D.displacement(tok, prods) if len(a) == 1}
            want = {((A,), beta) for A in nts for beta in D.pi(tok, (A,), d)}
            assert got == want
            # and the restricted result is a subset of the unrestricted one
            assert D.displacement(tok, prods) <= D.displacement(tok, prods, adjacency="all")


def test_stack_adjacency_covers_observed_pops():
    """Simulate the PDA on every short string from the start symbol and record
    which symbol is popped right after a unary production fired with deeper
    stack symbols left: every such pair must be in the computed relation."""
    rng = np.random.default_rng(11)
    total = 0
    for _ in range(8):
        nts, prods = _random_gnf(rng, n_nt=4, n_term=2, n_prod=10, max_rhs=3)
        adj = D.stack_adjacency(prods)
        d = D.delta(prods)
        observed = set()
        frontier = [((0,), None)]  # (stack, symbol whose unary pop exposed the top)
        for _depth in range(5):
            nxt = []
            for stack, exposed_by in frontier:
                if not stack:
                    continue
                top = stack[0]
                if exposed_by is not None:
                    observed.add((exposed_by, top))
                for a in range(2):
                    for beta in d.get((a, top), ()):
                        new = beta + stack[1:]
                        nxt.append((new, top if len(beta) == 0 else None))
            frontier = nxt
        total += len(observed)
        for (y, z) in observed:
            assert (y, z) in adj, ((y, z), prods)
    assert total >= 10, "the simulation should see exposed pops"


@pytest.mark.parametrize("seed", range(6))
def test_right_linear_grammar_partition_equals_walk_partition(seed):
    """A deterministic automaton written as a right-linear grammar: tokens have
    equal displacement sets exactly when they have equal walk signatures, the
    adjacency relation is empty, and each displacement is the set
    {(q, delta*(q,t))} plus {(q, empty)} where the walk ends in an accepting state."""
    rng = np.random.default_rng(200 + seed)
    S = int(rng.integers(3, 8))
    n_sym = 3
    table = np.zeros((S, 256), dtype=np.uint16)
    table[1:, :n_sym] = rng.integers(0, S, size=(S - 1, n_sym))
    accepting = {int(q) for q in range(1, S) if rng.random() < 0.4}
    prods = D.right_linear_grammar(table[:, :n_sym], accepting)
    assert D.stack_adjacency(prods) == set()
    toks = [bytes(w) for n in range(1, 5) for w in itertools.product(range(n_sym), repeat=n)]
    v = vocab_from_tokens(toks)
    sig = oracle.signatures(v.tok_bytes, v.tok_off, table)
    c, _ = oracle.build_classes(sig, v.tok_off)
    disp = [D.displacement(t, prods) for t in toks]
    for i, t in enumerate(toks):
        want = set()
        for q in range(1, S):
            e = int(sig[i][q])
            if e != 0:
                want.add(((q,), (e,)))
                if e in accepting:
                    want.add(((q,), ()))
        assert disp[i] == frozenset(want)
    for a, b in itertools.combinations(range(len(toks)), 2):
        assert (disp[a] == disp[b]) == (c[a] == c[b])


def test_bodies_of_any_length_are_pushed_whole():
    """Section 2.1: beta in delta_G(a, A) iff A -> a beta, whatever the length of beta.  A
    six-symbol body shows up whole on the output stack and is consumed symbol by symbol."""
    prods = [("S", "s", ("A", "B", "C", "A", "B", "C")), ("A", "a", ()), ("B", "b", ()), ("C", "c", ())]
    assert D.displacement("s", prods) == frozenset({(("S",), ("A", "B", "C", "A", "B", "C"))})
    assert D.displacement("sab", prods) == frozenset({(("S",), ("C", "A", "B", "C"))})
    assert D.displacement("sabcabc", prods) == frozenset({(("S",), ())})
    assert D.displacement("sb", prods) == frozenset()
    d = D.delta(prods)
    assert D.pi("sabcabc", ("S",), d) == {()}
