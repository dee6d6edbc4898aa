"""Seeded non-deterministic byte automata as bit matrices: nfa[b][q] = bit row (uint32 words,
bit q' & 31 of word q' >> 5) of the states that may follow state q on byte b.

Inputs only: nothing here reads a token or follows a path."""

from __future__ import annotations

import numpy as np

from .dfa import make_lexer_dfa


def nfa_from_dfa(table: np.ndarray, reject: int = 0) -> np.ndarray:
    """The deterministic automaton as a relation: one successor per (state, byte), none where
    the table rejects (and none out of the reject state)."""
    S = table.shape[0]
    W = (S + 31) // 32
    nfa = np.zeros((256, S, W), np.uint32)
    q = np.repeat(np.arange(S), 256)
    b = np.tile(np.arange(256), S)
    nxt = table.reshape(-1).astype(np.int64)
    keep = (nxt != reject) & (q != reject)
    np.bitwise_or.at(nfa, (b[keep], q[keep], nxt[keep] >> 5), (np.uint32(1) << (nxt[keep] & 31).astype(np.uint32)))
    return nfa


def add_transitions(nfa: np.ndarray, seed: int, fraction: float) -> np.ndarray:
    """Gives `fraction` of the (byte, state) pairs that have a successor one more, drawn
    uniformly from the states 1 .. S-1 (what a lexer with overlapping rules looks like before
    it is made deterministic)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = nfa.copy()
    S = nfa.shape[1]
    has = nfa.any(axis=2)
    bs, qs = np.nonzero(has)
    pick = rng.random(bs.size) < fraction
    extra = rng.integers(1, max(S, 2), size=int(pick.sum()))
    np.bitwise_or.at(out, (bs[pick], qs[pick], extra >> 5), (np.uint32(1) << (extra & 31).astype(np.uint32)))
    return out


def make_lexer_nfa(seed: int, S: int, fraction: float = 0.10) -> np.ndarray:
    """The lexer automaton of the class-build configurations with `fraction` of its live
    transitions doubled."""
    table, _keywords = make_lexer_dfa(seed, S)
    return add_transitions(nfa_from_dfa(table), seed + 1, fraction)
