"""Seeded token vocabularies in CSR form (token bytes + offsets).

Two recipes:

* ``make_vocab_uniform``  - lengths uniform on 1..max_len, bytes uniform over a
  fixed 64-symbol alphabet (the tiny configuration).
* ``make_vocab_mixture``  - lengths ``min(Geom(0.2), cap)`` (support 1, 2, ...),
  each token one of four (or five) kinds: leading-space identifier, digit run,
  whitespace run, operator/punctuation sequence and, optionally, a run of
  well-formed UTF-8 multi-byte characters.

Nothing here looks at an automaton or computes anything about the tokens.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

# 64 symbols: a-z, 0-9, space, JSON punctuation, and a few extras.
ALPHABET64 = (
    b"abcdefghijklmnopqrstuvwxyz"
    b"0123456789"
    b" "
    b"{}[]:,\"-.\\"
    b"+E_/\n\tABCDFTN'=;!"
)
assert len(ALPHABET64) == 64 and len(set(ALPHABET64)) == 64

IDENT_BYTES = b"abcdefghijklmnopqrstuvwxyz_"
DIGIT_BYTES = b"0123456789"
SPACE_BYTES = b" \t\n"
SPACE_WEIGHTS = (0.6, 0.1, 0.3)
PUNCT_BYTES = b"+-*/%=<>!&|^~?:;,.()[]{}#\"'\\"


@dataclass
class Vocab:
    """A vocabulary of V byte strings: token i is tok_bytes[tok_off[i]:tok_off[i+1]]."""

    tok_bytes: np.ndarray  # uint8 [sum of lengths]
    tok_off: np.ndarray  # int64 [V + 1]

    @property
    def V(self) -> int:
        return int(self.tok_off.shape[0] - 1)

    @property
    def lengths(self) -> np.ndarray:
        return np.diff(self.tok_off)

    def token(self, i: int) -> bytes:
        return self.tok_bytes[self.tok_off[i]:self.tok_off[i + 1]].tobytes()

    def tokens(self):
        return [self.token(i) for i in range(self.V)]


def vocab_from_tokens(tokens: Sequence[bytes]) -> Vocab:
    """Pack an explicit list of byte strings (tests build small cases with this)."""
    off = np.zeros(len(tokens) + 1, dtype=np.int64)
    if tokens:
        off[1:] = np.cumsum([len(t) for t in tokens])
    data = np.frombuffer(b"".join(tokens), dtype=np.uint8).copy()
    return Vocab(tok_bytes=data, tok_off=off)


def _pack_rows(rows: np.ndarray, lengths: np.ndarray) -> Vocab:
    """rows: uint8 [V, cap]; keep the first lengths[i] bytes of row i."""
    V, cap = rows.shape
    keep = np.arange(cap)[None, :] < lengths[:, None]
    off = np.zeros(V + 1, dtype=np.int64)
    off[1:] = np.cumsum(lengths)
    return Vocab(tok_bytes=np.ascontiguousarray(rows[keep]), tok_off=off)


def make_vocab_uniform(seed: int, V: int = 4096, max_len: int = 8,
                       alphabet: bytes = ALPHABET64) -> Vocab:
    rng = np.random.Generator(np.random.PCG64(seed))
    lengths = rng.integers(1, max_len + 1, size=V, dtype=np.int64)
    alpha = np.frombuffer(alphabet, dtype=np.uint8)
    rows = alpha[rng.integers(0, len(alpha), size=(V, max_len))]
    return _pack_rows(rows, lengths)


def _utf8_run(rng: np.random.Generator, length: int) -> bytes:
    """Well-formed UTF-8 characters of 2-4 bytes, total exactly `length` bytes
    (length >= 2); the last character is chosen to fit."""
    out = bytearray()
    left = length
    while left > 0:
        if left in (2, 3):
            n = left
        elif left == 4:
            n = int(rng.choice((2, 4)))
        elif left == 5:
            n = int(rng.choice((2, 3)))
        else:
            n = int(rng.integers(2, 5))
        if n == 2:
            cp = int(rng.integers(0x80, 0x800))
        elif n == 3:
            cp = int(rng.integers(0x800, 0x10000))
            if 0xD800 <= cp <= 0xDFFF:  # surrogates are not encodable
                cp = 0x4E00 + (cp - 0xD800)
        else:
            cp = int(rng.integers(0x10000, 0x110000))
        out += chr(cp).encode("utf-8")
        left -= n
    assert len(out) == length
    return bytes(out)


def make_vocab_mixture(seed: int, V: int, cap: int, utf8_fraction: float = 0.0,
                       keywords: Optional[Sequence[bytes]] = None,
                       keyword_fraction: float = 0.15) -> Vocab:
    """Token kinds (before the optional UTF-8 share is carved out, the other
    four are rescaled to 1 - utf8_fraction):

      40 %  leading-space identifier: b' ' + [a-z_]*        (length 1: one letter)
      20 %  digit run                 [0-9]+
      15 %  whitespace run            {space, tab, newline}+ (weights .6/.1/.3)
      25 %  operator / punctuation sequence

    If `keywords` is given, `keyword_fraction` of the identifier tokens take
    their letters from a prefix of a randomly chosen keyword (padded with random
    letters when the keyword is shorter), so that the vocabulary contains word
    pieces the automaton's keyword trie reacts to, as a real tokenizer's does.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    lengths = np.minimum(rng.geometric(0.2, size=V), cap).astype(np.int64)
    base = np.array([0.40, 0.20, 0.15, 0.25]) * (1.0 - utf8_fraction)
    probs = np.concatenate([base, [utf8_fraction]])
    kind = rng.choice(5, size=V, p=probs / probs.sum())

    ident = np.frombuffer(IDENT_BYTES, dtype=np.uint8)
    digit = np.frombuffer(DIGIT_BYTES, dtype=np.uint8)
    space = np.frombuffer(SPACE_BYTES, dtype=np.uint8)
    punct = np.frombuffer(PUNCT_BYTES, dtype=np.uint8)

    rows = np.zeros((V, cap), dtype=np.uint8)
    # identifiers
    m = kind == 0
    n = int(m.sum())
    r = ident[rng.integers(0, len(ident), size=(n, cap))]
    lead = lengths[m] >= 2
    r[lead, 0] = ord(" ")
    if keywords:
        use_kw = rng.random(n) < keyword_fraction
        kw_pick = rng.integers(0, len(keywords), size=n)
        for j in np.nonzero(use_kw)[0]:
            kw = np.frombuffer(keywords[int(kw_pick[j])], dtype=np.uint8)
            start = 1 if lead[j] else 0
            k = min(len(kw), cap - start)
            r[j, start:start + k] = kw[:k]
    rows[m] = r
    # digit runs
    m = kind == 1
    rows[m] = digit[rng.integers(0, len(digit), size=(int(m.sum()), cap))]
    # whitespace runs
    m = kind == 2
    rows[m] = space[rng.choice(len(space), size=(int(m.sum()), cap), p=SPACE_WEIGHTS)]
    # operator / punctuation sequences
    m = kind == 3
    rows[m] = punct[rng.integers(0, len(punct), size=(int(m.sum()), cap))]
    # UTF-8 runs (need at least two bytes)
    m = kind == 4
    idx = np.nonzero(m)[0]
    lengths[idx] = np.maximum(lengths[idx], 2)
    for i in idx:
        b = _utf8_run(rng, int(lengths[i]))
        rows[i, :len(b)] = np.frombuffer(b, dtype=np.uint8)
    return _pack_rows(rows, lengths)
