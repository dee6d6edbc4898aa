"""Seeded byte-level lexer automata as dense transition tables.

A table is ``uint16[S][256]``; entry ``table[q][b]`` is the state reached from
state ``q`` on byte ``b``.  State 0 is the reject state and is absorbing
(``table[0][b] == 0`` for every byte).  State 1 is the start state.  These are
generator conventions only; the library under test treats the table as an
arbitrary transformation of {0..S-1} per byte.

Two recipes:

* ``make_json_like_dfa``  - 24 states, JSON-flavoured modes over the 64-symbol
  alphabet, then thinly rewired at random until about 30 % of the transitions
  on alphabet bytes lead to reject.
* ``make_lexer_dfa``      - a C-flavoured token-stream lexer (identifiers,
  numbers, strings, comments, maximal-munch operators, UTF-8 continuation
  states) replicated in ``S // 256`` nested "contexts", each padded to its
  share of the S states with a keyword trie of seeded random words.

Nothing here walks tokens through the automaton.
"""

from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import numpy as np

from .vocab import ALPHABET64

REJECT = 0
START = 1

_LOWER = b"abcdefghijklmnopqrstuvwxyz"
_UPPER = b"ABCDEFGHIJKLMNOPQRSTUVWXYZ"
_DIGITS = b"0123456789"
_HEX = b"0123456789abcdefABCDEF"
_IDENT_CONT = _LOWER + _UPPER + _DIGITS + b"_"
_LEAD2 = bytes(range(0xC2, 0xE0))
_LEAD3 = bytes(range(0xE0, 0xF0))
_LEAD4 = bytes(range(0xF0, 0xF5))
_CONT = bytes(range(0x80, 0xC0))


class _Builder:
    """Accumulates named states with partial rows; unset entries are resolved
    at the end: an accepting (token-complete) state behaves like its context's
    start state on a byte it does not handle, any other state rejects."""

    def __init__(self) -> None:
        self.rows: List[Dict[int, int]] = []
        self.accepting: List[bool] = []
        self.start_of: List[int] = []  # which start state an accepting state falls through to

    def new(self, accepting: bool, start: int = START) -> int:
        self.rows.append({})
        self.accepting.append(accepting)
        self.start_of.append(start)
        return len(self.rows) - 1

    def set(self, q: int, bytes_: bytes, target: int, overwrite: bool = True) -> None:
        row = self.rows[q]
        for b in bytes_:
            if overwrite or b not in row:
                row[b] = target

    def table(self, S: int) -> np.ndarray:
        assert len(self.rows) <= S, (len(self.rows), S)
        t = np.zeros((S, 256), dtype=np.uint16)
        for q, row in enumerate(self.rows):
            for b, tgt in row.items():
                t[q, b] = tgt
        for q, row in enumerate(self.rows):
            if self.accepting[q] and q != self.start_of[q]:
                s = self.start_of[q]
                for b in range(256):
                    if b not in row:
                        t[q, b] = t[s, b]
        t[REJECT, :] = REJECT
        return t


def make_json_like_dfa(seed: int, S: int = 24, reject_fraction: float = 0.30,
                       alphabet: bytes = ALPHABET64) -> np.ndarray:
    """24-state JSON-flavoured automaton (value start, string, escape, number
    int/frac/exp, literal tries for true/false/null, after-value), bytes outside
    `alphabet` reject.  Random rewiring then moves the share of alphabet
    transitions (from non-reject states) that reject to `reject_fraction`."""
    assert S == 24
    rng = np.random.Generator(np.random.PCG64(seed))
    b = _Builder()
    rej = b.new(False)
    value = b.new(False)  # expecting a value (also after '{', '[', ',', ':')
    assert (rej, value) == (REJECT, START)
    string = b.new(False)
    esc = b.new(False)
    after = b.new(False)  # after a complete value
    minus = b.new(False)
    zero = b.new(False)
    integer = b.new(False)
    dot = b.new(False)
    frac = b.new(False)
    e = b.new(False)
    esign = b.new(False)
    exp = b.new(False)
    lit = {}
    for word in (b"true", b"false", b"null"):
        for k in range(1, len(word)):
            lit[word[:k]] = b.new(False)
    ukey = b.new(False)  # one hex digit of a shortened \u escape
    assert len(b.rows) == 24

    ws = b" \n\t"
    b.set(value, ws, value)
    b.set(value, b"{[", value)
    b.set(value, b"}]", after)
    b.set(value, b'"', string)
    b.set(value, b"-", minus)
    b.set(value, b"0", zero)
    b.set(value, b"123456789", integer)
    for word in (b"true", b"false", b"null"):
        prev = value
        for k in range(1, len(word)):
            b.set(prev, word[k - 1:k], lit[word[:k]])
            prev = lit[word[:k]]
        b.set(prev, word[-1:], after)
    for ch in alphabet:
        if ch not in b'"\\\n':
            b.set(string, bytes([ch]), string)
    b.set(string, b'"', after)
    b.set(string, b"\\", esc)
    b.set(esc, b'"\\/bfnrt', string)
    b.set(esc, b"u", ukey)
    b.set(ukey, _HEX, string)
    b.set(after, ws, after)
    b.set(after, b",:", value)
    b.set(after, b"}]", after)
    b.set(minus, b"0", zero)
    b.set(minus, b"123456789", integer)
    b.set(integer, _DIGITS, integer)
    for num in (zero, integer):
        b.set(num, b".", dot)
        b.set(num, b"eE", e)
    b.set(dot, _DIGITS, frac)
    b.set(frac, _DIGITS, frac)
    b.set(frac, b"eE", e)
    b.set(e, b"+-", esign)
    b.set(e, _DIGITS, exp)
    b.set(esign, _DIGITS, exp)
    b.set(exp, _DIGITS, exp)
    for num in (zero, integer, frac, exp):  # a number ends where "after" takes over
        b.set(num, ws, after, overwrite=False)
        b.set(num, b",:", value, overwrite=False)
        b.set(num, b"}]", after, overwrite=False)
    t = b.table(S)

    # bytes outside the alphabet always reject; rewire inside the alphabet
    alpha = np.frombuffer(alphabet, dtype=np.uint8).astype(np.int64)
    sub = t[1:, :][:, alpha]  # view copy [S-1, 64]
    total = sub.size
    want_reject = int(round(reject_fraction * total))
    is_rej = sub == REJECT
    n_rej = int(is_rej.sum())
    if n_rej > want_reject:
        cand = np.argwhere(is_rej)
        pick = rng.choice(len(cand), size=n_rej - want_reject, replace=False)
        for qi, bi in cand[pick]:
            sub[qi, bi] = rng.integers(1, S)
    elif n_rej < want_reject:
        cand = np.argwhere(~is_rej)
        pick = rng.choice(len(cand), size=want_reject - n_rej, replace=False)
        for qi, bi in cand[pick]:
            sub[qi, bi] = REJECT
    t[1:, alpha] = sub
    t[REJECT, :] = REJECT
    return np.ascontiguousarray(t)


def _random_words(rng: np.random.Generator, n: int) -> List[bytes]:
    lower = np.frombuffer(_LOWER, dtype=np.uint8)
    out = []
    for _ in range(n):
        k = int(rng.integers(2, 9))
        out.append(lower[rng.integers(0, 26, size=k)].tobytes())
    return out


def _add_context(b: _Builder, rng: np.random.Generator, budget: int,
                 pool: List[bytes], start: Optional[int],
                 parent_start: Optional[int], opener: bytes,
                 keywords_out: List[bytes]) -> Tuple[int, int]:
    """Append one lexer context using exactly `budget` new states (the first
    context's budget counts the reject and start states too).  Returns
    (start state, state count used)."""
    n0 = len(b.rows)
    if start is None:
        start = b.new(False)
    st = start

    def new(acc: bool) -> int:
        return b.new(acc, start=st)

    ident = new(True)
    idc = [new(False) for _ in range(3)]  # UTF-8 continuation inside identifiers
    integer, zero = new(True), new(True)
    hexp, hexs = new(False), new(True)
    frac = new(True)
    expe, exps, exp = new(False), new(False), new(True)
    intsuf, numsuf = new(True), new(True)
    dot, dot2 = new(True), new(False)
    string, stresc = new(False), new(False)
    strc = [new(False) for _ in range(3)]
    char, chresc = new(False), new(False)
    chrc = [new(False) for _ in range(3)]
    slash = new(True)
    lcom = new(False)
    lcomc = [new(False) for _ in range(3)]
    bcom, bstar = new(False), new(False)
    bcomc = [new(False) for _ in range(3)]
    ws = new(True)
    op = {ch: new(True) for ch in b"+-*%=<>!&|^:"}
    ltlt, gtgt = new(True), new(True)

    def utf8(q: int, conts: List[int], back: int) -> None:
        b.set(q, _LEAD2, conts[0])
        b.set(q, _LEAD3, conts[1])
        b.set(q, _LEAD4, conts[2])
        b.set(conts[0], _CONT, back)
        b.set(conts[1], _CONT, conts[0])
        b.set(conts[2], _CONT, conts[1])

    # start state
    b.set(st, _LOWER + _UPPER + b"_", ident)
    b.set(st, b"123456789", integer)
    b.set(st, b"0", zero)
    b.set(st, b'"', string)
    b.set(st, b"'", char)
    b.set(st, b"/", slash)
    b.set(st, b" \t\n\r", ws)
    b.set(st, b"()[]{};,?~#", st)
    for ch, q in op.items():
        b.set(st, bytes([ch]), q)
    b.set(st, b".", dot)
    utf8(st, idc, ident)
    # identifiers
    b.set(ident, _IDENT_CONT, ident)
    utf8(ident, idc, ident)
    # numbers; a letter that is not a valid suffix makes the number malformed
    letters = _LOWER + _UPPER + b"_"
    b.set(integer, _DIGITS, integer)
    b.set(zero, _DIGITS, integer)
    b.set(zero, b"xX", hexp)
    for q in (integer, zero):
        b.set(q, b".", frac)
        b.set(q, b"eE", expe)
        b.set(q, b"uUlL", intsuf)
        b.set(q, letters, REJECT, overwrite=False)
    b.set(intsuf, b"uUlL", intsuf)
    b.set(intsuf, letters + _DIGITS, REJECT, overwrite=False)
    b.set(hexp, _HEX, hexs)
    b.set(hexs, _HEX, hexs)
    b.set(hexs, b"uUlL", intsuf)
    b.set(hexs, letters, REJECT, overwrite=False)
    b.set(frac, _DIGITS, frac)
    b.set(frac, b"eE", expe)
    b.set(frac, b"fFlL", numsuf)
    b.set(frac, letters, REJECT, overwrite=False)
    b.set(expe, b"+-", exps)
    b.set(expe, _DIGITS, exp)
    b.set(exps, _DIGITS, exp)
    b.set(exp, _DIGITS, exp)
    b.set(exp, b"fFlL", numsuf)
    b.set(exp, letters, REJECT, overwrite=False)
    b.set(numsuf, letters + _DIGITS, REJECT)
    b.set(dot, _DIGITS, frac)
    b.set(dot, b".", dot2)
    b.set(dot2, b".", st)
    # string and character literals
    for q, qesc, conts, quote in ((string, stresc, strc, b'"'), (char, chresc, chrc, b"'")):
        b.set(q, bytes(range(0x80)), q)
        b.set(q, quote, st)
        b.set(q, b"\\", qesc)
        b.set(q, b"\n", REJECT)
        utf8(q, conts, q)
        b.set(qesc, b"nrt0\\'\"abfvx?\n" + _DIGITS, q)
    # comments
    b.set(slash, b"/", lcom)
    b.set(slash, b"*", bcom)
    b.set(slash, b"=", st)
    b.set(lcom, bytes(range(0x80)), lcom)
    b.set(lcom, b"\n", st)
    utf8(lcom, lcomc, lcom)
    b.set(bcom, bytes(range(0x80)), bcom)
    b.set(bcom, b"*", bstar)
    utf8(bcom, bcomc, bcom)
    b.set(bstar, bytes(range(0x80)), bcom)
    b.set(bstar, b"*", bstar)
    b.set(bstar, b"/", st)
    utf8(bstar, bcomc, bcom)
    # whitespace
    b.set(ws, b" \t\n\r", ws)
    # operators with maximal munch
    for ch in b"+-*%=<>!&|^":
        b.set(op[ch], b"=", st)
    b.set(op[ord("+")], b"+", st)
    b.set(op[ord("-")], b"->", st)
    b.set(op[ord("&")], b"&", st)
    b.set(op[ord("|")], b"|", st)
    b.set(op[ord(":")], b":", st)
    b.set(op[ord("<")], b"<", ltlt)
    b.set(op[ord(">")], b">", gtgt)
    b.set(ltlt, b"=", st)
    b.set(gtgt, b"=", st)
    # context nesting: '`' returns to the enclosing context
    if parent_start is not None:
        b.set(st, b"`", parent_start)

    # keyword trie on lower-case letters, rooted at the start state
    used = len(b.rows) - n0
    room = budget - used
    assert room >= 0, (budget, used)
    trie: Dict[bytes, int] = {}
    order = rng.permutation(len(pool))
    for wi in order:
        if room == 0:
            break
        word = pool[int(wi)]
        new_nodes = [word[:k] for k in range(1, len(word) + 1) if word[:k] not in trie]
        if not new_nodes:
            continue
        if len(new_nodes) > room:  # truncate the last word so the budget is met exactly
            word = new_nodes[room - 1]
            new_nodes = new_nodes[:room]
        for pref in new_nodes:
            q = new(True)
            trie[pref] = q
            b.set(q, _IDENT_CONT, ident)
            utf8(q, idc, ident)
        room -= len(new_nodes)
        keywords_out.append(word)
    for pref, q in trie.items():
        parent = st if len(pref) == 1 else trie[pref[:-1]]
        b.set(parent, pref[-1:], q)
    assert room == 0, "keyword pool too small to fill the context"
    return st, len(b.rows) - n0


def make_lexer_dfa(seed: int, S: int) -> Tuple[np.ndarray, List[bytes]]:
    """C-flavoured lexer automaton with exactly S states (S >= 128).

    ``S // 256`` (at least one) nested contexts share the reject state; context
    k+1 is entered from context k's start state on '@' (k even) or '$' (k odd)
    and left again on a back-quote.  Each context holds the same lexer skeleton
    plus a keyword trie over its own random subset of a common word pool.
    Returns (table, keywords); the keyword list feeds the vocabulary recipe."""
    assert S >= 128
    rng = np.random.Generator(np.random.PCG64(seed))
    n_ctx = max(1, S // 256)
    pool = _random_words(rng, max(64, S))
    b = _Builder()
    rej = b.new(False)
    st0 = b.new(False)
    assert (rej, st0) == (REJECT, START)
    keywords: List[bytes] = []
    base = S // n_ctx
    budgets = [base + (1 if k < S - base * n_ctx else 0) for k in range(n_ctx)]
    starts: List[int] = []
    for k in range(n_ctx):
        if k == 0:
            st, used = _add_context(b, rng, budgets[0] - 2, pool, st0, None, b"", keywords)
        else:
            st, used = _add_context(b, rng, budgets[k], pool, None, starts[k - 1], b"", keywords)
        starts.append(st)
    for k in range(n_ctx - 1):
        b.set(starts[k], b"@" if k % 2 == 0 else b"$", starts[k + 1])
    assert len(b.rows) == S, (len(b.rows), S)
    t = b.table(S)
    # de-duplicate keyword list, keep order
    seen = set()
    kws = [w for w in keywords if not (w in seen or seen.add(w))]
    return np.ascontiguousarray(t), kws
