"""Seeded context-free grammars in Greibach normal form over bytes, as flat arrays.

Every production is  A -> a B_1 .. B_n  with one terminal byte `a` and any number of
non-terminals.  Non-terminals are numbered 0 .. N-1.  Productions are unique and sorted by
(byte, head, body): the order in which the GPU library expects them; bodies are stored one
after the other with an offset array (CSR).

Nothing here parses anything or computes displacements: these are inputs only.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

from .vocab import Vocab, vocab_from_tokens



@dataclass
class Grammar:
    N: int                  # number of non-terminals
    head: np.ndarray        # uint16 [P]
    byte: np.ndarray        # uint8  [P]
    body_off: np.ndarray    # int32  [P + 1]: body of production i = body[body_off[i]:body_off[i+1]]
    body: np.ndarray        # uint16 [body_off[P]]

    @property
    def P(self) -> int:
        return int(self.head.shape[0])

    @property
    def length(self) -> np.ndarray:
        return np.diff(self.body_off)

    def arrays(self):
        """(head, byte, body_off, body): the argument order of the library."""
        return self.head, self.byte, self.body_off, self.body

    def productions(self) -> List[Tuple[int, int, Tuple[int, ...]]]:
        """[(A, a, (B_1, .., B_n))] in the array order."""
        return [(int(self.head[i]), int(self.byte[i]),
                 tuple(int(x) for x in self.body[int(self.body_off[i]):int(self.body_off[i + 1])]))
                for i in range(self.P)]


def grammar_from_productions(N: int, prods: Sequence[Tuple[int, int, Sequence[int]]]) -> Grammar:
    uniq = sorted({(int(a), int(A), tuple(int(x) for x in beta)) for (A, a, beta) in prods})
    P = len(uniq)
    body_off = np.zeros(P + 1, np.int32)
    body: List[int] = []
    head, byte = np.zeros(P, np.uint16), np.zeros(P, np.uint8)
    for i, (a, A, beta) in enumerate(uniq):
        assert 0 <= A < N and 0 <= a < 256 and all(0 <= b < N for b in beta)
        head[i], byte[i] = A, a
        body += beta
        body_off[i + 1] = len(body)
    return Grammar(N=N, head=head, byte=byte, body_off=body_off, body=np.array(body, np.uint16))


def make_random_gnf(seed: int, n_nt: int, alphabet: bytes, n_prod: int, max_body: int = 3,
                    unary_fraction: float = 0.35) -> Grammar:
    """Random productions; every non-terminal gets at least one production without body (so
    every symbol can be popped) and bodies of 1..max_body symbols otherwise."""
    rng = np.random.Generator(np.random.PCG64(seed))
    prods = set()
    for A in range(n_nt):
        prods.add((A, int(alphabet[rng.integers(len(alphabet))]), ()))
    while len(prods) < n_prod:
        A = int(rng.integers(n_nt))
        a = int(alphabet[rng.integers(len(alphabet))])
        k = 0 if rng.random() < unary_fraction else int(rng.integers(1, max_body + 1))
        prods.add((A, a, tuple(int(x) for x in rng.integers(0, n_nt, size=k))))
    return grammar_from_productions(n_nt, list(prods))


def make_bracket_gnf(seed: int, n_atoms: int = 6) -> Tuple[Grammar, bytes]:
    """A small expression language with nesting, already in Greibach normal form:
        E -> atom | atom O | '(' E C | '(' E C O | '[' E D | '[' E D O
        O -> op E            C -> ')'            D -> ']'
    over atoms a.., two bracket kinds and a few operators; plus a list rule
        E -> '{' E L         L -> ',' E L | '}' | '}' O
    Non-terminals: E=0, O=1, C=2, D=3, L=4."""
    rng = np.random.Generator(np.random.PCG64(seed))
    E, O, C, D, L = range(5)
    atoms = bytes(rng.choice(np.frombuffer(b"abcdefghijklmnopqrstuvwxyz0123456789", np.uint8),
                             size=n_atoms, replace=False))
    prods = []
    for a in atoms:
        prods += [(E, a, ()), (E, a, (O,))]
    prods += [(E, ord("("), (E, C)), (E, ord("("), (E, C, O)), (E, ord("["), (E, D)),
              (E, ord("["), (E, D, O)), (E, ord("{"), (E, L))]
    for op in b"+-*":
        prods.append((O, op, (E,)))
    prods += [(C, ord(")"), ()), (D, ord("]"), ()), (L, ord(","), (E, L)), (L, ord("}"), ()),
              (L, ord("}"), (O,))]
    return grammar_from_productions(5, prods), atoms


def make_token_strings(seed: int, V: int, alphabet: bytes, max_len: int) -> Vocab:
    """V byte strings, length uniform on 1..max_len, bytes uniform over `alphabet`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    alpha = np.frombuffer(alphabet, dtype=np.uint8)
    toks = [bytes(alpha[rng.integers(0, len(alpha), size=int(rng.integers(1, max_len + 1)))])
            for _ in range(V)]
    return vocab_from_tokens(toks)


JSON_NONTERMINALS = ["VAL", "STR", "ESC", "HEX", "NUMT", "NUMD", "FRAC", "FRACT", "EXP", "EXPD",
                     "EXPT", "OBJ", "OBJT", "MEMBER", "COLON", "ARR", "ARRT", "SP", "TR", "TU",
                     "TE", "FA", "FL", "FS", "NU", "NL", "NL2"]


def make_json_gnf() -> Grammar:
    """The JSON value language over bytes, written directly in Greibach normal form (every
    production starts with its terminal byte; what must follow waits on the stack).  Strings
    take any byte from 0x20 up except the quote and the backslash, with the usual escapes;
    numbers have optional fraction and exponent; one blank may follow ',' and ':' and '{'.
    Stands in for the JSON grammars of the paper's experiments, which come from a schema
    compiler that is not available here."""
    nt = {name: i for i, name in enumerate(JSON_NONTERMINALS)}
    P: List[Tuple[int, int, Tuple[int, ...]]] = []

    def add(head: str, byte, *body: str):
        b = byte if isinstance(byte, int) else ord(byte)
        P.append((nt[head], b, tuple(nt[x] for x in body)))

    digits = b"0123456789"
    value_starts: List[Tuple[int, Tuple[str, ...]]] = [(ord('"'), ("STR",)), (ord("-"), ("NUMD",)),
                                                       (ord("{"), ("OBJ",)), (ord("["), ("ARR",)),
                                                       (ord("t"), ("TR",)), (ord("f"), ("FA",)),
                                                       (ord("n"), ("NU",))]
    for d in digits:
        value_starts += [(d, ()), (d, ("NUMT",))]
    for b, body in value_starts:
        add("VAL", b, *body)
        add("ARR", b, *body, "ARRT")
    add("ARR", "]")
    add("ARRT", "]")
    add("ARRT", ",", "VAL", "ARRT")
    add("ARRT", ",", "SP", "VAL", "ARRT")
    add("OBJ", "}")
    add("OBJ", '"', "STR", "COLON", "VAL", "OBJT")
    add("OBJ", " ", "OBJ")
    add("OBJT", "}")
    add("OBJT", ",", "MEMBER", "OBJT")
    add("OBJT", ",", "SP", "MEMBER", "OBJT")
    add("MEMBER", '"', "STR", "COLON", "VAL")
    add("COLON", ":")
    add("COLON", ":", "SP")
    add("SP", " ")
    add("SP", "\n")
    # strings
    add("STR", '"')
    add("STR", "\\", "ESC", "STR")
    for c in range(0x20, 0x100):
        if c not in (ord('"'), ord("\\")):
            add("STR", c, "STR")
    for c in '"\\/bfnrt':
        add("ESC", c)
    add("ESC", "u", "HEX", "HEX", "HEX", "HEX")
    for c in b"0123456789abcdefABCDEF":
        add("HEX", c)
    # numbers
    for d in digits:
        add("NUMT", d), add("NUMT", d, "NUMT")
        add("NUMD", d), add("NUMD", d, "NUMT")
        add("FRAC", d), add("FRAC", d, "FRACT")
        add("FRACT", d), add("FRACT", d, "FRACT")
        add("EXP", d), add("EXP", d, "EXPT")
        add("EXPD", d), add("EXPD", d, "EXPT")
        add("EXPT", d), add("EXPT", d, "EXPT")
    add("NUMT", ".", "FRAC")
    for e in "eE":
        add("NUMT", e, "EXP")
        add("FRACT", e, "EXP")
    add("EXP", "+", "EXPD")
    add("EXP", "-", "EXPD")
    # literals true / false / null
    add("TR", "r", "TU"), add("TU", "u", "TE"), add("TE", "e")
    add("FA", "a", "FL"), add("FL", "l", "FS"), add("FS", "s", "TE")
    add("NU", "u", "NL"), add("NL", "l", "NL2"), add("NL2", "l")
    return grammar_from_productions(len(JSON_NONTERMINALS), P)


CLIKE_NONTERMINALS = ["PROG", "EXPR", "IDT", "NUMT", "FRAC", "ETL", "ARGS", "ARGT", "RP", "RB", "RBR", "STR",
                      "ESC", "K_F", "IFR", "K_H", "K_HI", "K_HIL", "K_HILE", "K_E", "K_ET", "K_ETU", "K_ETUR",
                      "K_ETURN", "RETR"]


def make_clike_gnf() -> Grammar:
    """A C-flavoured statement and expression language over bytes, written directly in Greibach
    normal form: identifiers, numbers, string literals, prefix and binary operators, calls,
    indexing, parentheses, ';'-separated statements, nested blocks, `if (..)`, `while (..)` and
    `return`.  Single blanks may precede operands and tails (so tokens with a leading blank stay
    alive).  It accepts a superset of what a C parser would (two-character operators are read as
    a binary operator followed by a prefix one); what matters here is its shape: nesting on the
    stack, keywords that compete with identifiers, a few hundred productions.  Stands in for
    the paper's C++ and Bython grammars, which are not available."""
    nt = {name: i for i, name in enumerate(CLIKE_NONTERMINALS)}
    P: List[Tuple[int, int, Tuple[int, ...]]] = []

    def add(head: str, byte, *body: str):
        b = byte if isinstance(byte, int) else ord(byte)
        P.append((nt[head], b, tuple(nt[x] for x in body)))

    id_start = b"abcdefghijklmnopqrstuvwxyzABCDEFGHIJKLMNOPQRSTUVWXYZ_"
    digits = b"0123456789"
    binary = b"+-*/%<>=&|^.,?:"
    prefix = b"-!~*&"

    # an operand and what may follow it; every list entry is (first byte, body)
    expr: List[Tuple[int, Tuple[str, ...]]] = []
    for c in id_start:
        expr += [(c, ()), (c, ("IDT",))]
    for d in digits:
        expr += [(d, ()), (d, ("NUMT",))]
    for p in prefix:
        expr.append((p, ("EXPR",)))
    expr += [(ord("("), ("EXPR", "RP")), (ord("("), ("EXPR", "RP", "ETL")),
             (ord('"'), ("STR",)), (ord('"'), ("STR", "ETL")), (ord(" "), ("EXPR",))]
    for b, body in expr:
        add("EXPR", b, *body)
        add("ARGS", b, *body, "ARGT")          # first argument of a call
        add("PROG", b, *body)                  # an expression statement (its tail takes the ';')
    add("ARGS", ")"), add("ARGS", ")", "ETL")
    add("ARGT", ")"), add("ARGT", ")", "ETL")
    add("ARGT", ",", "EXPR", "ARGT")
    add("RP", ")"), add("RB", "]"), add("RBR", "}")
    add("RP", " ", "RP"), add("RB", " ", "RB"), add("RBR", " ", "RBR"), add("RBR", "\n", "RBR")

    # tails: after an identifier, after a number, after any complete operand
    def tails(head: str):
        for op in binary:
            add(head, op, "EXPR")
        add(head, "(", "ARGS")
        add(head, "[", "EXPR", "RB"), add(head, "[", "EXPR", "RB", "ETL")
        add(head, ";"), add(head, ";", "PROG")
        add(head, " ", "ETL")

    for c in id_start + digits:
        add("IDT", c), add("IDT", c, "IDT")
    tails("IDT")
    for d in digits:
        add("NUMT", d), add("NUMT", d, "NUMT")
        add("FRAC", d), add("FRAC", d, "FRAC"), add("FRAC", d, "ETL")
    add("NUMT", ".", "FRAC")
    tails("NUMT")
    tails("ETL")

    # string literals
    add("STR", '"')
    add("STR", "\\", "ESC", "STR")
    for c in range(0x20, 0x7F):
        if c not in (ord('"'), ord("\\")):
            add("STR", c, "STR")
    for c in '"\\nt0':
        add("ESC", c)

    # statements that are not expressions
    add("PROG", ";"), add("PROG", ";", "PROG")
    add("PROG", "{", "PROG", "RBR"), add("PROG", "{", "PROG", "RBR", "PROG")
    add("PROG", "{", "RBR"), add("PROG", "{", "RBR", "PROG")
    add("PROG", "\n", "PROG"), add("PROG", " ", "PROG")
    add("PROG", "i", "K_F"), add("K_F", "f", "IFR")
    add("IFR", " ", "IFR"), add("IFR", "(", "EXPR", "RP", "PROG")
    add("PROG", "w", "K_H"), add("K_H", "h", "K_HI"), add("K_HI", "i", "K_HIL"), add("K_HIL", "l", "K_HILE")
    add("K_HILE", "e", "IFR")
    add("PROG", "r", "K_E"), add("K_E", "e", "K_ET"), add("K_ET", "t", "K_ETU"), add("K_ETU", "u", "K_ETUR")
    add("K_ETUR", "r", "K_ETURN"), add("K_ETURN", "n", "RETR")
    add("RETR", ";"), add("RETR", ";", "PROG"), add("RETR", " ", "EXPR")
    return grammar_from_productions(len(CLIKE_NONTERMINALS), P)
