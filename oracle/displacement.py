"""General displacement computation for tiny Greibach-normal-form grammars.
TEST INFRASTRUCTURE ONLY (pure Python, exponential; tokens of a few bytes).

Follows the paper's Section 3.2 (displacement equivalence), Algorithm 1
(computation of the displacement of a token, with stack backtrack restricted by
the stack-adjacency relation) and Appendix C (how that relation is computed).
Also holds the stack-transition function pi of Appendix B, Equation 2, and its
tagged variant pi' of Equation 3, used to pin the algorithm from a second,
independent formulation.

Grammar encoding: a list of productions ``(A, a, beta)`` meaning  A -> a beta,
with ``A`` a hashable non-terminal, ``a`` one terminal (an int byte or a 1-char
string) and ``beta`` a tuple of non-terminals.

Readings taken where the paper leaves room:
  * the very first backtrack (A_prev = empty) is unrestricted: any production
    whose terminal matches may start a displacement (the prose of Section 3.2.2
    says "first non-deterministically select a production");
  * the breadth-first search of Appendix C includes its own start node B_n
    (a path of length zero), otherwise a unary B_n would never be found;
  * the adjacency test of Algorithm 1 is on A_prev, the symbol popped or
    enqueued last, not on the previous element of the input queue.
"""

from __future__ import annotations

from collections import defaultdict, deque
from typing import Dict, FrozenSet, Hashable, Iterable, List, Sequence, Set, Tuple

NT = Hashable
Production = Tuple[NT, object, Tuple[NT, ...]]
Stack = Tuple[NT, ...]


def delta(productions: Sequence[Production]) -> Dict[Tuple[object, NT], List[Stack]]:
    """PDA transition function of Section 2.1: beta in delta(a, A) iff A -> a beta."""
    d: Dict[Tuple[object, NT], List[Stack]] = defaultdict(list)
    for A, a, beta in productions:
        if tuple(beta) not in d[(a, A)]:
            d[(a, A)].append(tuple(beta))
    return d


def stack_adjacency(productions: Sequence[Production]) -> Set[Tuple[NT, NT]]:
    """Appendix C.  Graph H has an edge A -> B for every production whose
    right-most non-terminal is B.  For every production A -> a B_1..B_n Z beta
    (n >= 1) every Y reachable in H from B_n that has a unary production Y -> y
    is popped immediately before Z in some parse: (Y, Z) is stack-adjacent."""
    edges: Dict[NT, Set[NT]] = defaultdict(set)
    unary: Set[NT] = set()
    for A, _a, beta in productions:
        if len(beta) == 0:
            unary.add(A)
        else:
            edges[A].add(beta[-1])
    adj: Set[Tuple[NT, NT]] = set()
    for _A, _a, beta in productions:
        for n in range(1, len(beta)):
            Bn, Z = beta[n - 1], beta[n]
            seen = {Bn}
            queue = deque([Bn])
            while queue:
                X = queue.popleft()
                if X in unary:
                    adj.add((X, Z))
                for Y in edges.get(X, ()):
                    if Y not in seen:
                        seen.add(Y)
                        queue.append(Y)
    return adj


def successors(config, ch, by_terminal, by_pair, adjacency):
    """One step of the one-state pushdown automaton as Algorithm 1 takes it.  A configuration is
    (input queue, output stack, symbol consumed last); `ch` is the byte read.
      * Output stack not empty: its top A is consumed by a production A -> ch beta, whose body
        takes A's place.
      * Output stack empty (stack backtrack): the token reaches below what it pushed itself, so
        the symbol it meets there is guessed: any A with a production A -> ch beta that may come
        right after the symbol consumed last (stack adjacency, Section 3.2.2) is appended to the
        input queue and beta becomes the output stack.  Before anything was consumed every A may
        be guessed."""
    queue, stack, last = config
    if stack:
        top = stack[0]
        for beta in by_pair.get((ch, top), ()):
            yield (queue, beta + stack[1:], top)
    else:
        for A, beta in by_terminal.get(ch, ()):
            if last is None or adjacency == "all" or (last, A) in adjacency:
                yield (queue + (A,), beta, A)


def displacement(token: Sequence, productions: Sequence[Production],
                 adjacency=None, index=None) -> FrozenSet[Tuple[Stack, Stack]]:
    """Algorithm 1: the displacement of `token`, the set of (input queue, output stack) pairs
    with which the automaton can read it.  Depth first over the bytes, from the configuration
    that has consumed and pushed nothing; a configuration met again at the same position is not
    explored twice.  `adjacency` defaults to stack_adjacency(productions); the string "all"
    leaves the stack backtrack unrestricted; `index` = index_productions(productions) if the
    caller already has it."""
    token = tuple(token)
    if adjacency is None:
        adjacency = stack_adjacency(productions)
    by_terminal, by_pair = index if index is not None else index_productions(productions)
    done: Dict[tuple, FrozenSet[Tuple[Stack, Stack]]] = {}

    def finish(pos: int, config) -> FrozenSet[Tuple[Stack, Stack]]:
        """Pairs reachable at the end of the token from `config` with token[:pos] read."""
        if pos == len(token):
            return frozenset({(config[0], config[1])})
        key = (pos, config)
        if key not in done:
            found: Set[Tuple[Stack, Stack]] = set()
            for nxt in successors(config, token[pos], by_terminal, by_pair, adjacency):
                found |= finish(pos + 1, nxt)
            done[key] = frozenset(found)
        return done[key]

    import sys
    if len(token) + 50 > sys.getrecursionlimit():
        sys.setrecursionlimit(len(token) + 200)
    return finish(0, ((), (), None))


def pi(token: Sequence, alpha: Stack, d) -> Set[Stack]:
    """Appendix B, Equation 2: stacks reachable from stack alpha by consuming token."""
    token = tuple(token)
    if len(token) == 0:
        return {tuple(alpha)}
    if len(alpha) == 0:
        return set()
    out: Set[Stack] = set()
    for beta in d.get((token[0], alpha[0]), ()):
        out |= pi(token[1:], tuple(beta) + tuple(alpha[1:]), d)
    return out


def restricted_pre_displacement(token: Sequence, productions: Sequence[Production],
                                nonterminals: Iterable[NT]) -> FrozenSet[Tuple[Stack, Stack]]:
    """Appendix B, D'_G(t) via Equation 3: pairs (alpha, beta) such that alpha is
    consumed entirely while parsing t and beta consists of pushed symbols only.
    Brute force over every alpha of length <= len(t); symbols carry a 0/1 tag
    (0 = was on the initial stack, 1 = pushed)."""
    from itertools import product as cartesian
    token = tuple(token)
    d = delta(productions)
    nts = list(nonterminals)

    def pi_tagged(pos: int, alpha) -> Set[tuple]:
        if pos == len(token):
            return {alpha}
        if len(alpha) == 0:
            return set()
        out = set()
        (A, _tag) = alpha[0]
        for beta in d.get((token[pos], A), ()):
            out |= pi_tagged(pos + 1, tuple((B, 1) for B in beta) + alpha[1:])
        return out

    result = set()
    for n in range(0, len(token) + 1):
        for alpha in cartesian(nts, repeat=n):
            for beta in pi_tagged(0, tuple((A, 0) for A in alpha)):
                if all(tag == 1 for (_B, tag) in beta):
                    result.add((tuple(alpha), tuple(B for (B, _t) in beta)))
    return frozenset(result)


def right_linear_grammar(table, accepting: Iterable[int], reject: int = 0) -> List[Production]:
    """A deterministic byte automaton as a right-linear (hence Greibach) grammar:
    q -> a q' for every transition delta(q, a) = q' != reject, plus q -> a when
    q' is accepting.  Non-terminals are the non-reject states."""
    acc = set(accepting)
    prods: List[Production] = []
    S = len(table)
    for q in range(S):
        if q == reject:
            continue
        for a in range(len(table[q])):
            q2 = int(table[q][a])
            if q2 == reject:
                continue
            prods.append((q, a, (q2,)))
            if q2 in acc:
                prods.append((q, a, ()))
    return prods


# ---------------------------------------------------------------------------------------------
# What a library with fixed-size buffers may give up on, and the fixed-length encoding of a set.
#
# Algorithm 1 has no bounds.  The C interface states limits (include/cfgzip.h, "Bounds"), over the
# quantities of Algorithm 1 itself: with C_p the set of configurations reached after p bytes,
#   * no successor of a configuration of C_p may hold more than LIMIT_QUEUE input-queue symbols or
#     more than LIMIT_STACK output-stack symbols;
#   * the successors of C_p, one per configuration and applicable production (counted before equal
#     ones fall together), may number at most LIMIT_SUCCESSORS;
#   * the encoded set must fit the caller's row.
# A token that breaks one of them OVERFLOWS: it gets a row and a hash no other token has (a class
# of its own: less compression, never a wrong answer).  Otherwise the row holds exactly the set
# displacement() returns; tests/test_oracle_displacement_rows.py pins that.
# ---------------------------------------------------------------------------------------------

LIMIT_QUEUE = 32
LIMIT_STACK = 32
LIMIT_SUCCESSORS = 256
DISP_ROW_LEN = 256            # default row length; any multiple of 256 up to 4096
DISP_OK = 0
DISP_OVERFLOW = 1
_M64 = (1 << 64) - 1


def index_productions(productions: Sequence[Production]):
    """The distinct productions, by terminal and by (terminal, head)."""
    by_terminal: Dict[object, List[Tuple[NT, Stack]]] = defaultdict(list)
    by_pair: Dict[Tuple[object, NT], List[Stack]] = defaultdict(list)
    for A, a, beta in sorted(set((A, a, tuple(beta)) for (A, a, beta) in productions)):
        by_terminal[a].append((A, beta))
        by_pair[(a, A)].append(beta)
    return by_terminal, by_pair


def displacement_within_limits(token: Sequence[int], productions: Sequence[Production], adjacency,
                               index=None, limits=(LIMIT_QUEUE, LIMIT_STACK, LIMIT_SUCCESSORS)):
    """The displacement of `token` if every prefix keeps within `limits` (queue, stack,
    successors per byte), else None.  Walks the sets C_0, C_1, .. of configurations reached after
    each byte, so that it stops where a limit breaks instead of exploring a blow-up."""
    max_queue, max_stack, max_successors = limits
    by_terminal, by_pair = index if index is not None else index_productions(productions)
    reached = {((), (), None)}
    for ch in token:
        following = [nxt for config in reached
                     for nxt in successors(config, ch, by_terminal, by_pair, adjacency)]
        if len(following) > max_successors:
            return None
        if any(len(q) > max_queue or len(s) > max_stack for (q, s, _last) in following):
            return None
        reached = set(following)
    return frozenset((q, s) for (q, s, _last) in reached)


def displacement_record(pair) -> List[int]:
    """ni, no, the queue, the stack (top first)."""
    q, s = pair
    return [len(q), len(s)] + list(q) + list(s)


def _record_key(rec: Sequence[int]):
    """Canonical order: by (ni, no), then the queue, then the stack, entry by entry."""
    return (rec[0], rec[1], tuple(rec[2:]))


def _mix_record(rec: Sequence[int], seed: int) -> int:
    """FNV-1a style pass over the 16-bit entries, then the SplitMix64 finaliser."""
    h = (seed ^ 0x9E3779B97F4A7C15) & _M64
    for x in rec:
        h = ((h ^ x) * 0x100000001B3) & _M64
    h ^= h >> 30
    h = (h * 0xBF58476D1CE4E5B9) & _M64
    h ^= h >> 27
    h = (h * 0x94D049BB133111EB) & _M64
    h ^= h >> 31
    return h


def encode_displacement(pairs, token_id: int, seed: int, row_len: int = DISP_ROW_LEN):
    """(row of row_len 16-bit values, 64-bit hash, status) of one token.
    Row: [number of pairs, then the records (ni, no, queue, stack) in canonical order], zero
    filled.  Hash: the sum over pairs of _mix_record(record).  Overflow (pairs is None, or the
    row is too short): row [0xFFFF, id low 16, id high 16, 0 ..], hash the mix of those three."""
    if pairs is not None:
        recs = sorted((displacement_record(p) for p in pairs), key=_record_key)
        flat = [len(recs)]
        for r in recs:
            flat += r
        if len(flat) <= row_len:
            row = flat + [0] * (row_len - len(flat))
            h = sum(_mix_record(r, seed) for r in recs) & _M64
            return row, h, DISP_OK
    head = [0xFFFF, token_id & 0xFFFF, (token_id >> 16) & 0xFFFF]
    return head + [0] * (row_len - 3), _mix_record(head, seed), DISP_OVERFLOW


def decode_displacement(row: Sequence[int]):
    """Inverse of encode_displacement for a row with status DISP_OK."""
    n, pos, out = int(row[0]), 1, set()
    for _ in range(n):
        ni, no = int(row[pos]), int(row[pos + 1])
        q = tuple(int(x) for x in row[pos + 2:pos + 2 + ni])
        s = tuple(int(x) for x in row[pos + 2 + ni:pos + 2 + ni + no])
        out.add((q, s))
        pos += 2 + ni + no
    return frozenset(out)


def displacement_rows(tokens: Sequence[bytes], productions: Sequence[Production], seed: int,
                      adjacency=None, row_len: int = DISP_ROW_LEN):
    """Rows, hashes and status of a whole vocabulary:
    (uint16 [V][row_len], uint64 [V], int32 [V])."""
    import numpy as np
    if adjacency is None:
        adjacency = stack_adjacency(productions)
    V = len(tokens)
    rows = np.zeros((V, row_len), np.uint16)
    hashes = np.zeros(V, np.uint64)
    status = np.zeros(V, np.int32)
    index = index_productions(productions)
    for t, tok in enumerate(tokens):
        pairs = displacement_within_limits(tuple(tok), productions, adjacency, index)
        if pairs is not None:   # within the limits: the set is Algorithm 1's, by the definition
            pairs = displacement(tuple(tok), productions, adjacency, index)
        rows[t], hashes[t], status[t] = encode_displacement(pairs, t, seed, row_len)
    return rows, hashes, status


def adjacency_bits(adjacency, N: int):
    """The relation as a bit matrix: bit (Y & 31) of word [Z][Y >> 5] is set iff (Y, Z) is
    stack-adjacent (rows indexed by the symbol consumed next)."""
    import numpy as np
    W = (N + 31) // 32
    bits = np.zeros((N, W), np.uint32)
    for (Y, Z) in adjacency:
        bits[Z, Y >> 5] |= np.uint32(1 << (Y & 31))
    return bits
