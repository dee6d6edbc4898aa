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


def displacement(token: Sequence, productions: Sequence[Production],
                 adjacency=None) -> FrozenSet[Tuple[Stack, Stack]]:
    """Algorithm 1: the set of (input queue, output stack) pairs of `token`.
    `adjacency` defaults to stack_adjacency(productions); pass the string
    "all" to leave the backtrack unrestricted."""
    token = tuple(token)
    d = delta(productions)
    if adjacency is None:
        adjacency = stack_adjacency(productions)
    by_terminal: Dict[object, List[Tuple[NT, Stack]]] = defaultdict(list)
    for A, a, beta in productions:
        if (A, tuple(beta)) not in by_terminal[a]:
            by_terminal[a].append((A, tuple(beta)))
    EMPTY = object()  # A_prev before anything was consumed

    def cd(pos: int, sigma_i: Stack, sigma_o: Stack, a_prev) -> Set[Tuple[Stack, Stack]]:
        if pos == len(token):
            return {(sigma_i, sigma_o)}
        out: Set[Tuple[Stack, Stack]] = set()
        ch = token[pos]
        if len(sigma_o) == 0:  # stack backtrack: consume one more symbol of the input stack
            for A, beta in by_terminal.get(ch, ()):
                if a_prev is EMPTY or adjacency == "all" or (a_prev, A) in adjacency:
                    out |= cd(pos + 1, sigma_i + (A,), beta, A)
        else:
            top = sigma_o[0]
            for beta in d.get((ch, top), ()):
                out |= cd(pos + 1, sigma_i, beta + sigma_o[1:], top)
        return out

    return frozenset(cd(0, (), (), EMPTY))


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
