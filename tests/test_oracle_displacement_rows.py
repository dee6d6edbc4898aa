"""Pins for the limits the C interface puts on Algorithm 1 (which tokens overflow) and for the
fixed-length row encoding of a displacement set.

Within the limits the result must be the set Algorithm 1 returns (oracle displacement(), itself
pinned by Figure 3, by Appendix B's second formulation and by the right-linear special case);
each limit is crossed alone by a grammar built for it; the encoding is pinned by decoding it."""

import itertools

import numpy as np
import pytest

from oracle import displacement as D
from synthetic_inputs.grammar import (grammar_from_productions, make_bracket_gnf, make_random_gnf,
                                      make_token_strings)


def _all_tokens(alphabet: bytes, max_len: int):
    return [bytes(w) for n in range(0, max_len + 1) for w in itertools.product(alphabet, repeat=n)]


@pytest.mark.parametrize("seed", range(8))
def test_within_limits_the_result_is_algorithm_1(seed):
    g = make_random_gnf(100 + seed, n_nt=5, alphabet=b"abc", n_prod=16, max_body=3)
    prods = g.productions()
    adj = D.stack_adjacency(prods)
    seen_backtrack = overflowed = 0
    toks = _all_tokens(b"abc", 4)
    for tok in toks:
        want = D.displacement(tuple(tok), prods, adjacency=adj)
        got = D.displacement_within_limits(tuple(tok), prods, adj)
        if got is None:      # a dense random grammar can cross the frontier bound
            overflowed += 1
            continue
        assert got == want, tok
        seen_backtrack += any(len(q) >= 2 for (q, _s) in want)
    assert seen_backtrack > 0, "some token must need a second stack backtrack"
    assert overflowed * 4 < len(toks)


@pytest.mark.parametrize("which", ["json", "clike"])
def test_within_limits_the_result_is_algorithm_1_on_the_measured_grammars(which):
    """The two hand-written grammars against the measured vocabulary: the first 3,000 tokens and
    every token of 13 bytes or more among the first 30,000 (long digit runs reach deep queues)."""
    import synthetic_inputs as si
    from synthetic_inputs.grammar import make_clike_gnf, make_json_gnf
    g = make_json_gnf() if which == "json" else make_clike_gnf()
    prods = g.productions()
    adj, index = D.stack_adjacency(prods), D.index_productions(prods)
    vocab = si.make_config(3)["vocab"]
    lens = np.diff(vocab.tok_off)
    picked = list(range(3000)) + [t for t in range(3000, 30000) if lens[t] >= 13]
    deep = alive = 0
    for t in picked:
        tok = tuple(vocab.token(t))
        got = D.displacement_within_limits(tok, prods, adj, index)
        if got is None:
            continue
        assert got == D.displacement(tok, prods, adj, index), (t, bytes(tok))
        alive += len(got) > 0
        deep += any(len(q) > 12 for (q, _s) in got)
    assert alive > 500
    if which == "json":
        assert deep > 5, "digit runs must reach queues beyond a dozen symbols"


def test_figure_3_is_within_limits():
    from golden_fixtures import read_fig3
    token, prods, _steps, res_i, res_o = read_fig3()
    names = sorted({p[0] for p in prods} | {b for p in prods for b in p[2]})
    num = {n: i for i, n in enumerate(names)}
    iprods = [(num[A], ord(a), tuple(num[b] for b in beta)) for (A, a, beta) in prods]
    adj = D.stack_adjacency(iprods)
    got = D.displacement_within_limits(tuple(token.encode()), iprods, adj)
    assert got == frozenset({(tuple(num[x] for x in res_i), tuple(num[x] for x in res_o))})


def test_empty_token_and_dead_token():
    g = make_random_gnf(3, n_nt=3, alphabet=b"ab", n_prod=6)
    prods = g.productions()
    adj = D.stack_adjacency(prods)
    assert D.displacement_within_limits((), prods, adj) == frozenset({((), ())})
    assert D.displacement_within_limits((ord("z"),), prods, adj) == frozenset()
    row, h, st = D.encode_displacement(frozenset(), 5, seed=1)
    assert st == D.DISP_OK and row == [0] * D.DISP_ROW_LEN and h == 0
    assert D.encode_displacement(frozenset({((), ())}), 5, seed=1)[0][:4] == [1, 0, 0, 0]


@pytest.mark.parametrize("caps", [(D.LIMIT_QUEUE, D.LIMIT_STACK, D.LIMIT_SUCCESSORS), (5, 7, 9)])
def test_the_input_queue_cap(caps):
    # X -> x A A makes (A, A) stack-adjacent; A -> a.  "a" * k keeps backtracking into A.
    max_in = caps[0]
    prods = [(0, ord("x"), (1, 1)), (1, ord("a"), ())]
    adj = D.stack_adjacency(prods)
    assert (1, 1) in adj
    ok = D.displacement_within_limits((ord("a"),) * max_in, prods, adj, limits=caps)
    assert ok == frozenset({((1,) * max_in, ())})
    assert D.displacement_within_limits((ord("a"),) * (max_in + 1), prods, adj, limits=caps) is None
    # the unbounded algorithm goes on
    assert D.displacement((ord("a"),) * (max_in + 1), prods) == frozenset({((1,) * (max_in + 1), ())})


@pytest.mark.parametrize("caps", [(D.LIMIT_QUEUE, D.LIMIT_STACK, D.LIMIT_SUCCESSORS), (5, 7, 9)])
def test_the_output_stack_cap(caps):
    max_out = caps[1]
    prods = [(0, ord("a"), (0, 0, 0, 0))]   # each byte: pop one, push four
    adj = D.stack_adjacency(prods)
    seen_none = False
    for k in range(1, 13):
        got = D.displacement_within_limits((ord("a"),) * k, prods, adj, limits=caps)
        depth = 4 + 3 * (k - 1)
        if depth <= max_out:
            assert got == frozenset({((0,), (0,) * depth)})
        else:
            assert got is None
            seen_none = True
    assert seen_none


@pytest.mark.parametrize("caps", [(D.LIMIT_QUEUE, D.LIMIT_STACK, D.LIMIT_SUCCESSORS), (5, 7, 9)])
def test_the_frontier_cap_counts_successors_with_multiplicity(caps):
    n = caps[2]
    prods = [(i, ord("a"), ()) for i in range(n)]
    adj = D.stack_adjacency(prods)
    got = D.displacement_within_limits((ord("a"),), prods, adj, limits=caps)
    assert got is not None and len(got) == n
    prods.append((n, ord("a"), ()))
    assert D.displacement_within_limits((ord("a"),), prods, D.stack_adjacency(prods), limits=caps) is None
    # one configuration with n + 1 successors
    prods = [(0, ord("s"), (1,))] + [(1, ord("b"), (2 + i,)) for i in range(n + 1)]
    assert D.displacement_within_limits((ord("s"), ord("b")), prods, set(), limits=caps) is None
    assert len(D.displacement((ord("s"), ord("b")), prods)) == n + 1
    # n + 1 successors that fall together into one configuration still count n + 1
    prods = [(i, ord("a"), (n + 1,)) for i in range(n + 1)] + [(n + 1, ord("b"), ())]
    got = D.displacement_within_limits((ord("a"),), prods, set(), limits=caps)
    assert got is None and len(D.displacement((ord("a"),), prods)) == n + 1


def test_rows_of_tokens_around_the_queue_limit():
    prods = [(0, ord("x"), (1, 1)), (1, ord("a"), ())]
    n = D.LIMIT_QUEUE
    toks = [b"a" * (n - 1), b"a" * n, b"a" * (n + 1)]
    rows, hashes, status = D.displacement_rows(toks, prods, seed=4)
    assert status.tolist() == [0, 0, 1]
    assert D.decode_displacement(rows[1]) == frozenset({((1,) * n, ())})
    # the definition itself goes on where the library gives up
    assert D.displacement(tuple(toks[2]), prods) == frozenset({((1,) * (n + 1), ())})


def test_overflow_of_the_row():
    # 100 pairs of 2 + 1 + 1 entries: 401 > 256 entries, though the frontier bound holds
    prods = [(i, ord("a"), (0,)) for i in range(100)]
    pairs = D.displacement_within_limits((ord("a"),), prods, set())
    assert pairs is not None and len(pairs) == 100
    row, h, st = D.encode_displacement(pairs, 70000, seed=9)
    assert st == D.DISP_OVERFLOW
    assert row[:4] == [0xFFFF, 70000 & 0xFFFF, 70000 >> 16, 0] and len(row) == D.DISP_ROW_LEN
    row2, h2, _ = D.encode_displacement(None, 70001, seed=9)
    assert row2 != row and h2 != h
    # the largest set that still fits: 63 pairs of 4 entries + the count = 253
    row, _h, st = D.encode_displacement(frozenset(list(pairs)[:63]), 0, seed=9)
    assert st == D.DISP_OK and row[0] == 63
    _row, _h, st = D.encode_displacement(frozenset(list(pairs)[:64]), 0, seed=9)
    assert st == D.DISP_OVERFLOW   # 1 + 64 * 4 = 257
    # a longer row takes it, and starts like the short one would
    row512, h512, st = D.encode_displacement(pairs, 70000, seed=9, row_len=512)
    assert st == D.DISP_OK and len(row512) == 512 and row512[0] == 100 and D.decode_displacement(row512) == pairs
    short = D.encode_displacement(frozenset(list(pairs)[:63]), 0, seed=9)
    long_ = D.encode_displacement(frozenset(list(pairs)[:63]), 0, seed=9, row_len=1024)
    assert long_[0][:256] == short[0] and long_[1] == short[1] and not any(long_[0][256:])


def test_canonical_order():
    pairs = [((2,), (1, 1)), ((1, 5), ()), ((1,), (9,)), ((1,), (3, 0)), ((), ()), ((0, 0), ())]
    row, _h, st = D.encode_displacement(pairs, 0, seed=1)
    assert st == D.DISP_OK
    # by (ni, no), then queue, then stack
    want = [0, 0, 1, 1, 1, 9, 1, 2, 1, 3, 0, 1, 2, 2, 1, 1, 2, 0, 0, 0, 2, 0, 1, 5]
    assert row[0] == 6 and row[1:1 + len(want)] == want


@pytest.mark.parametrize("seed", range(4))
def test_encoding_round_trip_and_order_freedom(seed):
    g = make_random_gnf(40 + seed, n_nt=5, alphabet=b"abc", n_prod=12, max_body=3)
    prods = g.productions()
    adj = D.stack_adjacency(prods)
    rng = np.random.default_rng(seed)
    rows = {}
    checked = 0
    for t, tok in enumerate(_all_tokens(b"abc", 4)):
        pairs = D.displacement_within_limits(tuple(tok), prods, adj)
        row, h, st = D.encode_displacement(pairs, t, seed=77)
        if st != D.DISP_OK:     # a large set of an ambiguous grammar
            assert pairs is None or 1 + sum(2 + len(q) + len(o) for q, o in pairs) > D.DISP_ROW_LEN
            continue
        checked += 1
        assert D.decode_displacement(row) == pairs
        assert all(0 <= x < 65536 for x in row)
        # a set has no order: any order of the same pairs encodes alike
        shuffled = list(pairs)
        rng.shuffle(shuffled)
        assert D.encode_displacement(shuffled, t, seed=77)[:2] == (row, h)
        # equal rows <=> equal sets, and then equal hashes
        key = tuple(row)
        if key in rows:
            assert rows[key] == (pairs, h)
        rows[key] = (pairs, h)
    assert checked >= 100
    by_set = {}
    for key, (pairs, h) in rows.items():
        assert pairs not in by_set
        by_set[pairs] = key
    hashes = [h for (_p, h) in rows.values()]
    assert len(set(hashes)) == len(hashes), "distinct small sets should not collide"


def test_hash_depends_on_seed_and_on_every_record_entry():
    base = ((1, 2, 3), (4, 5))
    h0 = D.encode_displacement([base], 0, seed=1)[1]
    assert D.encode_displacement([base], 0, seed=2)[1] != h0
    for variant in [((1, 2), (3, 4, 5)), ((1, 2, 3, 0), (4, 5)), ((1, 2, 3), (4, 5, 0)),
                    ((3, 2, 1), (4, 5)), ((1, 2, 3), (5, 4))]:
        assert D.encode_displacement([variant], 0, seed=1)[1] != h0
    two = D.encode_displacement([base, ((), ())], 0, seed=1)[1]
    assert two == (h0 + D.encode_displacement([((), ())], 0, seed=1)[1]) % (1 << 64)


def test_rows_of_a_vocabulary_and_bracket_grammar_classes():
    g, atoms = make_bracket_gnf(5)
    prods = g.productions()
    v = make_token_strings(6, 300, atoms + b"()[]{},+-*", 4)
    toks = v.tokens()
    rows, hashes, status = D.displacement_rows(toks, prods, seed=3)
    assert rows.shape == (300, D.DISP_ROW_LEN) and rows.dtype == np.uint16
    assert (status == D.DISP_OK).all()
    adj = D.stack_adjacency(prods)
    for t in range(0, 300, 7):
        assert D.decode_displacement(rows[t]) == D.displacement(tuple(toks[t]), prods, adjacency=adj)
    # two atoms are interchangeable everywhere, an atom and an operator are not
    a0, a1 = bytes([atoms[0]]), bytes([atoms[1]])
    r = D.displacement_rows([a0, a1, b"+", a0 + b"+" + a1, a1 + b"+" + a0, b"(" + a0, b"[" + a0],
                            prods, seed=3)[0]
    assert (r[0] == r[1]).all() and not (r[0] == r[2]).all()
    assert (r[3] == r[4]).all() and not (r[5] == r[6]).all()


def test_adjacency_bit_matrix_layout():
    adj = {(3, 1), (40, 1), (0, 2)}
    bits = D.adjacency_bits(adj, 41)
    assert bits.shape == (41, 2)
    assert bits[1, 0] == 1 << 3 and bits[1, 1] == 1 << 8 and bits[2, 0] == 1
    assert int(bits.sum()) == (1 << 3) + (1 << 8) + 1


def test_json_and_clike_grammars_accept_what_they_should():
    """The hand-written grammars are in normal form, sorted, and their one-state pushdown automaton
    (Equation 2) accepts well-formed texts and rejects broken ones."""
    from synthetic_inputs.grammar import make_clike_gnf, make_json_gnf
    cases = {
        make_json_gnf: ([b'{"a": [1,2.5e-3,true,null], "b":{"c":"x\\n\\u00e9"}}', b'[]', b'-0.5', b'"s"'],
                        [b'[1,]', b'{"a" 1}', b'tru', b'{"a":}', b'01x']),
        make_clike_gnf: ([b'x = foo(a, b[3]) + 2.5;', b'if (x<1) { return y; }',
                          b'while (i) { i = i - 1; s = "a\\n"; }', b'{ f(); { g(1,2); } }'],
                         [b'x = (1;', b'if x;', b'{ x; ', b'x = );', b'f(;']),
    }
    for make, (good, bad) in cases.items():
        g = make()
        prods = g.productions()
        assert prods == sorted(set(prods), key=lambda p: (p[1], p[0], p[2])) and len(prods) == g.P
        assert all(0 <= A < g.N and all(0 <= b < g.N for b in beta) for A, _a, beta in prods)
        d = D.delta(prods)
        for text in good:
            assert () in D.pi(tuple(text), (0,), d), text
        for text in bad:
            assert () not in D.pi(tuple(text), (0,), d), text
