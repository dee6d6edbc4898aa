"""GPU parity, general case: cfgzip_stack_adjacency (Appendix C) and cfgzip_displacements
(Algorithm 1) against the CPU oracle.  For every token the library's status must be what the
interface's limits say, and with status OK the row, decoded, must be the SET that the oracle's
Algorithm 1 returns.  Row layout and hash are checked separately (canonical order, zero fill,
sum of record mixes).  The classes cfgzip_build_classes forms from the rows are compared with
the oracle's grouping of oracle-side rows and, for right-linear grammars, with the byte-walk
classes."""

import itertools

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from oracle import displacement as D
from synthetic_inputs.grammar import (Grammar, grammar_from_productions, make_bracket_gnf,
                                      make_random_gnf, make_token_strings)
from synthetic_inputs.vocab import vocab_from_tokens

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SEED = 0x5EED


@pytest.fixture(scope="module")
def lib():
    import paper_2605_29986_amd as p
    p.load_library()
    return p


def _grammar_dev(g: Grammar):
    from gpu_util import dev
    return tuple(dev(x) for x in g.arrays())


def _check_adjacency(lib, g: Grammar):
    prods = g.productions()
    want = D.adjacency_bits(D.stack_adjacency(prods), g.N)
    adj, invalid = lib.cfgzip_stack_adjacency(*_grammar_dev(g), g.N)
    assert int(invalid.item()) == 0
    assert (adj.cpu().numpy().view(np.uint32) == want).all()


def _check_rows(lib, g: Grammar, vocab, expect_overflow=None, row_len=256):
    from gpu_util import dev, hash_np
    prods = g.productions()
    toks = vocab.tokens()
    adj, index = D.stack_adjacency(prods), D.index_productions(prods)
    rows, hashes, status = lib.cfgzip_displacements(dev(vocab.tok_bytes), dev(vocab.tok_off),
                                                    *_grammar_dev(g), g.N, row_len=row_len,
                                                    hash_seed=SEED)
    got_status, got_rows, got_hash = status.cpu().numpy(), rows.cpu().numpy(), hash_np(hashes)
    want_rows = np.zeros((vocab.V, row_len), np.uint16)
    want_status = np.zeros(vocab.V, np.int32)
    known = {}   # distinct byte string -> (set by Algorithm 1 or None when a limit breaks, its encoding)
    for t, tok in enumerate(toks):
        if t and t % 25000 == 0:
            print(f"  {t} of {vocab.V} tokens compared", flush=True)
        if tok not in known:
            pairs = D.displacement_within_limits(tuple(tok), prods, adj, index)
            if pairs is not None:   # within the limits the library must find Algorithm 1's set
                assert pairs == D.displacement(tuple(tok), prods, adj, index), (t, tok)
            known[tok] = (pairs, D.encode_displacement(pairs, 0, SEED, row_len))
        pairs, (row, h, st) = known[tok]
        if st == D.DISP_OVERFLOW:   # the row of an overflowing token carries its id
            row, h, st = D.encode_displacement(None, t, SEED, row_len)
        assert got_status[t] == st, (t, tok, got_status[t], st)
        if st == D.DISP_OK:
            # the result proper: the decoded row is the set
            assert D.decode_displacement(got_rows[t]) == pairs, (t, tok)
        # the format: canonical order, zero fill, hash
        assert (got_rows[t] == np.asarray(row, np.uint16)).all(), (t, tok, got_rows[t][:24], row[:24])
        assert got_hash[t] == h, (t, tok)
        want_rows[t], want_status[t] = row, st
    if expect_overflow is not None:
        assert bool((want_status == D.DISP_OVERFLOW).any()) == expect_overflow
    # grouping: the library's classes of its rows against the oracle's classes of the oracle's rows
    c, r, C, _coll = lib.cfgzip_build_classes(dev(vocab.tok_bytes), dev(vocab.tok_off), None, rows,
                                              hashes)
    want_c, want_r = oracle.build_classes(want_rows, vocab.tok_off)
    assert C == len(want_r)
    assert (c.cpu().numpy() == want_c).all() and (r.cpu().numpy() == want_r).all()
    return want_rows, want_status, want_c


def _all_tokens(alphabet: bytes, max_len: int):
    return vocab_from_tokens([bytes(w) for n in range(0, max_len + 1)
                              for w in itertools.product(alphabet, repeat=n)])


def _figure3_grammar():
    from golden_fixtures import read_fig3
    token, prods, _steps, res_i, res_o = read_fig3()
    names = sorted({p[0] for p in prods} | {b for p in prods for b in p[2]})
    num = {n: i for i, n in enumerate(names)}
    g = grammar_from_productions(len(names), [(num[A], ord(a), tuple(num[b] for b in beta))
                                              for (A, a, beta) in prods])
    return g, token.encode(), tuple(num[x] for x in res_i), tuple(num[x] for x in res_o)


def test_figure_3(lib):
    print("case figure 3", flush=True)
    g, token, res_i, res_o = _figure3_grammar()
    _check_adjacency(lib, g)
    vocab = vocab_from_tokens([token[:n] for n in range(len(token) + 1)] + [b"xyz", b"zz", b"abx"])
    rows, status, _c = _check_rows(lib, g, vocab, expect_overflow=False)
    assert D.decode_displacement(rows[len(token)]) == frozenset({(res_i, res_o)})


@pytest.mark.parametrize("seed", range(6))
def test_random_grammars_every_short_token(lib, seed):
    print(f"case random grammar seed={seed}", flush=True)
    g = make_random_gnf(300 + seed, n_nt=5 + seed, alphabet=b"abc", n_prod=12 + 3 * seed, max_body=3)
    _check_adjacency(lib, g)
    _check_rows(lib, g, _all_tokens(b"abc", 5))


@pytest.mark.parametrize("n_nt,n_prod,max_body", [(1, 3, 2), (33, 120, 4), (64, 300, 4), (65, 500, 3),
                                                  (700, 3000, 4), (4096, 9000, 4)])
def test_adjacency_sizes(lib, n_nt, n_prod, max_body):
    print(f"case adjacency N={n_nt} P={n_prod}", flush=True)
    g = make_random_gnf(n_nt * 3 + 1, n_nt=n_nt, alphabet=bytes(range(97, 123)), n_prod=max(n_prod, n_nt + 1),
                        max_body=max_body)
    _check_adjacency(lib, g)


def test_chain_of_right_most_symbols_needs_every_closure_round(lib):
    """A_0 -> a A_1, A_1 -> a A_2, .., A_k -> a (unary only at the end of the chain), and
    S -> s A_0 Z: (A_k, Z) is found only by following all k edges."""
    print("case closure chain", flush=True)
    k = 200
    prods = [(i, ord("a"), (i + 1,)) for i in range(k)] + [(k, ord("a"), ())]
    prods += [(k + 1, ord("s"), (0, k + 2)), (k + 2, ord("z"), ())]
    g = grammar_from_productions(k + 3, prods)
    assert D.stack_adjacency(g.productions()) == {(k, k + 2)}
    _check_adjacency(lib, g)


def test_bracket_grammar_vocabulary(lib):
    print("case bracket grammar", flush=True)
    g, atoms = make_bracket_gnf(5)
    _check_adjacency(lib, g)
    vocab = make_token_strings(6, 5000, atoms + b"()[]{},+-*", 6)
    rows, status, c = _check_rows(lib, g, vocab)
    assert (status == D.DISP_OK).mean() > 0.99
    assert len(set(c.tolist())) < 0.5 * vocab.V, "an expression grammar compresses"


def test_large_grammar(lib):
    """Thousands of productions over all 256 byte values."""
    print("case large grammar", flush=True)
    g = make_random_gnf(77, n_nt=60, alphabet=bytes(range(256)), n_prod=5000, max_body=4)
    assert g.P == 5000
    _check_adjacency(lib, g)
    vocab = make_token_strings(78, 6000, bytes(range(256)), 5)
    rows, status, _c = _check_rows(lib, g, vocab)
    assert ((status == D.DISP_OK) & (rows[:, 0] > 0)).sum() > 500, "enough tokens must stay alive"


def test_more_symbols_than_fit_a_byte(lib):
    """Above 255 symbols the kernel keeps 16-bit entries in its records."""
    print("case 300 and 256 symbols", flush=True)
    for n_nt, n_prod in ((300, 900), (256, 800), (255, 800)):
        g = make_random_gnf(n_nt, n_nt=n_nt, alphabet=bytes(range(64, 128)), n_prod=n_prod, max_body=3)
        vocab = make_token_strings(n_nt + 1, 3000, bytes(range(64, 128)), 4)
        rows, status, _c = _check_rows(lib, g, vocab)
        assert ((status == D.DISP_OK) & (rows[:, 0] > 0)).sum() > 300
        assert rows[:, 2:].max() >= 200, "high symbol numbers must show up in the rows"


def test_long_tokens(lib):
    print("case long tokens", flush=True)
    g, atoms = make_bracket_gnf(5)
    a0 = bytes([atoms[0]])
    toks = [b"((" + a0, (a0 + b"+") * 40 + a0, (a0 + b"+") * 32, b"[" + (a0 + b"*") * 70 + a0 + b"]",
            a0 * 200, (a0 + b"-") * 31 + a0 + b"+" , b""]
    rows, status, _c = _check_rows(lib, g, vocab_from_tokens(toks))
    assert status.tolist() == [0] * len(toks)
    assert rows[1][0] > 0 and rows[3][0] > 0 and rows[4][0] == 0


# The kernel first takes every token in small buffers (queue 12, stack 12, 128 successors) and
# again in larger ones when those do not suffice; which attempt finishes a token must not show in
# any output.  The inputs below sit on both sides of the small sizes and of the interface's limits.
KERNEL_FIRST_ATTEMPT = (12, 12, 128)


def test_each_limit_and_the_sizes_of_the_first_attempt(lib):
    print("case limits", flush=True)
    a = ord("a")
    in1, in2 = KERNEL_FIRST_ATTEMPT[0], D.LIMIT_QUEUE
    g = grammar_from_productions(2, [(0, ord("x"), (1, 1)), (1, a, ())])
    _check_adjacency(lib, g)
    toks = [b"a" * n for n in range(0, in2 + 4)]
    rows, status, _ = _check_rows(lib, g, vocab_from_tokens(toks), expect_overflow=True)
    assert status.tolist() == [0] * (in2 + 1) + [1] * 3
    assert D.decode_displacement(rows[in1 + 1]) == frozenset({((1,) * (in1 + 1), ())})
    assert D.decode_displacement(rows[in2]) == frozenset({((1,) * in2, ())})
    # output stack: each byte pops one symbol and pushes four
    g = grammar_from_productions(1, [(0, a, (0, 0, 0, 0))])
    toks = [b"a" * n for n in range(0, 13)]
    depth = [0] + [4 + 3 * (n - 1) for n in range(1, 13)]
    rows, status, _ = _check_rows(lib, g, vocab_from_tokens(toks), expect_overflow=True)
    assert status.tolist() == [0 if d <= D.LIMIT_STACK else 1 for d in depth]
    assert any(KERNEL_FIRST_ATTEMPT[1] < d <= D.LIMIT_STACK for d in depth)
    # successors per byte, counted one per configuration and production
    for n in (KERNEL_FIRST_ATTEMPT[2], KERNEL_FIRST_ATTEMPT[2] + 1, D.LIMIT_SUCCESSORS,
              D.LIMIT_SUCCESSORS + 1):
        over = n > D.LIMIT_SUCCESSORS
        g = grammar_from_productions(n, [(i, a, ()) for i in range(n)])
        _check_rows(lib, g, vocab_from_tokens([b"a", b"aa", b"b", b""]), row_len=2048, expect_overflow=over)
        g = grammar_from_productions(n + 3, [(0, ord("s"), (1,))] + [(1, ord("b"), (2 + i,)) for i in range(n)])
        _check_rows(lib, g, vocab_from_tokens([b"s", b"sb", b"b"]), row_len=2048, expect_overflow=over)
        # successors that fall together into one configuration still count one each
        g = grammar_from_productions(n + 2, [(i, a, (n + 1,)) for i in range(n)] + [(n + 1, ord("b"), ())])
        _check_rows(lib, g, vocab_from_tokens([b"a", b"ab"]), row_len=2048, expect_overflow=over)


@pytest.mark.parametrize("row_len", [256, 512, 1024, 4096])
def test_row_lengths(lib, row_len):
    print(f"case row_len={row_len}", flush=True)
    a = ord("a")
    # k pairs of 2 + 1 + 1 entries: fits while 1 + 4k <= row_len (and k <= 256 successors)
    for heads in (63, 64, 127, 128, 200, 255, 256):
        g = grammar_from_productions(heads, [(i, a, (0,)) for i in range(heads)])
        rows, status, _ = _check_rows(lib, g, vocab_from_tokens([b"a", b"", b"b"]), row_len=row_len)
        assert (status[0] == 0) == (1 + 4 * heads <= row_len)
    # records that straddle the 256-entry chunks the kernel writes: long queues and stacks
    prods = [(0, ord("x"), (1, 1)), (1, a, ()), (1, ord("b"), (2, 2, 2, 2)), (2, ord("c"), (2, 2, 2, 2)),
             (2, ord("c"), (1, 2, 2)), (2, ord("c"), (2, 1)), (2, ord("d"), ()), (1, ord("c"), (2,))]
    g = grammar_from_productions(3, prods)
    toks = [b"a" * i + b"b" + b"c" * j for i in (0, 3, 7, 20, 31) for j in range(0, 8)]
    rows, status, _ = _check_rows(lib, g, vocab_from_tokens(toks), row_len=row_len)
    ok = status == 0
    used = [1 + sum(2 + len(q) + len(o) for q, o in D.decode_displacement(r)) for r in rows[ok]]
    assert max(used) > min(row_len, 2000) * 0.7, "some row must reach into the last chunk"


def test_long_stacks_and_queues_at_their_bounds(lib):
    print("case bounds reached", flush=True)
    # queue and stack exactly at the sizes of the first attempt and at the limits, and one beyond
    (in1, out1, _f1), (in2, out2) = KERNEL_FIRST_ATTEMPT, (D.LIMIT_QUEUE, D.LIMIT_STACK)
    prods = [(0, ord("x"), (1, 1)), (1, ord("a"), ()), (1, ord("b"), (2, 2, 2, 2)),
             (2, ord("c"), (2, 2, 2)), (2, ord("d"), ())]     # b: stack 4; each c: +2; each d: -1
    g = grammar_from_productions(3, prods)

    def tok(queue, stack):     # a token whose only pair has that queue length and stack depth
        assert queue >= 1 and stack >= 4 and stack % 2 == 0
        return b"a" * (queue - 1) + b"b" + b"c" * ((stack - 4) // 2)

    toks = [tok(in1, 4), tok(in1, out1), tok(in1, out1 + 2), tok(in1 + 1, 4), tok(in2, out2), tok(in2, out2 + 2),
            tok(in2 + 1, 4), b"bccdddd", b"bdddd", b"bddddd"]
    rows, status, _ = _check_rows(lib, g, vocab_from_tokens(toks))
    assert status.tolist() == [0, 0, 0, 0, 0, 1, 1, 0, 0, 0]
    assert D.decode_displacement(rows[1]) == frozenset({((1,) * in1, (2,) * out1)})
    assert D.decode_displacement(rows[4]) == frozenset({((1,) * in2, (2,) * out2)})


def test_right_linear_grammar_gives_the_byte_walk_classes(lib, cfg1):
    """Config 1's automaton as a right-linear grammar: displacement classes == walk classes."""
    print("case right-linear config 1", flush=True)
    from gpu_util import dev, vocab_dev
    table, vocab = cfg1["table"], cfg1["vocab"]
    S = table.shape[0]
    accepting = [q for q in range(1, S) if q % 3 == 1]
    g = grammar_from_productions(S, D.right_linear_grammar(table, accepting))
    _check_adjacency(lib, g)
    _rows, status, c_disp = _check_rows(lib, g, vocab, expect_overflow=False)
    tb, to, tt = vocab_dev(vocab, table)
    sig, h = lib.cfgzip_signatures(tb, to, tt)
    c_walk, _r, _C, _ = lib.cfgzip_build_classes(tb, to, tt, sig, h)
    assert (c_walk.cpu().numpy() == c_disp).all()


def test_unsorted_or_out_of_range_grammar_is_reported(lib):
    print("case bad grammar", flush=True)
    from gpu_util import dev
    g = make_random_gnf(9, n_nt=6, alphabet=b"ab", n_prod=14)
    vocab = _all_tokens(b"ab", 3)
    tb, to = dev(vocab.tok_bytes), dev(vocab.tok_off)

    def run(gr, N):
        rows, hashes, status = lib.cfgzip_displacements(tb, to, *_grammar_dev(gr), N)
        _adj, invalid = lib.cfgzip_stack_adjacency(*_grammar_dev(gr), N)
        return rows.cpu().numpy(), status.cpu().numpy(), int(invalid.item())

    rows, status, invalid = run(g, g.N)
    assert invalid == 0 and (status != 2).all()
    prods = g.productions()
    swapped = list(prods)
    swapped[3], swapped[4] = swapped[4], swapped[3]

    def flat(N, plist):     # the arrays in the order given, not sorted
        off = np.zeros(len(plist) + 1, np.int32)
        off[1:] = np.cumsum([len(p[2]) for p in plist])
        body = np.array([x for p in plist for x in p[2]], np.uint16)
        return Grammar(N, np.array([p[0] for p in plist], np.uint16), np.array([p[1] for p in plist], np.uint8),
                       off, body)

    rows, status, invalid = run(flat(g.N, swapped), g.N)
    assert invalid == 1 and (status == 2).all() and (rows == 0).all()
    assert run(flat(g.N, [p for p in prods for _ in range(2)]), g.N)[2] == 1      # every production twice
    rows, status, invalid = run(g, int(g.head.max()))        # a head >= N
    assert invalid == 1 and (status == 2).all()
    # body offsets that decrease, start above 0, or end short of the stated total
    for damage in ("decrease", "start", "end"):
        bad = Grammar(g.N, g.head, g.byte, g.body_off.copy(), g.body)
        if damage == "decrease":
            k = int(np.nonzero(g.length >= 2)[0][0])
            bad.body_off[k + 1] = bad.body_off[k] - 1 if bad.body_off[k] > 0 else bad.body_off[k + 2] + 1
        elif damage == "start":
            bad.body_off[0] = 1
        else:
            bad.body_off[-1] -= 1
        assert run(bad, g.N)[2] == 1, damage


def test_long_bodies(lib):
    """Productions with more body symbols than a fixed-width record would hold: six and nine
    symbols, a body as long as the stack limit, and one beyond it (its tokens overflow)."""
    print("case long bodies", flush=True)
    a = ord("a")
    prods = [(0, ord("s"), (1, 2, 3, 1, 2, 3)), (0, ord("t"), (1,) * 9), (0, ord("u"), (2,) * D.LIMIT_STACK),
             (0, ord("v"), (2,) * (D.LIMIT_STACK + 1)), (1, a, ()), (2, ord("b"), ()), (3, ord("c"), ()),
             (1, ord("x"), (3, 3, 3, 3, 3)), (3, ord("c"), (1,))]
    g = grammar_from_productions(4, prods)
    _check_adjacency(lib, g)
    toks = [b"s", b"sa", b"sab", b"sabc", b"sabcab", b"sabcabc", b"t", b"t" + b"a" * 9, b"taaaa", b"u", b"ub",
            b"u" + b"b" * D.LIMIT_STACK, b"v", b"vb", b"sx", b"sxccccc", b"sxcacccc", b"abc", b""]
    rows, status, _ = _check_rows(lib, g, vocab_from_tokens(toks), row_len=512)
    assert status[toks.index(b"v")] == 1 and status[toks.index(b"vb")] == 1
    assert status[toks.index(b"u")] == 0 and status[toks.index(b"sabcabc")] == 0
    assert D.decode_displacement(rows[0]) == frozenset({((0,), (1, 2, 3, 1, 2, 3))})
    # random grammars with bodies of up to eight symbols
    for seed in range(4):
        g = make_random_gnf(900 + seed, n_nt=6 + seed, alphabet=b"abcd", n_prod=30 + 6 * seed, max_body=8,
                            unary_fraction=0.5)
        assert g.length.max() >= 6
        _check_adjacency(lib, g)
        _check_rows(lib, g, _all_tokens(b"abcd", 4))


def test_argument_errors(lib):
    from gpu_util import dev
    g = make_random_gnf(9, n_nt=6, alphabet=b"ab", n_prod=14)
    vocab = _all_tokens(b"ab", 2)
    tb, to = dev(vocab.tok_bytes), dev(vocab.tok_off)
    with pytest.raises(lib.CfgzipError):
        lib.cfgzip_displacements(tb, to, *_grammar_dev(g), 5000)
    with pytest.raises(lib.CfgzipError):
        lib.cfgzip_displacements(tb, to, *_grammar_dev(g), g.N,
                                 workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    with pytest.raises(lib.CfgzipError):   # no automaton and no rows
        lib.cfgzip_build_classes(tb, to, None, None, torch.zeros(vocab.V, dtype=torch.int64, device="cuda"))


def test_json_grammar_full_vocabulary(lib):
    """The measured workload at full size: the JSON grammar against config 3's 128,256 tokens,
    every token against Algorithm 1, the classes against the oracle's grouping of its own rows."""
    print("case json grammar, full vocabulary", flush=True)
    from synthetic_inputs.grammar import make_json_gnf
    g = make_json_gnf()
    vocab = si.make_config(3)["vocab"]
    _check_adjacency(lib, g)
    rows, status, c = _check_rows(lib, g, vocab)
    # long digit runs hold deep queues; the longest sets need more than 256 entries
    ok = status == D.DISP_OK
    assert 0 < (~ok).sum() < 2000
    long_ok = [t for t in np.nonzero(ok)[0] if vocab.tok_off[t + 1] - vocab.tok_off[t] >= 13]
    assert any(len(q) > KERNEL_FIRST_ATTEMPT[0] for t in long_ok for (q, _s) in D.decode_displacement(rows[t]))
    assert len(set(c.tolist())) < vocab.V // 50
    _check_rows(lib, g, vocab, row_len=1024, expect_overflow=False)


def test_clike_grammar_full_vocabulary(lib):
    """The second measured grammar: statements and expressions with nesting and keywords, against
    config 3's vocabulary, every token."""
    print("case c-like grammar, full vocabulary", flush=True)
    from synthetic_inputs.grammar import make_clike_gnf
    g = make_clike_gnf()
    vocab = si.make_config(3)["vocab"]
    _check_adjacency(lib, g)
    _rows, status, c = _check_rows(lib, g, vocab, expect_overflow=False)
    assert len(set(c.tolist())) < vocab.V // 50


def test_many_random_grammars(lib):
    """Sixty grammars of random shape (1-40 symbols, 1-6 terminals, bodies up to 1-4, sparse to
    dense), 300 random tokens each, random row length: relation, rows, hashes, status, classes."""
    rng = np.random.default_rng(2024)
    seen_overflow = seen_ok = 0
    for case in range(60):
        n_nt, asz = int(rng.integers(1, 40)), int(rng.integers(1, 7))
        alphabet = bytes(rng.choice(np.arange(97, 123), size=asz, replace=False).astype(np.uint8))
        max_body = int(rng.integers(1, 5))
        possible = n_nt * asz * sum(n_nt ** k for k in range(0, max_body + 1))
        n_prod = max(n_nt, min(int(rng.integers(n_nt, min(n_nt * asz * 6, 400) + n_nt)), possible // 2))
        seed = int(rng.integers(1 << 30))
        print(f"case {case}: N={n_nt} terminals={asz} P={n_prod} body<={max_body} seed={seed}", flush=True)
        g = make_random_gnf(seed, n_nt=n_nt, alphabet=alphabet, n_prod=n_prod, max_body=max_body,
                            unary_fraction=float(rng.uniform(0.1, 0.7)))
        vocab = make_token_strings(seed + 1, 300, alphabet + b"z", int(rng.integers(1, 12)))
        _check_adjacency(lib, g)
        _rows, status, _c = _check_rows(lib, g, vocab, row_len=int(rng.choice([256, 512, 1024])))
        seen_overflow += int((status == D.DISP_OVERFLOW).sum())
        seen_ok += int((status == D.DISP_OK).sum())
    assert seen_overflow > 1000 and seen_ok > 5000


def test_status_pointer_is_optional(lib):
    """status_out = NULL: rows and hashes are the same, nothing else is written."""
    print("case no status array", flush=True)
    import ctypes
    from gpu_util import dev, hash_np
    g, atoms = make_bracket_gnf(5)
    vocab = make_token_strings(6, 700, atoms + b"()[]{},+-*", 6)
    tb, to = dev(vocab.tok_bytes), dev(vocab.tok_off)
    gd = _grammar_dev(g)
    rows, hashes, _status = lib.cfgzip_displacements(tb, to, *gd, g.N, hash_seed=SEED)
    raw = lib.load_library()
    rows2 = torch.zeros_like(rows)
    hashes2 = torch.zeros_like(hashes)
    ws = torch.empty(raw.cfgzip_displacements_workspace_bytes(vocab.V, g.N, g.P), dtype=torch.uint8, device="cuda")
    rc = raw.cfgzip_displacements(tb.data_ptr(), to.data_ptr(), vocab.V, gd[0].data_ptr(), gd[1].data_ptr(),
                                  gd[2].data_ptr(), gd[3].data_ptr(), g.body.size, g.P, g.N, rows2.data_ptr(), 256,
                                  hashes2.data_ptr(), None, ctypes.c_uint64(SEED), ws.data_ptr(), ws.numel(),
                                  None)
    assert rc == 0
    torch.cuda.synchronize()
    assert (rows2.cpu().numpy() == rows.cpu().numpy()).all()
    assert (hash_np(hashes2) == hash_np(hashes)).all()


def test_deep_queues_with_sixteen_bit_symbols(lib):
    """More than 255 symbols and queues beyond what the kernel's first attempt holds: the second
    attempt's 16-bit records (its largest LDS footprint)."""
    print("case deep queues, 300 symbols", flush=True)
    a, in1, in2 = ord("a"), KERNEL_FIRST_ATTEMPT[0], D.LIMIT_QUEUE
    prods = [(0, ord("x"), (299, 299)), (299, a, ()), (299, ord("b"), (298, 297, 296, 295)),
             (298, ord("c"), ()), (297, ord("c"), (298,)), (296, ord("c"), ()), (295, ord("c"), (296, 296))]
    prods += [(i, ord("z"), (i + 1,)) for i in range(1, 290)]      # fillers: 300 symbols in use
    g = grammar_from_productions(300, prods)
    toks = [b"a" * n for n in (1, in1, in1 + 1, 20, in2, in2 + 1)] + [b"a" * 15 + b"b" + b"c" * k for k in range(6)]
    rows, status, _ = _check_rows(lib, g, vocab_from_tokens(toks))
    assert status.tolist() == [0, 0, 0, 0, 0, 1] + [0] * 6
    assert D.decode_displacement(rows[4]) == frozenset({((299,) * in2, ())})
