"""Pins for the oracle's byte-walk signature (regular case of the paper's
displacement, Section 3.2.1 / Algorithm 1): closed-form automata, the
composition law of a transition monoid, and one-byte tokens."""

import numpy as np
import pytest

import oracle
from synthetic_inputs.vocab import vocab_from_tokens, make_vocab_uniform


def _sig(tokens, table):
    v = vocab_from_tokens(tokens)
    return oracle.signatures(v.tok_bytes, v.tok_off, table)


def _random_tokens(rng, n, max_len, alphabet=None):
    out = []
    for _ in range(n):
        k = int(rng.integers(0, max_len + 1))
        if alphabet is None:
            out.append(rng.integers(0, 256, size=k, dtype=np.uint8).tobytes())
        else:
            out.append(bytes(rng.choice(list(alphabet), size=k).astype(np.uint8)))
    return out


def test_identity_automaton_gives_identity_signature():
    S = 37
    table = np.repeat(np.arange(S, dtype=np.uint16)[:, None], 256, axis=1)
    rng = np.random.default_rng(1)
    sig = _sig(_random_tokens(rng, 50, 9), table)
    assert (sig == np.arange(S)[None, :]).all()


def test_all_reject_automaton():
    S = 11
    table = np.zeros((S, 256), dtype=np.uint16)
    rng = np.random.default_rng(2)
    toks = [t for t in _random_tokens(rng, 40, 6) if len(t) > 0]
    assert (_sig(toks, table) == 0).all()


def test_empty_token_is_identity(cfg1):
    sig = _sig([b"", b"a", b""], cfg1["table"])
    S = cfg1["S"]
    assert (sig[0] == np.arange(S)).all() and (sig[2] == np.arange(S)).all()


def test_counter_automaton_depends_only_on_length():
    # delta(0, b) = 0; delta(q, b) = 1 + (q mod (S-1)): one cycle through states 1..S-1
    S = 8
    table = np.zeros((S, 256), dtype=np.uint16)
    for q in range(1, S):
        table[q, :] = 1 + (q % (S - 1))
    rng = np.random.default_rng(3)
    toks = _random_tokens(rng, 200, 20)
    sig = _sig(toks, table)
    for t, row in zip(toks, sig):
        assert row[0] == 0
        for q in range(1, S):
            assert row[q] == 1 + ((q - 1 + len(t)) % (S - 1))


def test_first_byte_automaton():
    # state 1 jumps to sink 2 + (byte mod K); sinks are absorbing
    K = 5
    S = 2 + K
    table = np.zeros((S, 256), dtype=np.uint16)
    table[1, :] = 2 + (np.arange(256) % K)
    for k in range(K):
        table[2 + k, :] = 2 + k
    rng = np.random.default_rng(4)
    toks = [t for t in _random_tokens(rng, 200, 7) if t]
    sig = _sig(toks, table)
    for t, row in zip(toks, sig):
        assert row[0] == 0 and row[1] == 2 + (t[0] % K)
        assert (row[2:] == np.arange(2, S)).all()


def test_single_byte_tokens_read_one_table_column(cfg2_small):
    table = cfg2_small["table"]
    toks = [bytes([b]) for b in range(256)]
    sig = _sig(toks, table)
    assert (sig == table.T).all()  # sig[b][q] == table[q][b]; a transposed operand fails here


def test_byte_order_matters():
    # table where 'a' then 'b' differs from 'b' then 'a' (catches a reversed walk)
    S = 4
    table = np.zeros((S, 256), dtype=np.uint16)
    table[1, ord("a")] = 2
    table[2, ord("b")] = 3
    table[3, :] = 3
    sig = _sig([b"ab", b"ba"], table)
    assert sig[0, 1] == 3 and sig[1, 1] == 0


@pytest.mark.parametrize("which", ["cfg1", "cfg2_small"])
def test_composition_law(which, request):
    """sig(t u)[q] == sig(u)[ sig(t)[q] ] for concatenated tokens."""
    cfg = request.getfixturevalue(which)
    v, table = cfg["vocab"], cfg["table"]
    rng = np.random.default_rng(5)
    ids = rng.integers(0, v.V, size=(300, 2))
    toks = v.tokens()
    cat = [toks[a] + toks[b] for a, b in ids]
    sig = oracle.signatures(v.tok_bytes, v.tok_off, table)
    sig_cat = _sig(cat, table)
    for (a, b), row in zip(ids, sig_cat):
        assert (row == sig[b][sig[a]]).all()


def test_signature_is_the_product_of_transition_matrices():
    """Linear-algebra form: with M_b[q][q'] = 1 iff the automaton goes from q to q' on byte b,
    row q of the product M_{t_1} .. M_{t_n} (numpy matrix products) is the unit vector of
    sig[t][q].  A swapped operand order or a transposed table breaks it."""
    rng = np.random.default_rng(6)
    for S in (1, 2, 5, 9):
        table = rng.integers(0, S, size=(S, 256)).astype(np.uint16)
        M = np.zeros((256, S, S), dtype=np.int64)
        for b in range(256):
            M[b, np.arange(S), table[:, b]] = 1
        toks = _random_tokens(rng, 30, 5)
        sig = _sig(toks, table)
        for t, row in zip(toks, sig):
            prod = np.eye(S, dtype=np.int64)
            for byte in t:
                prod = prod @ M[byte]
            assert (prod.sum(axis=1) == 1).all()
            assert (prod.argmax(axis=1) == row).all()


def test_uniform_vocab_shapes():
    v = make_vocab_uniform(7, V=100, max_len=8)
    assert v.V == 100 and v.tok_off[-1] == len(v.tok_bytes)
    assert v.lengths.min() >= 1 and v.lengths.max() <= 8
