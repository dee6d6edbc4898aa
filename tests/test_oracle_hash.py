"""Pins for the oracle's copy of the library's signature hash
H(t) = sum_q a_q * sig[t][q] mod 2^64, a_q = SplitMix64 stream | 1."""

import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_seed1234567.txt")


def test_splitmix64_published_vector():
    want = [int(l) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    got = oracle.splitmix64_stream(1234567, len(want))
    assert [int(x) for x in got] == want


def test_unit_vectors_give_the_multipliers():
    S, seed = 13, 99
    a = oracle.splitmix64_stream(seed, S) | np.uint64(1)
    sig = np.eye(S, dtype=np.uint16)
    assert (oracle.signature_hash(sig, seed) == a).all()
    assert (oracle.signature_hash(np.zeros((1, S), dtype=np.uint16), seed) == 0).all()


def test_linearity_mod_2_64():
    rng = np.random.default_rng(0)
    S, seed = 40, 7
    x = rng.integers(0, 30000, size=(20, S)).astype(np.uint16)
    y = rng.integers(0, 30000, size=(20, S)).astype(np.uint16)
    hx, hy = oracle.signature_hash(x, seed), oracle.signature_hash(y, seed)
    hxy = oracle.signature_hash((x + y).astype(np.uint16), seed)
    with np.errstate(over="ignore"):
        assert (hxy == hx + hy).all()
    # python big-int evaluation of the formula for one row
    a = [int(v) | 1 for v in oracle.splitmix64_stream(seed, S)]
    assert int(hx[0]) == sum(ai * int(xi) for ai, xi in zip(a, x[0])) % (1 << 64)


def test_position_matters():
    sig = np.array([[1, 2, 3], [3, 2, 1], [2, 1, 3]], dtype=np.uint16)
    h = oracle.signature_hash(sig, 5)
    assert len(set(int(v) for v in h)) == 3
