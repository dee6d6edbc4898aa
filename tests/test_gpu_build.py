"""GPU parity, offline path: cfgzip_signatures and cfgzip_build_classes against
the CPU oracle, bit for bit, on the four class-build configurations and on edge
cases (tiny and odd state counts, empty / long / duplicate tokens, forced hash
collisions, hash seeds)."""

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from synthetic_inputs.vocab import vocab_from_tokens

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lib():
    import paper_2605_29986_amd as p
    p.load_library()
    return p


def _random_vocab(rng, V, max_len, n_bytes=256, empties=True):
    toks = []
    for _ in range(V):
        k = int(rng.integers(0 if empties else 1, max_len + 1))
        toks.append(rng.integers(0, n_bytes, size=k, dtype=np.uint8).tobytes())
    return vocab_from_tokens(toks)


def _check_signatures(lib, vocab, table, seed=None):
    from gpu_util import vocab_dev, hash_np
    seed = lib.DEFAULT_HASH_SEED if seed is None else seed
    tb, to, tt = vocab_dev(vocab, table)
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    want_hash = oracle.signature_hash(want_sig, seed)
    sig, h = lib.cfgzip_signatures(tb, to, tt, hash_seed=seed)
    torch.cuda.synchronize()
    assert (sig.cpu().numpy() == want_sig).all(), "signatures"
    assert (hash_np(h) == want_hash).all(), "hash (with signatures stored)"
    _, h2 = lib.cfgzip_signatures(tb, to, tt, want_sig=False, hash_seed=seed)
    assert (hash_np(h2) == want_hash).all(), "hash (on the fly)"
    sig3, _ = lib.cfgzip_signatures(tb, to, tt, want_hash=False, hash_seed=seed)
    assert (sig3.cpu().numpy() == want_sig).all(), "signatures (no hash)"
    return want_sig, sig, h


def _check_build(lib, vocab, table, stored=True, hash_override=None, use_store=None):
    """Builds the classes and compares them with the oracle's.  `use_store`: hand the
    signature call's workspace to the class builder (True), do not (False), or both (None)."""
    from gpu_util import vocab_dev, dev
    tb, to, tt = vocab_dev(vocab, table)
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    want_c, want_r = oracle.build_classes(want_sig, vocab.tok_off)
    V, S = vocab.V, table.shape[0]
    ws = torch.empty(lib.load_library().cfgzip_signatures_workspace_bytes(V, S), dtype=torch.uint8,
                     device="cuda")
    sig, h = lib.cfgzip_signatures(tb, to, tt, want_sig=stored, workspace=ws)
    if hash_override is not None:
        h = hash_override(h)
    out = None
    for with_store in ([True, False] if use_store is None else [use_store]):
        c, r, C, coll = lib.cfgzip_build_classes(tb, to, tt, sig if stored else None, h,
                                                 signatures_workspace=ws if with_store else None)
        assert C == len(want_r), (with_store, C, len(want_r))
        assert (c.cpu().numpy() == want_c).all(), f"class_of_token (store={with_store})"
        assert (r.cpu().numpy() == want_r).all(), f"rep_of_class (store={with_store})"
        if out is not None:
            assert (C, coll > 0) == (out[0], out[1] > 0)
        out = (C, coll)
    return out


@pytest.mark.parametrize("S", [1, 2, 3, 24, 33, 63, 64, 65, 100, 128, 129, 200, 256, 257, 288, 289,
                               300, 513, 1000])
def test_signatures_state_counts(lib, S):
    print(f"case S={S}", flush=True)
    rng = np.random.default_rng(S)
    table = rng.integers(0, S, size=(S, 256)).astype(np.uint16)
    vocab = _random_vocab(rng, 257, 9)
    _check_signatures(lib, vocab, table)


@pytest.mark.parametrize("S", [9000, 40000, 65536])
def test_large_state_counts(lib, S):
    """State counts whose walk vectors need more than the minimum LDS buffer (S > 8192)
    and, for the re-walk verification, more than LDS holds (2 S entries > 144 KB)."""
    print(f"case S={S}", flush=True)
    rng = np.random.default_rng(S)
    table = rng.integers(0, S, size=(S, 256)).astype(np.uint16)
    table[:, 65:91] = (np.arange(S)[:, None] % 7).astype(np.uint16)  # a few narrow columns
    toks = [b"", b"A", b"AB", b"Ab", b"ab", b"abc", b"ab", b"zzzz", b"B", b"A"] * 3
    toks += [rng.integers(0, 256, size=int(rng.integers(1, 6)), dtype=np.uint8).tobytes()
             for _ in range(40)]
    vocab = vocab_from_tokens(toks)
    _check_signatures(lib, vocab, table)
    _check_build(lib, vocab, table, stored=False)
    _check_build(lib, vocab, table, stored=True)


def test_signatures_long_and_empty_tokens(lib):
    rng = np.random.default_rng(0)
    for S in (24, 256, 700):
        print(f"case long tokens S={S}", flush=True)
        table = rng.integers(0, S, size=(S, 256)).astype(np.uint16)
        toks = [b"", b"a", rng.integers(0, 256, size=5000, dtype=np.uint8).tobytes(),
                rng.integers(0, 256, size=64, dtype=np.uint8).tobytes(),
                rng.integers(0, 256, size=65, dtype=np.uint8).tobytes(), b"",
                rng.integers(0, 256, size=200, dtype=np.uint8).tobytes(),
                rng.integers(0, 256, size=129, dtype=np.uint8).tobytes(), b"zz", b""]
        toks += [toks[2], toks[5], b"zz", toks[2]]  # duplicates: members to verify against a head
        _check_signatures(lib, vocab_from_tokens(toks), table)
        _check_build(lib, vocab_from_tokens(toks), table, stored=False)
        _check_build(lib, vocab_from_tokens(toks), table, stored=True)


def test_signatures_all_tokens_empty(lib):
    table = np.random.default_rng(1).integers(0, 70, size=(70, 256)).astype(np.uint16)
    _check_signatures(lib, vocab_from_tokens([b"", b"", b""]), table)


def test_signatures_hash_seeds(lib, cfg1):
    for seed in (0, 1, 0xFFFFFFFFFFFFFFFF, 1234567):
        _check_signatures(lib, cfg1["vocab"], cfg1["table"], seed=seed)


def test_config1_build(lib, cfg1):
    _check_signatures(lib, cfg1["vocab"], cfg1["table"])
    C, coll = _check_build(lib, cfg1["vocab"], cfg1["table"])
    assert coll == 0
    _check_build(lib, cfg1["vocab"], cfg1["table"], stored=False)


def test_config2_build(lib):
    cfg = si.make_config(2)
    _check_signatures(lib, cfg["vocab"], cfg["table"])
    C, coll = _check_build(lib, cfg["vocab"], cfg["table"])
    print("config 2: C =", C, "V/C =", cfg["vocab"].V / C, flush=True)
    assert coll == 0
    _check_build(lib, cfg["vocab"], cfg["table"], stored=False)


def test_config3_build(lib):
    cfg = si.make_config(3)
    _check_signatures(lib, cfg["vocab"], cfg["table"])
    C, coll = _check_build(lib, cfg["vocab"], cfg["table"])
    print("config 3: C =", C, "V/C =", cfg["vocab"].V / C, flush=True)
    assert coll == 0


def test_config4_build_hash_on_the_fly(lib):
    """Signatures are never stored: hashed on the fly, verified by re-walking."""
    from gpu_util import vocab_dev, hash_np
    cfg = si.make_config(4)
    vocab, table = cfg["vocab"], cfg["table"]
    tb, to, tt = vocab_dev(vocab, table)
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    want_c, want_r = oracle.build_classes(want_sig, vocab.tok_off)
    _, h = lib.cfgzip_signatures(tb, to, tt, want_sig=False)
    assert (hash_np(h) == oracle.signature_hash(want_sig, lib.DEFAULT_HASH_SEED)).all()
    c, r, C, coll = lib.cfgzip_build_classes(tb, to, tt, None, h)
    print("config 4: C =", C, "V/C =", vocab.V / C, "collisions =", coll, flush=True)
    assert C == len(want_r) and coll == 0
    assert (c.cpu().numpy() == want_c).all() and (r.cpu().numpy() == want_r).all()
    # the same, comparing the compressed signatures the signature call left in its workspace
    ws = torch.empty(lib.load_library().cfgzip_signatures_workspace_bytes(vocab.V, cfg["S"]),
                     dtype=torch.uint8, device="cuda")
    _, h = lib.cfgzip_signatures(tb, to, tt, want_sig=False, workspace=ws)
    c, r, C, coll = lib.cfgzip_build_classes(tb, to, tt, None, h, signatures_workspace=ws)
    assert C == len(want_r) and coll == 0
    assert (c.cpu().numpy() == want_c).all() and (r.cpu().numpy() == want_r).all()


@pytest.mark.parametrize("stored", [True, False])
@pytest.mark.parametrize("bits", [0, 3, 8])
def test_forced_hash_collisions(lib, cfg2_small, stored, bits):
    """A hash cut down to a few bits (still a function of the signature) forces
    thousands of collisions; classes and representatives must not change."""
    print(f"case stored={stored} bits={bits}", flush=True)
    mask = (1 << bits) - 1
    C, coll = _check_build(lib, cfg2_small["vocab"], cfg2_small["table"], stored=stored,
                           hash_override=lambda h: h & mask)
    assert coll > 0


def test_classes_do_not_depend_on_hash_seed(lib, cfg1):
    from gpu_util import vocab_dev
    tb, to, tt = vocab_dev(cfg1["vocab"], cfg1["table"])
    outs = []
    for seed in (1, 2, 3):
        sig, h = lib.cfgzip_signatures(tb, to, tt, hash_seed=seed)
        c, r, C, _ = lib.cfgzip_build_classes(tb, to, tt, sig, h)
        outs.append((c.cpu().numpy().copy(), r.cpu().numpy().copy(), C))
    for o in outs[1:]:
        assert o[2] == outs[0][2] and (o[0] == outs[0][0]).all() and (o[1] == outs[0][1]).all()


def test_build_edge_vocabularies(lib, cfg1):
    table = cfg1["table"]
    for toks in ([b"a"], [b"", b""], [b"ab", b"", b"ab", b"{", b"", b"ab"],
                 [bytes([97 + (i % 3)]) * (1 + i % 5) for i in range(2049)]):
        print("case vocabulary of", len(toks), flush=True)
        _check_build(lib, vocab_from_tokens(toks), table)
        _check_build(lib, vocab_from_tokens(toks), table, stored=False)


def test_build_random_automaton_every_token_its_own_class(lib):
    rng = np.random.default_rng(5)
    S = 300
    table = rng.integers(0, S, size=(S, 256)).astype(np.uint16)
    vocab = _random_vocab(rng, 5000, 6, empties=False)
    _check_build(lib, vocab, table)
    _check_build(lib, vocab, table, stored=False)


def _prefix_heavy_vocab(rng, V, alphabet=b"ab{ 1"):
    """Short strings over a tiny alphabet: nearly every token of four bytes or more has a
    two- or three-byte token as a prefix."""
    alpha = np.frombuffer(alphabet, dtype=np.uint8)
    toks = [bytes(alpha[rng.integers(0, len(alpha), size=int(rng.integers(0, 9)))]) for _ in range(V)]
    toks += [b"", b"a", b"ab", b"abb", b"abba", b"abbab" * 3, b"ab" * 40, bytes(200)]
    return vocab_from_tokens(toks)


@pytest.mark.parametrize("S", [7, 24, 256, 300, 1024])
def test_signatures_by_composition(lib, S):
    """cfgzip_signatures_composed (Appendix A, Lemma 1) against the oracle and against the plain
    call: signatures, hashes, and the kept walk vectors as the class builder reads them."""
    from gpu_util import vocab_dev, hash_np
    print(f"case composition S={S}", flush=True)
    rng = np.random.default_rng(3000 + S)
    raw = lib.load_library()
    for vocab, table in ((_prefix_heavy_vocab(rng, 3000), _structured_table(rng, S, n_narrow=256)),
                         (_prefix_heavy_vocab(rng, 700), rng.integers(0, S, size=(S, 256)).astype(np.uint16)),
                         (_random_vocab(rng, 900, 9, n_bytes=4), _structured_table(rng, S, n_narrow=2))):
        tb, to, tt = vocab_dev(vocab, table)
        want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
        want_hash = oracle.signature_hash(want_sig, lib.DEFAULT_HASH_SEED)
        want_c, want_r = oracle.build_classes(want_sig, vocab.tok_off)
        ws = torch.empty(raw.cfgzip_signatures_composed_workspace_bytes(vocab.V, S), dtype=torch.uint8, device="cuda")
        sig, h = lib.cfgzip_signatures(tb, to, tt, workspace=ws, composed=True)
        assert (sig.cpu().numpy() == want_sig).all(), "signatures"
        assert (hash_np(h) == want_hash).all(), "hash"
        c, r, C, _ = lib.cfgzip_build_classes(tb, to, tt, None, h, signatures_workspace=ws)
        assert C == len(want_r) and (c.cpu().numpy() == want_c).all() and (r.cpu().numpy() == want_r).all()
        _, h2 = lib.cfgzip_signatures(tb, to, tt, want_sig=False, workspace=ws, composed=True)
        assert (hash_np(h2) == want_hash).all(), "hash (on the fly)"
        sig3, _ = lib.cfgzip_signatures(tb, to, tt, want_hash=False, workspace=ws, composed=True)
        assert (sig3.cpu().numpy() == want_sig).all(), "signatures (no hash)"


def test_signatures_by_composition_config3(lib):
    from gpu_util import vocab_dev, hash_np
    cfg = si.make_config(3)
    vocab, table = cfg["vocab"], cfg["table"]
    tb, to, tt = vocab_dev(vocab, table)
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    sig, h = lib.cfgzip_signatures(tb, to, tt, composed=True)
    assert (sig.cpu().numpy() == want_sig).all()
    assert (hash_np(h) == oracle.signature_hash(want_sig, lib.DEFAULT_HASH_SEED)).all()


def test_random_automaton_at_scale(lib):
    """An automaton without structure at the size of the measured ones: every byte leaves about
    0.63 S distinct states, the image walk saves nothing, the walk vectors the signature call
    keeps overflow, and the builder falls back to walking again (or to stored rows).  Config 2's
    32,000 tokens against 1,024 uniformly random states; nearly every token is its own class."""
    print("case random automaton S=1024 V=32000", flush=True)
    rng = np.random.default_rng(4242)
    S = 1024
    table = rng.integers(0, S, size=(S, 256)).astype(np.uint16)
    table[0, :] = 0
    vocab = si.make_config(2)["vocab"]
    assert vocab.V >= 32000
    want_sig, _sig, _h = _check_signatures(lib, vocab, table)
    assert np.unique(want_sig[:2000], axis=0).shape[0] > 1000
    C, _coll = _check_build(lib, vocab, table, stored=False, use_store=True)   # store overflows -> second walk
    assert C > vocab.V // 2
    _check_build(lib, vocab, table, stored=False, use_store=False)
    _check_build(lib, vocab, table, stored=True)


def _structured_table(rng, S, n_narrow):
    """A random automaton in which `n_narrow` byte columns have few distinct states (like a
    lexer's) and the rest reject or scatter: mixes short and long walk vectors in one batch."""
    table = np.zeros((S, 256), dtype=np.uint16)
    for b in range(256):
        kind = rng.integers(0, 3) if b >= n_narrow else 0
        if kind == 0:      # few distinct targets
            k = int(rng.integers(1, min(S, 12) + 1))
            targets = rng.integers(0, S, size=k)
            table[:, b] = targets[rng.integers(0, k, size=S)]
        elif kind == 1:    # everything rejects
            table[:, b] = 0
        else:              # arbitrary
            table[:, b] = rng.integers(0, S, size=S)
    table[0, :] = 0        # state 0 absorbs
    return table


@pytest.mark.parametrize("seed", range(24))
def test_random_cases_against_oracle(lib, seed):
    """Random automata and vocabularies of many shapes: signatures, hash, classes and
    representatives with every source of signatures the class builder knows."""
    rng = np.random.default_rng(1000 + seed)
    S = int(rng.choice([1, 2, 7, 24, 63, 64, 65, 130, 255, 256, 257, 300, 511, 777, 1024, 1500, 2100]))
    V = int(rng.choice([1, 2, 63, 64, 65, 127, 129, 500, 2047, 2048, 2049, 3000]))
    max_len = int(rng.choice([1, 2, 4, 9, 40]))
    n_bytes = int(rng.choice([2, 5, 40, 256]))
    table = _structured_table(rng, S, n_narrow=int(rng.choice([0, n_bytes // 2, n_bytes])))
    vocab = _random_vocab(rng, V, max_len, n_bytes=n_bytes)
    print(f"case seed={seed} S={S} V={V} max_len={max_len} n_bytes={n_bytes}", flush=True)
    _check_signatures(lib, vocab, table)
    stored = bool(rng.integers(0, 2))
    _check_build(lib, vocab, table, stored=stored)
    # a weak hash on top: collisions inside and across first-byte groups
    _check_build(lib, vocab, table, stored=not stored, hash_override=lambda h: h & 0x3)


def test_million_token_vocabulary(lib):
    """Many tiles in the sort (489) and in the scans; the tiny automaton keeps the oracle fast."""
    cfg = si.make_config(1, V=1_000_003)
    vocab, table = cfg["vocab"], cfg["table"]
    _check_signatures(lib, vocab, table)
    C, coll = _check_build(lib, vocab, table)
    print("V = 1,000,003: C =", C, "collisions =", coll, flush=True)
    _check_build(lib, vocab, table, stored=False, use_store=False)
    # 393,149 classes squeezed into 2^20 hash values: tens of thousands of collisions at scale
    C2, coll2 = _check_build(lib, vocab, table, use_store=True, hash_override=lambda h: h & 0xFFFFF)
    print("with a 20-bit hash: collisions =", coll2, flush=True)
    assert C2 == C and coll2 > 1000


@pytest.mark.parametrize("V", [262_144, 262_145])
def test_vocabulary_sizes_around_the_switch_to_wider_keys(lib, V):
    """Up to 262,144 tokens the sort key holds 32 hash bits (four passes) and the ranking keeps its
    bit vector in LDS; one token more and it is 40 bits (five passes) and scan kernels."""
    print(f"case V={V}", flush=True)
    cfg = si.make_config(1, V=V)
    C, coll = _check_build(lib, cfg["vocab"], cfg["table"], use_store=True)
    assert coll == 0 and C > 1000
    _check_build(lib, cfg["vocab"], cfg["table"], stored=False, use_store=False,
                 hash_override=lambda h: h & 0xFFFF)


def test_signature_workspace_that_does_not_match_is_ignored(lib, cfg1, cfg2_small):
    """A workspace left by a call on another vocabulary / automaton, a zeroed one, and one
    whose compressed signatures overflowed (random automaton: ~0.63 S states per token, more
    than the 256 kept) must all give the same classes as no workspace at all."""
    from gpu_util import vocab_dev
    raw = lib.load_library()
    v1, t1 = cfg1["vocab"], cfg1["table"]
    v2, t2 = cfg2_small["vocab"], cfg2_small["table"]
    tb, to, tt = vocab_dev(v2, t2)
    want_sig = oracle.signatures(v2.tok_bytes, v2.tok_off, t2)
    want_c, want_r = oracle.build_classes(want_sig, v2.tok_off)
    need = max(raw.cfgzip_signatures_workspace_bytes(v1.V, 24),
               raw.cfgzip_signatures_workspace_bytes(v2.V, 256))
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    _, h = lib.cfgzip_signatures(tb, to, tt, want_sig=False)
    for case in ("zeroed", "other call"):
        print("case", case, flush=True)
        if case == "other call":
            lib.cfgzip_signatures(*vocab_dev(v1, t1), want_sig=False, workspace=ws)
        c, r, C, _ = lib.cfgzip_build_classes(tb, to, tt, None, h, signatures_workspace=ws)
        assert C == len(want_r)
        assert (c.cpu().numpy() == want_c).all() and (r.cpu().numpy() == want_r).all()
    print("case a workspace no larger than the smaller call needs", flush=True)
    small = torch.zeros(raw.cfgzip_signatures_workspace_bytes(v1.V, 24), dtype=torch.uint8, device="cuda")
    assert small.numel() < raw.cfgzip_signatures_workspace_bytes(v2.V, 256) // 4
    lib.cfgzip_signatures(*vocab_dev(v1, t1), want_sig=False, workspace=small)
    c, r, C, _ = lib.cfgzip_build_classes(tb, to, tt, None, h, signatures_workspace=small)
    assert C == len(want_r)
    assert (c.cpu().numpy() == want_c).all() and (r.cpu().numpy() == want_r).all()
    print("case empty tokens next to an automaton of more states than a kept vector holds", flush=True)
    rng = np.random.default_rng(78)
    S = 700
    table = _structured_table(rng, S, n_narrow=256)       # every column narrow: the vectors fit
    toks = [b"", b"ab", b"", b"ba", b"ab", b"a", b"", b"b"] * 40
    raw_ws = torch.zeros(raw.cfgzip_signatures_workspace_bytes(len(toks), S), dtype=torch.uint8, device="cuda")
    ev = vocab_from_tokens(toks)
    etb, eto, ett = vocab_dev(ev, table)
    _, eh = lib.cfgzip_signatures(etb, eto, ett, want_sig=False, workspace=raw_ws)
    hdr = raw_ws[:32].cpu().numpy().view(np.uint32)
    assert hdr[1] == len(toks) and hdr[2] == S and hdr[4] == 0, "the empty tokens must not mark the store overflowed"
    _check_build(lib, ev, table, stored=False, use_store=True)
    print("case overflow", flush=True)
    rng = np.random.default_rng(77)
    S = 1000
    table = rng.integers(0, S, size=(S, 256)).astype(np.uint16)
    vocab = _random_vocab(rng, 700, 5, empties=True)
    _check_build(lib, vocab, table, stored=False, use_store=True)
    _check_build(lib, vocab, table, stored=True, use_store=True)


def test_workspace_and_argument_errors(lib):
    raw = lib.load_library()
    assert raw.cfgzip_signatures_workspace_bytes(100, 0) == 0
    assert raw.cfgzip_signatures_workspace_bytes(100, 65537) == 0
    t = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    # no output requested
    assert raw.cfgzip_signatures(t.data_ptr(), t.data_ptr(), 4, t.data_ptr(), 2, None, None, 0,
                                 t.data_ptr(), 1024, None) == -1
    # workspace too small
    assert raw.cfgzip_signatures(t.data_ptr(), t.data_ptr(), 4, t.data_ptr(), 2, t.data_ptr(), None,
                                 0, t.data_ptr(), 16, None) == -2
