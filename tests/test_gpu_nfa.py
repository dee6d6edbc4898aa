"""GPU parity, non-deterministic byte automata: cfgzip_nfa_signatures against the oracle bit
for bit (relations and hashes), and the classes cfgzip_build_classes forms from the relations."""

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from synthetic_inputs.nfa import add_transitions, make_lexer_nfa, nfa_from_dfa
from synthetic_inputs.vocab import vocab_from_tokens

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SEED = 0xC0FFEE


@pytest.fixture(scope="module")
def lib():
    import paper_2605_29986_amd as p
    p.load_library()
    return p


def _check(lib, vocab, nfa, classes=True):
    from gpu_util import dev, hash_np
    V, S, W = vocab.V, nfa.shape[1], nfa.shape[2]
    want = oracle.nfa_signatures(vocab.tok_bytes, vocab.tok_off, nfa)
    tb, to = dev(vocab.tok_bytes), dev(vocab.tok_off)
    rel, h = lib.cfgzip_nfa_signatures(tb, to, dev(nfa), hash_seed=SEED)
    got = rel.cpu().numpy().view(np.uint32)
    bad = np.nonzero((got != want).any(axis=(1, 2)))[0]
    assert bad.size == 0, (bad[:5], [vocab.token(int(i)) for i in bad[:5]])
    rows16 = np.ascontiguousarray(want).view(np.uint16).reshape(V, S * W * 2)
    assert (hash_np(h) == oracle.signature_hash(rows16, SEED)).all()
    if classes:
        rows = rel.view(torch.uint16).reshape(V, S * W * 2)
        c, r, C, _coll = lib.cfgzip_build_classes(tb, to, None, rows, h)
        want_c, want_r = oracle.build_classes(rows16, vocab.tok_off)
        assert C == len(want_r)
        assert (c.cpu().numpy() == want_c).all() and (r.cpu().numpy() == want_r).all()
        return want, want_c
    return want, None


def _random_nfa(rng, S, n_sym, per_row):
    """every (byte < n_sym, state) gets Poisson(per_row) successors"""
    W = (S + 31) // 32
    nfa = np.zeros((256, S, W), np.uint32)
    for b in range(n_sym):
        for q in range(S):
            for x in rng.integers(0, S, size=rng.poisson(per_row)):
                nfa[b, q, x >> 5] |= np.uint32(1 << (int(x) & 31))
    return nfa


@pytest.mark.parametrize("S", [1, 2, 31, 32, 33, 64, 65, 100, 128, 129, 160, 190, 200, 255, 256])
def test_random_relations(lib, S):
    print(f"case S={S}", flush=True)
    rng = np.random.default_rng(S)
    nfa = _random_nfa(rng, S, 4, 1.2)
    toks = [bytes(rng.integers(0, 5, size=int(n)).astype(np.uint8)) for n in rng.integers(0, 9, size=700)]
    toks += [b"", bytes([0, 1, 2, 3] * 40), bytes([9]), bytes([0] * 300)]
    want, _ = _check(lib, vocab_from_tokens(toks), nfa)
    assert want.any() and not want[len(toks) - 2].any()


@pytest.mark.parametrize("S", [257, 300, 512, 700, 1024])
def test_more_states_than_registers_hold(lib, S):
    """Automata of more than 256 states: the sets live in LDS.  Sparse relations (a lexer's shape)
    and a denser one; relations, hashes and classes against the oracle."""
    print(f"case large S={S}", flush=True)
    rng = np.random.default_rng(7000 + S)
    nfa = _random_nfa(rng, S, 4, 1.1)
    toks = [bytes(rng.integers(0, 5, size=int(n)).astype(np.uint8)) for n in rng.integers(0, 8, size=120)]
    toks += [b"", bytes([0, 1, 2, 3] * 20), bytes([9]), bytes([0] * 100)]
    want, _ = _check(lib, vocab_from_tokens(toks), nfa)
    assert want.any()
    if S <= 512:
        dense = _random_nfa(rng, S, 2, 3.0)
        toks = [bytes(rng.integers(0, 2, size=int(n)).astype(np.uint8)) for n in rng.integers(1, 6, size=60)]
        _check(lib, vocab_from_tokens(toks), dense)


def test_lexer_nfa_with_1024_states(lib):
    """Config 3's 1,024-state lexer with a tenth of its live transitions doubled, 1,500 tokens."""
    print("case lexer nfa S=1024", flush=True)
    cfg = si.make_config(3, V=1500)
    nfa = make_lexer_nfa(cfg["seed"] + 500, cfg["S"], 0.10)
    want, c = _check(lib, cfg["vocab"], nfa)
    assert len(set(c.tolist())) < cfg["vocab"].V


def test_engine_over_state_sets(lib, cfg2_small):
    """Closed decode loop over a non-deterministic lexer: class masks from state sets, fused
    expand + apply on the logits, advance on the representatives of sampled tokens.  Every step's
    class mask and state sets against the oracle; the token-level mask against the definition
    evaluated on every token's own relation (losslessness)."""
    from gpu_util import dev, logits_dev, logits_bits
    print("case nfa engine loop", flush=True)
    vocab, S = cfg2_small["vocab"], cfg2_small["S"]
    nfa = make_lexer_nfa(cfg2_small["seed"] + 500, S, 0.10)
    V, W = vocab.V, nfa.shape[2]
    tb, to = dev(vocab.tok_bytes), dev(vocab.tok_off)
    rel, h = lib.cfgzip_nfa_signatures(tb, to, dev(nfa), hash_seed=SEED)
    c, r, C, _ = lib.cfgzip_build_classes(tb, to, None, rel.view(torch.uint16).reshape(V, S * W * 2), h)
    want_rel = oracle.nfa_signatures(vocab.tok_bytes, vocab.tok_off, nfa)
    c_np, r_np = c.cpu().numpy(), r.cpu().numpy()
    rel_rep = rel[r.long()].contiguous()                         # plumbing: rows of the representatives
    rng = np.random.default_rng(11)
    accept = (rng.random(S) < 0.3).astype(np.uint8)
    live = oracle.nfa_live_states(nfa, accept)
    state_mask = lib.cfgzip_nfa_state_masks(rel_rep, dev(live))
    want_sm = oracle.nfa_state_masks(want_rel[r_np], live)
    assert (state_mask.cpu().numpy() == want_sm).all()
    B = 24
    members = np.zeros((B, W * 32), bool)
    for b in range(B):
        members[b, rng.integers(1, S, size=int(rng.integers(0, 4)))] = True
    sets_np = np.packbits(members, axis=1, bitorder="little").view(np.uint32)
    sets = dev(sets_np)
    unpack = lambda rows, n: np.unpackbits(np.ascontiguousarray(rows).view(np.uint8), axis=-1, bitorder="little")[..., :n].astype(bool)
    R = None
    for step in range(4):
        cls = lib.cfgzip_nfa_class_masks(state_mask, C, sets)
        want_cls = oracle.nfa_class_masks(want_sm, C, sets_np)
        assert (cls.cpu().numpy() == want_cls).all(), step
        d = si.make_decode_inputs(500 + step, B, V, C, "f32", sigma=2.0)
        lg = logits_dev(d["logits"], "f32")
        tbits = torch.empty((B, (V + 31) // 32), dtype=torch.int32, device="cuda")
        lib.cfgzip_apply_mask(lg, cls, class_of_token=c, C=C, tok_bits_out=tbits)
        # the definition, token by token: allowed iff some state of the set reaches a live state
        if R is None:
            R = unpack(want_rel, S)                                             # [V, S, S]
            reach_live = (R & live.astype(bool)[None, None, :]).any(axis=2)     # [V, S]
        cur = unpack(sets_np, S)
        want_tok = (cur[:, None, :] & reach_live[None, :, :]).any(axis=2)
        assert (unpack(tbits.cpu().numpy(), V) == want_tok).all(), step
        want_logits = oracle.apply_mask(d["logits"].view(np.uint32), np.packbits(
            np.pad(want_tok, ((0, 0), (0, (-V) % 32))), axis=1, bitorder="little").view(np.int32), "f32")
        assert (logits_bits(lg) == want_logits).all(), step
        # sample an allowed token where there is one (else any), advance on representatives
        tok = np.array([int(rng.choice(np.nonzero(want_tok[b])[0])) if want_tok[b].any() else int(rng.integers(V))
                        for b in range(B)], dtype=np.int32)
        if step == 1:
            tok[0] = -1
        lib.cfgzip_nfa_advance_states(rel_rep, c, dev(tok), sets)
        sets_np = oracle.nfa_advance_states(want_rel[r_np], c_np, tok, sets_np)
        assert (sets.cpu().numpy().view(np.uint32) == sets_np).all(), step
        # and that is where the tokens' own bytes lead
        for b in range(B):
            if tok[b] >= 0:
                assert (unpack(sets_np[b], S) == (cur[b][:, None] & R[tok[b]]).any(axis=0)).all()


def test_dense_relation_fills_every_row(lib):
    print("case dense", flush=True)
    rng = np.random.default_rng(3)
    nfa = _random_nfa(rng, 256, 2, 6.0)
    toks = [bytes(rng.integers(0, 2, size=int(n)).astype(np.uint8)) for n in rng.integers(1, 7, size=300)]
    want, _ = _check(lib, vocab_from_tokens(toks), nfa)
    long_ones = want[np.array([len(t) for t in toks]) >= 5]
    assert np.unpackbits(long_ones.view(np.uint8)).mean() > 0.95, "nearly every pair is reachable"


def test_deterministic_automaton_gives_the_byte_walk_classes(lib, cfg1, cfg2_small):
    from gpu_util import vocab_dev
    for cfg in (cfg1, cfg2_small):
        print(f"case config {cfg['index']}", flush=True)
        table, vocab = cfg["table"], cfg["vocab"]
        _want, c_rel = _check(lib, vocab, nfa_from_dfa(table))
        tb, to, tt = vocab_dev(vocab, table)
        sig, h = lib.cfgzip_signatures(tb, to, tt)
        c_walk, _r, _C, _ = lib.cfgzip_build_classes(tb, to, tt, sig, h)
        assert (c_walk.cpu().numpy() == c_rel).all()


def test_lexer_nfa_full_vocabulary(lib):
    """The measured workload: config 2's vocabulary against its lexer with a tenth of the live
    transitions doubled."""
    print("case lexer nfa, config 2", flush=True)
    cfg = si.make_config(2)
    nfa = make_lexer_nfa(cfg["seed"] + 500, cfg["S"], 0.10)
    want, c = _check(lib, cfg["vocab"], nfa)
    det, c_det = _check(lib, cfg["vocab"], nfa_from_dfa(cfg["table"]), classes=True)
    assert ((want & det) == det).all(), "added transitions only add pairs"
    assert len(set(c.tolist())) != len(set(c_det.tolist()))


def test_hash_is_optional(lib, cfg1):
    from gpu_util import dev
    vocab = cfg1["vocab"]
    nfa = add_transitions(nfa_from_dfa(cfg1["table"]), 3, 0.3)
    tb, to, nd = dev(vocab.tok_bytes), dev(vocab.tok_off), dev(nfa)
    rel, h = lib.cfgzip_nfa_signatures(tb, to, nd)
    rel2, h2 = lib.cfgzip_nfa_signatures(tb, to, nd, want_hash=False)
    assert h2 is None and h is not None
    assert (rel.cpu().numpy() == rel2.cpu().numpy()).all()
    assert (rel.cpu().numpy().view(np.uint32) == oracle.nfa_signatures(vocab.tok_bytes, vocab.tok_off, nfa)).all()


def test_nfa_engine_argument_errors(lib):
    raw = lib.load_library()
    assert raw.cfgzip_nfa_state_masks(None, 1, 1, None, None, None) == -1
    assert raw.cfgzip_nfa_class_masks(None, 1, 1, None, 1, None, None) == -1
    assert raw.cfgzip_nfa_advance_states(None, 1, 1, None, 1, None, 1, None, None) == -1


def test_argument_errors(lib):
    from gpu_util import dev
    v = vocab_from_tokens([b"a", b"b"])
    tb, to = dev(v.tok_bytes), dev(v.tok_off)
    with pytest.raises(lib.CfgzipError):
        lib.cfgzip_nfa_signatures(tb, to, torch.zeros((256, 1025, 33), dtype=torch.int32, device="cuda"))
    with pytest.raises(ValueError):
        lib.cfgzip_nfa_signatures(tb, to, torch.zeros((256, 40, 1), dtype=torch.int32, device="cuda"))
