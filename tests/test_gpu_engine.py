"""GPU parity, engine side for a byte automaton: cfgzip_state_masks, cfgzip_class_masks and
cfgzip_advance_states against the CPU oracle, bit for bit, and a closed decode loop (class mask
-> fused expand + apply -> sampled token -> state advance on the representative) whose every
step is compared with the oracle walking the real tokens byte by byte."""

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from synthetic_inputs.configs import words_for
from synthetic_inputs.vocab import vocab_from_tokens

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lib():
    import paper_2605_29986_amd as p
    p.load_library()
    return p


def _accepting(rng, S, fraction=0.35):
    accept = (rng.random(S) < fraction).astype(np.uint8)
    accept[0] = 0  # the absorbing reject state of the generators
    return accept


def _rep_signatures_on_gpu(lib, vocab, table, r):
    """Signatures of the representatives, computed by the library on their byte strings."""
    from gpu_util import vocab_dev
    reps = vocab_from_tokens([vocab.token(int(t)) for t in r])
    tb, to, tt = vocab_dev(reps, table)
    sig_rep, _ = lib.cfgzip_signatures(tb, to, tt, want_hash=False)
    return sig_rep


@pytest.mark.parametrize("C,S", [(1, 1), (5, 3), (31, 64), (32, 65), (33, 100), (70, 24), (257, 300),
                                 (1000, 1024), (2049, 130)])
def test_state_masks_shapes(lib, C, S):
    print(f"case C={C} S={S}", flush=True)
    from gpu_util import dev
    rng = np.random.default_rng(C * 7 + S)
    sig_rep = rng.integers(0, S, size=(C, S)).astype(np.uint16)
    live = (rng.random(S) < 0.5).astype(np.uint8)
    want = oracle.state_masks(sig_rep, live)
    got = torch.full((S, words_for(C)), -1, dtype=torch.int32, device="cuda")  # pad bits must be written 0
    lib.cfgzip_state_masks(dev(sig_rep), dev(live), state_mask=got)
    assert (got.cpu().numpy() == want).all()
    states = rng.integers(-2, S + 2, size=37).astype(np.int32)
    want_cls = oracle.class_masks(want, C, states)
    got_cls = lib.cfgzip_class_masks(got, C, dev(states))
    assert (got_cls.cpu().numpy() == want_cls).all()


def test_advance_states(lib):
    from gpu_util import dev
    rng = np.random.default_rng(11)
    C, S, V, B = 300, 200, 5000, 513
    sig_rep = rng.integers(0, S, size=(C, S)).astype(np.uint16)
    c = rng.integers(0, C, size=V).astype(np.int32)
    tok = rng.integers(-3, V + 3, size=B).astype(np.int32)
    states = rng.integers(-2, S + 2, size=B).astype(np.int32)
    want = oracle.advance_states(sig_rep, c, tok, states)
    got = lib.cfgzip_advance_states(dev(sig_rep), dev(c), dev(tok), dev(states))
    assert (got.cpu().numpy() == want).all()


@pytest.mark.parametrize("config", [1, 2])
def test_closed_decode_loop(lib, config):
    """Every step: the library's class mask, expanded and applied to logits, must equal the mask
    the definition gives token by token (live state after the token's bytes), and advancing on
    representatives must track the automaton walked on the sampled tokens themselves."""
    from gpu_util import dev, vocab_dev, logits_dev, logits_bits
    cfg = si.make_config(config, V=4096 if config == 1 else 6000)
    vocab, table = cfg["vocab"], cfg["table"]
    V, S = vocab.V, cfg["S"]
    tb, to, tt = vocab_dev(vocab, table)
    sig, h = lib.cfgzip_signatures(tb, to, tt)
    c_d, r_d, C, _ = lib.cfgzip_build_classes(tb, to, tt, sig, h)
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    want_c, want_r = oracle.build_classes(want_sig, vocab.tok_off)
    assert (c_d.cpu().numpy() == want_c).all() and (r_d.cpu().numpy() == want_r).all()

    rng = np.random.default_rng(cfg["seed"] + 5)
    accept = _accepting(rng, S)
    live = oracle.live_states(table, accept)
    sig_rep = _rep_signatures_on_gpu(lib, vocab, table, want_r)
    assert (sig_rep.cpu().numpy() == want_sig[want_r]).all()
    state_mask = lib.cfgzip_state_masks(sig_rep, dev(live))
    assert (state_mask.cpu().numpy() == oracle.state_masks(want_sig[want_r], live)).all()

    B, steps = 16, 10
    start = rng.integers(1, S, size=B).astype(np.int32)
    states = dev(start)
    direct = start.copy()  # the automaton walked on the real tokens, on the CPU
    for step in range(steps):
        cls = lib.cfgzip_class_masks(state_mask, C, states)
        x = rng.standard_normal((B, V)).astype(np.float32)
        lg = logits_dev(x, "f32")
        tok_bits = torch.empty((B, words_for(V)), dtype=torch.int32, device="cuda")
        lib.cfgzip_apply_mask(lg, cls, class_of_token=c_d, C=C, tok_bits_out=tok_bits)
        got_bits = np.unpackbits(tok_bits.cpu().numpy().view(np.uint8), axis=1, bitorder="little")[:, :V]
        masked = logits_bits(lg)
        for b in range(B):
            allowed = live[want_sig[:, direct[b]]] if 0 <= direct[b] < S else np.zeros(V, np.uint8)
            assert (got_bits[b] == allowed).all(), (step, b)
            want_row = np.where(allowed.astype(bool), x[b].view(np.uint32), np.uint32(0xFF800000))
            assert (masked[b] == want_row).all(), (step, b)
        tok = rng.integers(0, V, size=B).astype(np.int32)  # the sampler is not part of the path
        lib.cfgzip_advance_states(sig_rep, c_d, dev(tok), states)
        for b in range(B):
            q = int(direct[b])
            for byte in vocab.token(int(tok[b])):
                q = int(table[q, byte])
            direct[b] = q
        assert (states.cpu().numpy() == direct).all(), step


def test_engine_argument_errors(lib):
    raw = lib.load_library()
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    assert raw.cfgzip_state_masks(None, 1, 1, t.data_ptr(), t.data_ptr(), None) == -1
    assert raw.cfgzip_state_masks(t.data_ptr(), 1, 70000, t.data_ptr(), t.data_ptr(), None) == -1
    assert raw.cfgzip_class_masks(t.data_ptr(), 1, 1, t.data_ptr(), 0, t.data_ptr(), None) == -1
    assert raw.cfgzip_advance_states(t.data_ptr(), 1, 1, None, 1, t.data_ptr(), 1, t.data_ptr(), None) == -1


@pytest.mark.parametrize("which", ["cfg1", "cfg2_small"])
def test_representative_vocabulary(lib, which, request):
    print(f"case representative vocabulary {which}", flush=True)
    from gpu_util import dev, vocab_dev
    cfg = request.getfixturevalue(which)
    vocab, table = cfg["vocab"], cfg["table"]
    tb, to, tt = vocab_dev(vocab, table)
    sig, h = lib.cfgzip_signatures(tb, to, tt)
    c, r, C, _ = lib.cfgzip_build_classes(tb, to, tt, sig, h)
    rep_bytes, rep_off = lib.cfgzip_representative_vocabulary(tb, to, r.contiguous())
    want_bytes, want_off = oracle.representative_vocabulary(vocab.tok_bytes, vocab.tok_off, r.cpu().numpy())
    got_off = rep_off.cpu().numpy()
    assert (got_off == want_off).all()
    assert (rep_bytes.cpu().numpy()[:got_off[-1]] == want_bytes).all()
    # the engine's view: signatures of that vocabulary are the representatives' rows
    sig_rep, _ = lib.cfgzip_signatures(rep_bytes[:max(int(got_off[-1]), 1)].contiguous(), rep_off, tt,
                                       want_hash=False)
    assert (sig_rep.cpu().numpy() == sig.cpu().numpy()[r.cpu().numpy()]).all()


def test_representative_vocabulary_edge_cases(lib, cfg1):
    print("case representative vocabulary edges", flush=True)
    from gpu_util import dev
    vocab = cfg1["vocab"]
    tb, to = dev(vocab.tok_bytes), dev(vocab.tok_off)
    rng = np.random.default_rng(1)
    for n in (1, 2, 1023, 1024, 1025, 5000, 70001):
        ids = rng.integers(-3, vocab.V + 3, size=n).astype(np.int32)
        want_bytes, want_off = oracle.representative_vocabulary(vocab.tok_bytes, vocab.tok_off, ids)
        raw = lib.load_library()
        ids_dev = dev(ids)
        rep_off = torch.empty(n + 1, dtype=torch.int64, device="cuda")
        cap = int(want_off[-1])
        rep_bytes = torch.full((cap + 64,), 0xAB, dtype=torch.uint8, device="cuda")
        rc = raw.cfgzip_representative_vocabulary(tb.data_ptr(), to.data_ptr(), vocab.V, ids_dev.data_ptr(), n,
                                                  rep_off.data_ptr(), rep_bytes.data_ptr(), cap, None)
        assert rc == 0
        torch.cuda.synchronize()
        assert (rep_off.cpu().numpy() == want_off).all()
        got = rep_bytes.cpu().numpy()
        assert (got[:cap] == want_bytes).all() and (got[cap:] == 0xAB).all()
        # a capacity that is too small: nothing is written beyond it, the offsets still tell the need
        small = cap // 2
        rep_bytes.fill_(0xCD)
        rc = raw.cfgzip_representative_vocabulary(tb.data_ptr(), to.data_ptr(), vocab.V, ids_dev.data_ptr(), n,
                                                  rep_off.data_ptr(), rep_bytes.data_ptr(), small, None)
        assert rc == 0
        torch.cuda.synchronize()
        got = rep_bytes.cpu().numpy()
        assert (got[:small] == want_bytes[:small]).all() and (got[small:] == 0xCD).all()
        assert int(rep_off[-1].item()) == cap


@pytest.mark.parametrize("config,dtype", [(1, "f32"), (2, "bf16")])
def test_closed_decode_loop_in_one_launch_per_step(lib, config, dtype):
    """cfgzip_engine_step (advance on the last sampled tokens, class masks, fused expand + apply
    in one launch) against the definition, step by step, including sequences that fall into the
    reject state, an invalid state and out-of-range token ids."""
    from gpu_util import dev, vocab_dev, logits_dev, logits_bits
    cfg = si.make_config(config, V=4096 if config == 1 else 6000)
    vocab, table = cfg["vocab"], cfg["table"]
    V, S = vocab.V, cfg["S"]
    tb, to, tt = vocab_dev(vocab, table)
    sig, h = lib.cfgzip_signatures(tb, to, tt)
    c_d, r_d, C, _ = lib.cfgzip_build_classes(tb, to, tt, sig, h)
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    want_c, want_r = oracle.build_classes(want_sig, vocab.tok_off)
    rng = np.random.default_rng(cfg["seed"] + 6)
    live = oracle.live_states(table, _accepting(rng, S))
    sig_rep = _rep_signatures_on_gpu(lib, vocab, table, want_r)
    state_mask = lib.cfgzip_state_masks(sig_rep, dev(live))
    want_sm = oracle.state_masks(want_sig[want_r], live)

    B, steps = 19, 8         # 19 rows: a ragged last row chunk
    states_np = rng.integers(1, S, size=B).astype(np.int32)
    states_np[3] = S + 5     # not a state: everything is masked, the state stays invalid
    states = [dev(states_np), torch.empty(B, dtype=torch.int32, device="cuda")]
    tok_prev = None
    ninf = np.uint32(0xFF800000) if dtype == "f32" else np.uint16(0xFF80)
    for step in range(steps):
        if dtype == "f32":
            x = rng.standard_normal((B, V)).astype(np.float32).view(np.uint32)
        else:
            x = si.make_decode_inputs(step, B, V, C, "bf16")["logits"]
        lg = logits_dev(x, dtype)
        tok_bits = torch.full((B, words_for(V)), -1, dtype=torch.int32, device="cuda")
        src, dst = states[step % 2], states[(step + 1) % 2]
        out = lib.cfgzip_engine_step(lg, state_mask, C, c_d, sig_rep, None if tok_prev is None else dev(tok_prev),
                                     src, states_out=dst, tok_bits_out=tok_bits)
        assert out.data_ptr() == dst.data_ptr()
        # the definition: advance, then the class mask of the new state, expanded and applied
        if tok_prev is not None:
            states_np = oracle.advance_states(want_sig[want_r], want_c, tok_prev, states_np)
        assert (dst.cpu().numpy() == states_np).all(), step
        want_bits = oracle.expand_mask(oracle.class_masks(want_sm, C, states_np), want_c, C)
        assert (tok_bits.cpu().numpy() == want_bits).all(), step
        assert (logits_bits(lg) == oracle.apply_mask(x, want_bits, dtype)).all(), step
        allowed = np.unpackbits(want_bits.view(np.uint8), axis=1, bitorder="little")[:, :V].astype(bool)
        assert (logits_bits(lg)[~allowed] == ninf).all()
        assert not allowed[3].any()
        # the separate calls give the same
        cls = lib.cfgzip_class_masks(state_mask, C, dst)
        lg2 = logits_dev(x, dtype)
        lib.cfgzip_apply_mask(lg2, cls, class_of_token=c_d, C=C)
        assert (logits_bits(lg2) == logits_bits(lg)).all()
        tok_prev = rng.integers(0, V, size=B).astype(np.int32)
        tok_prev[5] = V + 1 if step == 2 else tok_prev[5]   # once: an id out of range -> state -1
    assert (states_np[[3, 5]] == -1).all()


def test_engine_step_argument_errors(lib):
    raw = lib.load_library()
    t = torch.zeros(256, dtype=torch.int32, device="cuda")
    p = t.data_ptr()
    ok = dict(logits=p, dtype=0, B=1, V=8, stride=8, sm=p, S=1, C=1, c=p, sr=p, tp=p, si=p, so=p + 64, tb=None)

    def call(**kw):
        a = dict(ok); a.update(kw)
        return raw.cfgzip_engine_step(a["logits"], a["dtype"], a["B"], a["V"], a["stride"], a["sm"], a["S"], a["C"],
                                      a["c"], a["sr"], a["tp"], a["si"], a["so"], a["tb"], None)
    assert call(so=p) == -1            # states_out must differ from states_in
    assert call(sr=None) == -1         # an advance needs the representatives' signatures
    assert call(S=70000) == -1 and call(stride=4) == -1 and call(dtype=7) == -1 and call(sm=None) == -1
    assert call(sr=None, tp=None) == 0
    torch.cuda.synchronize()
