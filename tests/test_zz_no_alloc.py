"""cfgzip_signatures_static (the entry point that allocates nothing: its tables live in device
memory that is part of the loaded library) against cfgzip_signatures, bit for bit, through the
C ABI: two calls in a row on one stream, the second with a smaller vocabulary and automaton, then
further shapes up to the largest automaton it takes, and the refusal beyond it."""

import ctypes

import numpy as np
import pytest

import synthetic_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SEED = 0xABCDEF0123


def _both(raw, vocab, table, want_sig=True, want_hash=True):
    """(sig, hash) of the workspace entry point and of the static one, as numpy arrays."""
    from gpu_util import dev
    V, S = vocab.V, table.shape[0]
    tb, to, tt = dev(vocab.tok_bytes), dev(vocab.tok_off), dev(table)
    stream = ctypes.c_void_p(int(torch.cuda.current_stream().cuda_stream))
    out = []
    for static in (False, True):
        sig = torch.full((V, S), 0xAAAA, dtype=torch.uint16, device="cuda") if want_sig else None
        h = torch.full((V,), -1, dtype=torch.int64, device="cuda") if want_hash else None
        args = [ctypes.c_void_p(tb.data_ptr() if tb.numel() else 0), ctypes.c_void_p(to.data_ptr()),
                ctypes.c_int32(V), ctypes.c_void_p(tt.data_ptr()), ctypes.c_int32(S),
                ctypes.c_void_p(sig.data_ptr() if want_sig else 0),
                ctypes.c_void_p(h.data_ptr() if want_hash else 0), ctypes.c_uint64(SEED)]
        if static:
            rc = raw.cfgzip_signatures_static(*args, stream)
        else:
            need = raw.cfgzip_signatures_workspace_bytes(V, S)
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            rc = raw.cfgzip_signatures(*args, ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(need), stream)
        assert rc == 0, (static, rc)
        torch.cuda.synchronize()
        out.append((sig.cpu().numpy() if want_sig else None, h.cpu().numpy() if want_hash else None))
    return out


def _same(pair):
    (sig_a, h_a), (sig_b, h_b) = pair
    if sig_a is not None:
        assert (sig_a == sig_b).all(), "signatures"
    if h_a is not None:
        assert (h_a == h_b).all(), "hashes"


def test_static_entry_point_matches_the_workspace_one():
    import paper_2605_29986_amd as lib
    raw = lib.load_library()
    print("case 1: 6,000 tokens x 256 states", flush=True)
    big = si.make_config(2, V=6000)
    _same(_both(raw, big["vocab"], big["table"]))
    print("case 2 (smaller, right after): 4,096 tokens x 24 states", flush=True)
    small = si.make_config(1)
    _same(_both(raw, small["vocab"], small["table"]))
    print("case 3: 3,000 tokens x 1,024 states, hash only, then rows only", flush=True)
    mid = si.make_config(3, V=3000)
    _same(_both(raw, mid["vocab"], mid["table"], want_sig=False))
    _same(_both(raw, mid["vocab"], mid["table"], want_hash=False))
    print("case 4: the largest automaton it takes, 2,000 tokens x 4,096 states", flush=True)
    top = si.make_config(4, V=2000)
    assert top["table"].shape[0] == lib.binding.STATIC_MAX_STATES
    _same(_both(raw, top["vocab"], top["table"]))
    print("case 5: back to the small one", flush=True)
    _same(_both(raw, small["vocab"], small["table"]))


def test_static_entry_point_against_the_oracle():
    import oracle
    import paper_2605_29986_amd as lib
    from gpu_util import dev, hash_np
    cfg = si.make_config(1)
    vocab, table = cfg["vocab"], cfg["table"]
    sig = torch.empty((vocab.V, cfg["S"]), dtype=torch.uint16, device="cuda")
    h = torch.empty((vocab.V,), dtype=torch.int64, device="cuda")
    lib.cfgzip_signatures_static(dev(vocab.tok_bytes), dev(vocab.tok_off), dev(table), sig, h, hash_seed=SEED)
    torch.cuda.synchronize()
    want = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    assert (sig.cpu().numpy() == want).all()
    assert (hash_np(h) == oracle.signature_hash(want, SEED)).all()


def test_static_entry_point_refuses_what_does_not_fit():
    import paper_2605_29986_amd as lib
    from gpu_util import dev
    raw = lib.load_library()
    S = lib.binding.STATIC_MAX_STATES + 1
    table = np.zeros((S, 256), dtype=np.uint16)
    tt, to, tb = dev(table), dev(np.array([0, 1], dtype=np.int64)), dev(np.array([65], dtype=np.uint8))
    h = torch.zeros(1, dtype=torch.int64, device="cuda")
    rc = raw.cfgzip_signatures_static(ctypes.c_void_p(tb.data_ptr()), ctypes.c_void_p(to.data_ptr()), 1,
                                      ctypes.c_void_p(tt.data_ptr()), S, None, ctypes.c_void_p(h.data_ptr()),
                                      ctypes.c_uint64(1), None)
    assert rc == -5
    with pytest.raises(lib.CfgzipError):
        lib.cfgzip_signatures_static(tb, to, tt, None, h)
    # bad arguments answer before any device work, as for the workspace entry point
    assert raw.cfgzip_signatures_static(None, None, 1, None, 5, None, None, ctypes.c_uint64(1), None) == -1


def test_static_entry_point_and_decode_step_in_a_captured_graph():
    """What the entry point is for: a HIP graph captures cfgzip_signatures_static and
    cfgzip_decode_step (neither allocates); the graph is replayed several times, with eager work and
    waits in between, and every replay is checked against the oracle."""
    import oracle
    import paper_2605_29986_amd as lib
    from gpu_util import dev, hash_np, logits_dev, logits_bits
    cfg = si.make_config(1)
    vocab, table = cfg["vocab"], cfg["table"]
    V, S = vocab.V, cfg["S"]
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    want_c, want_r = oracle.build_classes(want_sig, vocab.tok_off)
    C, B = len(want_r), 8
    d = si.make_decode_inputs(321, B, V, C, "bf16", sigma=2.0)
    want_bits = oracle.expand_mask(d["cls_bits"], want_c, C)
    want_logits = oracle.apply_mask(d["logits"], want_bits, "bf16")
    want_rep = oracle.map_to_rep(d["tok"], want_c, want_r)

    tb, to, tt = dev(vocab.tok_bytes), dev(vocab.tok_off), dev(table)
    sig = torch.zeros((V, S), dtype=torch.uint16, device="cuda")
    h = torch.zeros((V,), dtype=torch.int64, device="cuda")
    pristine = logits_dev(d["logits"], "bf16")
    logits = pristine.clone()
    cls, c_d, r_d, tok = dev(d["cls_bits"]), dev(want_c), dev(want_r), dev(d["tok"])
    tbits = torch.zeros((B, (V + 31) // 32), dtype=torch.int32, device="cuda")
    rep = torch.zeros((B,), dtype=torch.int32, device="cuda")

    def step():
        lib.cfgzip_signatures_static(tb, to, tt, sig, h, hash_seed=SEED)
        lib.cfgzip_decode_step(logits, cls, c_d, C, tok, r_d, tok_bits_out=tbits, rep_out=rep)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                      # first call on this device outside the capture: it looks the array up
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(4):
        print(f"replay {replay}", flush=True)
        logits.copy_(pristine)      # eager work between the replays
        sig.zero_(), h.zero_(), tbits.zero_(), rep.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert (sig.cpu().numpy() == want_sig).all(), replay
        assert (hash_np(h) == oracle.signature_hash(want_sig, SEED)).all(), replay
        assert (logits_bits(logits) == want_logits).all(), replay
        assert (tbits.cpu().numpy() == want_bits).all() and (rep.cpu().numpy() == want_rep).all(), replay
