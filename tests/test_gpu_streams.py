"""Every entry point enqueues on the stream it is given: the whole path on a stream of its own,
with the results read only after that stream has been waited for, against the oracle."""

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from oracle import displacement as D
from synthetic_inputs.grammar import make_bracket_gnf, make_token_strings
from synthetic_inputs.nfa import add_transitions, nfa_from_dfa

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_whole_path_on_a_side_stream(cfg1):
    import paper_2605_29986_amd as lib
    from gpu_util import dev, hash_np, vocab_dev
    lib.load_library()
    table, vocab = cfg1["table"], cfg1["vocab"]
    tb, to, tt = vocab_dev(vocab, table)
    B = 16
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    want_c, want_r = oracle.build_classes(want_sig, vocab.tok_off)
    C = len(want_r)
    d = si.make_decode_inputs(cfg1["seed"] + 77, B, vocab.V, C, "bf16")
    logits = torch.from_numpy(d["logits"]).cuda().view(torch.bfloat16)
    cls_bits, tok = dev(d["cls_bits"]), dev(d["tok"])
    nfa_np = add_transitions(nfa_from_dfa(table), 5, 0.2)
    nfa = dev(nfa_np)
    g, atoms = make_bracket_gnf(5)
    gv = make_token_strings(6, 400, atoms + b"()[]{},+-*", 5)
    gtb, gto = dev(gv.tok_bytes), dev(gv.tok_off)
    gd = [dev(x) for x in g.arrays()]
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        sig, h = lib.cfgzip_signatures(tb, to, tt)
        c, r, got_C, coll = lib.cfgzip_build_classes(tb, to, tt, sig, h)
        tok_bits = torch.empty((B, (vocab.V + 31) // 32), dtype=torch.int32, device="cuda")
        lib.cfgzip_apply_mask(logits, cls_bits, class_of_token=c, C=C, tok_bits_out=tok_bits)
        expanded = lib.cfgzip_expand_mask(cls_bits, C, c)
        rep = lib.cfgzip_map_to_rep(tok, c, r)
        rel, rel_hash = lib.cfgzip_nfa_signatures(tb, to, nfa)
        rows, row_hash, status = lib.cfgzip_displacements(gtb, gto, *gd, g.N, hash_seed=3)
        adj, invalid = lib.cfgzip_stack_adjacency(*gd, g.N)
    side.synchronize()

    assert got_C == C and coll == 0
    assert (sig.cpu().numpy() == want_sig).all()
    assert (c.cpu().numpy() == want_c).all() and (r.cpu().numpy() == want_r).all()
    want_bits = oracle.expand_mask(d["cls_bits"], want_c, C)
    assert (tok_bits.cpu().numpy() == want_bits).all() and (expanded.cpu().numpy() == want_bits).all()
    assert (logits.view(torch.uint16).cpu().numpy() == oracle.apply_mask(d["logits"], want_bits, "bf16")).all()
    assert (rep.cpu().numpy() == oracle.map_to_rep(d["tok"], want_c, want_r)).all()
    assert (rel.cpu().numpy().view(np.uint32) == oracle.nfa_signatures(vocab.tok_bytes, vocab.tok_off, nfa_np)).all()
    want_rows, want_hash, want_status = D.displacement_rows(gv.tokens(), g.productions(), seed=3)
    assert (rows.cpu().numpy() == want_rows).all() and (hash_np(row_hash) == want_hash).all()
    assert (status.cpu().numpy() == want_status).all() and int(invalid.item()) == 0
    assert (adj.cpu().numpy().view(np.uint32) ==
            D.adjacency_bits(D.stack_adjacency(g.productions()), g.N)).all()


def test_class_builds_from_two_host_threads(cfg1, cfg2_small):
    """Two host threads, each with a stream, workspaces and outputs of its own, build classes at
    the same time (the call waits for its stream and keeps its counts in per-thread pinned
    memory): both must match the oracle, call after call."""
    import threading

    import paper_2605_29986_amd as lib
    from gpu_util import vocab_dev
    lib.load_library()
    jobs = []
    for cfg in (cfg1, cfg2_small):
        vocab, table = cfg["vocab"], cfg["table"]
        want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
        jobs.append((vocab_dev(vocab, table), oracle.build_classes(want_sig, vocab.tok_off)))
    torch.cuda.synchronize()
    errors = []

    def work(k):
        try:
            (tb, to, tt), (want_c, want_r) = jobs[k]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for rep in range(12):
                    ws = torch.empty(lib.load_library().cfgzip_signatures_workspace_bytes(to.numel() - 1, tt.shape[0]),
                                     dtype=torch.uint8, device="cuda")
                    _sig, h = lib.cfgzip_signatures(tb, to, tt, want_sig=False, workspace=ws, stream=stream)
                    c, r, C, coll = lib.cfgzip_build_classes(tb, to, tt, None, h, signatures_workspace=ws,
                                                             stream=stream)
                    if C != len(want_r) or coll != 0:
                        errors.append((k, rep, "count", C, coll))
                    if not (c.cpu().numpy() == want_c).all() or not (r.cpu().numpy() == want_r).all():
                        errors.append((k, rep, "classes"))
        except Exception as e:  # noqa: BLE001 - reported by the main thread
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads)
    assert not errors, errors[:3]
