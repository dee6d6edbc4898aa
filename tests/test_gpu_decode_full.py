"""GPU parity at the benchmark's full decode-step size (batch 256, V = 128,256,
C = 8,000, bf16 logits), in the launch configuration bench.py times: the fused
expand + apply with the token mask as by-product and the map to
representatives, as two calls and as the single-launch decode step.  The class map comes from the config-3 class build (HIP and
oracle builds are compared first), resized to exactly 8,000 classes."""

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from synthetic_inputs.configs import words_for

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_config5_full_size():
    import paper_2605_29986_amd as lib
    from gpu_util import dev, vocab_dev, logits_dev, logits_bits
    cfg = si.make_config(5)
    vocab, table = cfg["vocab"], cfg["table"]
    tb, to, tt = vocab_dev(vocab, table)
    sig, h = lib.cfgzip_signatures(tb, to, tt)
    c3, r3, C3, _ = lib.cfgzip_build_classes(tb, to, tt, sig, h)
    want_sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    want_c3, want_r3 = oracle.build_classes(want_sig, vocab.tok_off)
    assert (c3.cpu().numpy() == want_c3).all() and (r3.cpu().numpy() == want_r3).all()

    C = 8000
    c5, r5 = si.adjust_class_count(want_c3, C)
    B, V = 256, vocab.V
    d = si.make_decode_inputs(si.config_seed(5), B, V, C, "bf16", sigma=2.0)
    want_bits = oracle.expand_mask(d["cls_bits"], c5, C)
    want_logits = oracle.apply_mask(d["logits"], want_bits, "bf16")
    want_rep = oracle.map_to_rep(d["tok"], c5, r5)

    c_d, r_d, cls_d = dev(c5), dev(r5), dev(d["cls_bits"])
    lg = logits_dev(d["logits"], "bf16")
    tbits = torch.full((B, words_for(V)), -1, dtype=torch.int32, device="cuda")
    lib.cfgzip_apply_mask(lg, cls_d, class_of_token=c_d, C=C, tok_bits_out=tbits)
    rep = lib.cfgzip_map_to_rep(dev(d["tok"]), c_d, r_d)
    torch.cuda.synchronize()
    assert (tbits.cpu().numpy() == want_bits).all()
    assert (logits_bits(lg) == want_logits).all()
    assert (rep.cpu().numpy() == want_rep).all()
    # the whole step in one launch (what bench.py times): mask and map together
    lg1 = logits_dev(d["logits"], "bf16")
    tbits1 = torch.full((B, words_for(V)), -1, dtype=torch.int32, device="cuda")
    rep1 = lib.cfgzip_decode_step(lg1, cls_d, c_d, C, dev(d["tok"]), r_d, tok_bits_out=tbits1)
    torch.cuda.synchronize()
    assert (tbits1.cpu().numpy() == want_bits).all()
    assert (logits_bits(lg1) == want_logits).all()
    assert (rep1.cpu().numpy() == want_rep).all()
    # the unfused pair gives the same result
    lg2 = logits_dev(d["logits"], "bf16")
    tb2 = lib.cfgzip_expand_mask(cls_d, C, c_d)
    lib.cfgzip_apply_mask(lg2, tb2)
    assert (tb2.cpu().numpy() == want_bits).all()
    assert (logits_bits(lg2) == want_logits).all()
