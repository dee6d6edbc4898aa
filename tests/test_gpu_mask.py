"""GPU parity, per-step path: cfgzip_expand_mask, cfgzip_apply_mask (token bits,
class bits fused, with and without the token-mask by-product) and
cfgzip_map_to_rep against the CPU oracle, bit for bit (tolerance 0: masking only
copies values or writes -inf)."""

import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from synthetic_inputs.configs import words_for

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lib():
    import paper_2605_29986_amd as p
    p.load_library()
    return p


def _class_map(rng, V, C):
    """A class map with every class used and heavy-tailed sizes (an input, not a result)."""
    c = np.minimum((rng.pareto(0.7, size=V)).astype(np.int64), C - 1).astype(np.int32)
    c[rng.choice(V, size=min(C, V), replace=False)] = np.arange(min(C, V), dtype=np.int32)
    return c


SPECIAL_F32 = np.array([0x7FC00001, 0xFFC12345, 0x80000000, 0x00000000, 0x7F800000, 0xFF800000,
                        0x00000001, 0x807FFFFF, 0x7F7FFFFF, 0xFF7FFFFF], dtype=np.uint32)


def _run_all_variants(lib, B, V, C, dtype, seed, stride=None, p_allowed=0.5):
    from gpu_util import dev, logits_dev, logits_bits
    rng = np.random.default_rng(seed)
    c = _class_map(rng, V, C)
    d = si.make_decode_inputs(seed, B, V, C, dtype, p_allowed=p_allowed, sigma=2.0)
    logits = d["logits"]
    if dtype == "f32":
        logits = logits.view(np.uint32).copy()
        k = min(len(SPECIAL_F32), V)
        logits[:, :k] = SPECIAL_F32[:k]
    else:
        logits = logits.copy()
        k = min(len(SPECIAL_F32), V)
        logits[:, :k] = (SPECIAL_F32[:k] >> 16).astype(np.uint16)
    stride = stride or V
    padded = np.zeros((B, stride), dtype=logits.dtype)
    padded[:, :V] = logits
    padded[:, V:] = 0x1234  # must stay untouched
    cls_bits = d["cls_bits"]

    want_bits = oracle.expand_mask(cls_bits, c, C)
    want_logits = oracle.apply_mask(padded, want_bits, dtype, V=V)

    c_d, cls_d = dev(c), dev(cls_bits)
    # B1 alone
    got_bits = lib.cfgzip_expand_mask(cls_d, C, c_d)
    assert (got_bits.cpu().numpy() == want_bits).all(), "expand_mask"
    # B2 from token bits
    lg = logits_dev(padded, dtype)
    lib.cfgzip_apply_mask(lg, dev(want_bits), V=V)
    assert (logits_bits(lg) == want_logits).all(), "apply_mask(token bits)"
    # fused, no by-product
    lg = logits_dev(padded, dtype)
    lib.cfgzip_apply_mask(lg, cls_d, V=V, class_of_token=c_d, C=C)
    assert (logits_bits(lg) == want_logits).all(), "apply_mask(class bits)"
    # fused, with the token mask as by-product (poisoned first: pad bits must be written as 0)
    lg = logits_dev(padded, dtype)
    tb = torch.full((B, words_for(V)), -1, dtype=torch.int32, device="cuda")
    lib.cfgzip_apply_mask(lg, cls_d, V=V, class_of_token=c_d, C=C, tok_bits_out=tb)
    assert (logits_bits(lg) == want_logits).all(), "apply_mask(class bits + token bits out)"
    assert (tb.cpu().numpy() == want_bits).all(), "token bits by-product"
    # idempotent
    lib.cfgzip_apply_mask(lg, cls_d, V=V, class_of_token=c_d, C=C)
    assert (logits_bits(lg) == want_logits).all(), "second application changes nothing"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,V,C", [
    (1, 1, 1), (1, 7, 3), (3, 31, 31), (2, 32, 5), (5, 33, 33), (4, 77, 10), (17, 2048, 100),
    (16, 2049, 64), (33, 4099, 700), (64, 4096, 2980), (7, 10000, 1), (3, 20000, 20000),
])
def test_mask_shapes(lib, dtype, B, V, C):
    print(f"case dtype={dtype} B={B} V={V} C={C}", flush=True)
    _run_all_variants(lib, B, V, C, dtype, seed=B * 1000 + V)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stride_extra", [1, 3, 8, 24])
def test_mask_row_stride_and_alignment(lib, dtype, stride_extra):
    print(f"case dtype={dtype} stride_extra={stride_extra}", flush=True)
    _run_all_variants(lib, 9, 1000, 77, dtype, seed=5, stride=1000 + stride_extra)


@pytest.mark.parametrize("p", [0.0, 0.01, 0.99, 1.0])
def test_mask_extreme_densities(lib, p):
    print(f"case p={p}", flush=True)
    _run_all_variants(lib, 8, 3000, 257, "bf16", seed=11, p_allowed=p)


def test_mask_unaligned_base_pointers(lib):
    """Views that start 2 / 4 bytes into an allocation take the element-wise path."""
    from gpu_util import dev, logits_bits
    rng = np.random.default_rng(3)
    B, V, C = 4, 515, 40
    c = _class_map(rng, V, C)
    d = si.make_decode_inputs(3, B, V, C, "bf16")
    want_bits = oracle.expand_mask(d["cls_bits"], c, C)
    want = oracle.apply_mask(d["logits"], want_bits, "bf16")
    flat = torch.zeros(B * V + 1, dtype=torch.uint16, device="cuda")
    flat[1:] = dev(d["logits"]).reshape(-1)
    lg = flat[1:].view(torch.bfloat16).reshape(B, V)
    cpad = torch.zeros(V + 1, dtype=torch.int32, device="cuda")
    cpad[1:] = dev(c)
    lib.cfgzip_apply_mask(lg, dev(d["cls_bits"]), class_of_token=cpad[1:], C=C)
    assert (logits_bits(lg) == want).all()


def test_map_to_rep(lib):
    from gpu_util import dev
    rng = np.random.default_rng(9)
    V, C, B = 5000, 300, 257
    c = _class_map(rng, V, C)
    r = rng.integers(0, V, size=C).astype(np.int32)
    tok = rng.integers(0, V, size=B).astype(np.int32)
    tok[:4] = [-1, V, V + 100, -2 ** 31]
    want = oracle.map_to_rep(tok, c, r)
    got = lib.cfgzip_map_to_rep(dev(tok), dev(c), dev(r)).cpu().numpy()
    assert (got == want).all() and list(got[:4]) == [-1, -1, -1, -1]


def test_config1_masks(lib, cfg1):
    """Tiny configuration: 64 class masks over the oracle-built classes, applied to 64
    copies of one fp32 row."""
    from gpu_util import dev, logits_dev, logits_bits
    v, table = cfg1["vocab"], cfg1["table"]
    sig = oracle.signatures(v.tok_bytes, v.tok_off, table)
    c, r = oracle.build_classes(sig, v.tok_off)
    C = len(r)
    d = si.make_decode_inputs(cfg1["seed"] + 900, 64, v.V, C, "f32", sigma=1.0,
                              shared_logits_row=True)
    want_bits = oracle.expand_mask(d["cls_bits"], c, C)
    want = oracle.apply_mask(d["logits"].view(np.uint32), want_bits, "f32")
    tb = lib.cfgzip_expand_mask(dev(d["cls_bits"]), C, dev(c))
    lg = logits_dev(d["logits"], "f32")
    lib.cfgzip_apply_mask(lg, tb)
    assert (tb.cpu().numpy() == want_bits).all()
    assert (logits_bits(lg) == want).all()
    got_rep = lib.cfgzip_map_to_rep(dev(d["tok"]), dev(c), dev(r)).cpu().numpy()
    assert (got_rep == oracle.map_to_rep(d["tok"], c, r)).all()


def test_invalid_arguments_are_rejected(lib):
    from paper_2605_29986_amd import CfgzipError
    c = torch.zeros(64, dtype=torch.int32, device="cuda")
    bits = torch.zeros((2, 1), dtype=torch.int32, device="cuda")
    lg = torch.zeros((2, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(CfgzipError):
        lib.cfgzip_apply_mask(lg, bits, V=128, class_of_token=c, C=7)  # V larger than the row
    raw = lib.load_library()
    assert raw.cfgzip_expand_mask(None, 1, 1, c.data_ptr(), 64, bits.data_ptr(), None) == -1
    assert raw.cfgzip_map_to_rep(c.data_ptr(), 0, c.data_ptr(), 64, c.data_ptr(), 1,
                                 c.data_ptr(), None) == -1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_decode_step_in_one_launch(lib, dtype):
    """cfgzip_decode_step = cfgzip_apply_mask (class bits) + cfgzip_map_to_rep, with and without
    the token mask, odd sizes, token ids out of range, more sequences than a workgroup has
    threads."""
    from gpu_util import dev, logits_dev, logits_bits
    for case, (B, V, C) in enumerate([(1, 1, 1), (3, 77, 5), (300, 2049, 300), (17, 70001, 4099)]):
        print(f"case decode step B={B} V={V} C={C} {dtype}", flush=True)
        rng = np.random.default_rng(900 + case)
        c = _class_map(rng, V, C)
        r = rng.integers(0, V, size=C).astype(np.int32)
        d = si.make_decode_inputs(77 + case, B, V, C, dtype, sigma=2.0)
        tok = d["tok"].copy()
        tok[::5] = [-1, V, V + 7, -2 ** 31, 2 ** 31 - 1][case % 5]
        want_bits = oracle.expand_mask(d["cls_bits"], c, C)
        logits = d["logits"].view(np.uint32) if dtype == "f32" else d["logits"]
        want_logits = oracle.apply_mask(logits, want_bits, dtype)
        want_rep = oracle.map_to_rep(tok, c, r)
        assert (want_rep[::5] == -1).all()
        for with_bits in (True, False):
            lg = logits_dev(logits, dtype)
            tbits = torch.full((B, words_for(V)), -1, dtype=torch.int32, device="cuda") if with_bits else None
            rep = lib.cfgzip_decode_step(lg, dev(d["cls_bits"]), dev(c), C, dev(tok), dev(r),
                                         tok_bits_out=tbits)
            torch.cuda.synchronize()
            assert (logits_bits(lg) == want_logits).all()
            if with_bits:
                assert (tbits.cpu().numpy() == want_bits).all()
            assert (rep.cpu().numpy() == want_rep).all()
