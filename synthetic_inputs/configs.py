"""The five seeded workload configurations and the decode-step inputs.

Config index i (1-based) uses seed ``0xCF6 * 1000 + i``.  Configs 1-4 are class
build workloads (vocabulary + automaton); config 5 is the per-step decode
workload (class bitmasks, bf16 logits, sampled ids) over a class map that the
caller supplies (it comes from a config-3-style class build, resized to exactly
8,000 classes by ``adjust_class_count``).
"""

from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from .dfa import make_json_like_dfa, make_lexer_dfa
from .vocab import make_vocab_mixture, make_vocab_uniform

CONFIG_SEED_BASE = 0xCF6 * 1000

# (V, length cap, S, utf8 fraction)
_BUILD_SHAPES = {
    2: (32_000, 16, 256, 0.0),
    3: (128_256, 32, 1024, 0.10),
    4: (151_936, 64, 4096, 0.10),
}


def config_seed(index: int) -> int:
    return CONFIG_SEED_BASE + index


def make_config(index: int, V: Optional[int] = None) -> Dict:
    """Vocabulary and automaton of build config 1-4 (config 5 reuses config 3's).
    `V` overrides the vocabulary size (tests use it for reduced cases)."""
    if index == 5:
        index = 3
    seed = config_seed(index)
    if index == 1:
        vocab = make_vocab_uniform(seed, V=V or 4096, max_len=8)
        table = make_json_like_dfa(seed + 500)
        keywords = []
    else:
        Vd, cap, S, utf8 = _BUILD_SHAPES[index]
        table, keywords = make_lexer_dfa(seed + 500, S)
        vocab = make_vocab_mixture(seed, V or Vd, cap, utf8_fraction=utf8, keywords=keywords)
    return {"index": index, "seed": seed, "vocab": vocab, "table": table,
            "S": int(table.shape[0]), "keywords": keywords}


def words_for(n_bits: int) -> int:
    return (n_bits + 31) // 32


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of float32 values to bfloat16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = u + 0x7FFF + ((u >> 16) & 1)
    return (rounded >> 16).astype(np.uint16)


def make_decode_inputs(seed: int, B: int, V: int, C: int, dtype: str,
                       p_allowed: float = 0.5, sigma: float = 1.0,
                       shared_logits_row: bool = False) -> Dict:
    """Inputs of one decode step.

    cls_bits : int32 [B, W(C)]  bit (k & 31) of word (k >> 5) = 1 iff class k allowed,
               Bernoulli(p_allowed); the pad bits of the last word are random too
               (consumers must ignore them).
    logits   : fp32 values (dtype 'f32') or bf16 bit patterns as uint16 (dtype 'bf16'),
               N(0, sigma^2), shape [B, V]; with shared_logits_row every row is a copy
               of one drawn row (the tiny configuration applies 64 masks to one row).
    tok      : int32 [B] sampled token ids, uniform on [0, V).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    Wc = words_for(C)
    bits = rng.random((B, Wc * 32)) < p_allowed
    cls_bits = np.packbits(bits, axis=1, bitorder="little").view(np.uint32).astype(np.uint32)
    cls_bits = cls_bits.reshape(B, Wc).view(np.int32)
    rows = 1 if shared_logits_row else B
    x = (rng.standard_normal((rows, V), dtype=np.float32) * np.float32(sigma))
    if shared_logits_row:
        x = np.repeat(x, B, axis=0)
    if dtype == "f32":
        logits = np.ascontiguousarray(x)
    elif dtype == "bf16":
        logits = f32_to_bf16_bits(x).reshape(B, V)
    else:
        raise ValueError(dtype)
    tok = rng.integers(0, V, size=B, dtype=np.int64).astype(np.int32)
    return {"cls_bits": np.ascontiguousarray(cls_bits), "logits": logits, "tok": tok,
            "B": B, "V": V, "C": C, "dtype": dtype}


def adjust_class_count(class_of_token: np.ndarray, target_C: int):
    """Resize a class map to exactly `target_C` classes, deterministically.

    Too few classes: repeatedly split the currently largest class (ties: lowest
    id) into its first and second half by member order.  Too many: repeatedly
    merge the two smallest classes (ties: highest ids).  The result is
    renumbered by first appearance and the representative of a class is its
    smallest member.  This only prepares a measurement input; it is not part
    of the method.  Returns (class_of_token int32 [V], rep_of_class int32 [C])."""
    c = np.asarray(class_of_token, dtype=np.int64).copy()
    V = c.shape[0]
    assert 1 <= target_C <= V
    members = {}
    order = np.argsort(c, kind="stable")
    bounds = np.flatnonzero(np.diff(c[order])) + 1
    for k, grp in enumerate(np.split(order, bounds)):
        members[k] = grp
    next_id = len(members)
    import heapq
    if len(members) < target_C:
        heap = [(-len(g), k) for k, g in members.items()]
        heapq.heapify(heap)
        while len(members) < target_C:
            neg, k = heapq.heappop(heap)
            g = members.pop(k)
            assert len(g) >= 2
            h = len(g) // 2
            for part in (g[:h], g[h:]):
                members[next_id] = part
                heapq.heappush(heap, (-len(part), next_id))
                next_id += 1
    elif len(members) > target_C:
        heap = [(len(g), -k) for k, g in members.items()]
        heapq.heapify(heap)
        while len(members) > target_C:
            _, nk1 = heapq.heappop(heap)
            _, nk2 = heapq.heappop(heap)
            g = np.sort(np.concatenate([members.pop(-nk1), members.pop(-nk2)]))
            members[next_id] = g
            heapq.heappush(heap, (len(g), -next_id))
            next_id += 1
    groups = sorted(members.values(), key=lambda g: int(g.min()))
    out = np.empty(V, dtype=np.int32)
    rep = np.empty(len(groups), dtype=np.int32)
    for k, g in enumerate(groups):
        out[g] = k
        rep[k] = int(g.min())
    return out, rep
