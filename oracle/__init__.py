"""CPU oracle for the CFGzip hot path.  TEST INFRASTRUCTURE ONLY.

Thin numpy wrappers over ``cfgzip_oracle.c`` (compiled with gcc into
``liboracle.so`` next to it).  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the HIP library and its Python
binding never do, and this package never imports them.

``oracle.displacement`` additionally holds a pure-Python implementation of the
paper's general displacement computation (Algorithm 1 with the stack-adjacency
relation of Appendix C) for tiny grammars; it pins the regular-grammar reading
used by ``signatures``.
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cfgzip_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_build_classes.restype = ctypes.c_int32
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_splitmix64_next.restype = ctypes.c_uint64
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def words_for(n: int) -> int:
    return (int(n) + 31) // 32


def signatures(tok_bytes, tok_off, table) -> np.ndarray:
    """uint16 [V, S]: sig[t][q] = state reached from q on the bytes of token t."""
    tok_bytes = _c(tok_bytes, np.uint8)
    tok_off = _c(tok_off, np.int64)
    table = _c(table, np.uint16)
    V = tok_off.shape[0] - 1
    S = table.shape[0]
    assert table.shape == (S, 256)
    sig = np.empty((V, S), dtype=np.uint16)
    _load().oracle_signatures(_p(tok_bytes), _p(tok_off), ctypes.c_int32(V), _p(table),
                              ctypes.c_int32(S), _p(sig))
    return sig


def build_classes(sig, tok_off) -> Tuple[np.ndarray, np.ndarray]:
    """(class_of_token int32 [V], rep_of_class int32 [C]) by full-signature equality."""
    sig = _c(sig, np.uint16)
    tok_off = _c(tok_off, np.int64)
    V, S = sig.shape
    c = np.empty(V, dtype=np.int32)
    r = np.empty(max(V, 1), dtype=np.int32)
    C = _load().oracle_build_classes(_p(sig), _p(tok_off), ctypes.c_int32(V), ctypes.c_int32(S),
                                     _p(c), _p(r))
    return c, r[:C].copy()


def expand_mask(cls_bits, class_of_token, C: int) -> np.ndarray:
    """int32 [B, W(V)] token-level bit masks from int32 [B, W(C)] class-level ones."""
    cls_bits = _c(cls_bits, np.int32)
    c = _c(class_of_token, np.int32)
    B = cls_bits.shape[0]
    V = c.shape[0]
    assert cls_bits.shape[1] == words_for(C)
    out = np.empty((B, words_for(V)), dtype=np.int32)
    _load().oracle_expand_mask(_p(cls_bits), ctypes.c_int32(B), ctypes.c_int32(C), _p(c),
                               ctypes.c_int32(V), _p(out))
    return out


def apply_mask(logits, tok_bits, dtype: str, V: Optional[int] = None) -> np.ndarray:
    """Returns a masked copy of `logits`.  dtype 'f32': float32 or uint32 array;
    dtype 'bf16': uint16 bit patterns.  Rows may be wider than V (row stride)."""
    tok_bits = _c(tok_bits, np.int32)
    B = tok_bits.shape[0]
    if dtype == "f32":
        out = np.array(logits, copy=True, order="C")
        assert out.dtype in (np.float32, np.uint32) and out.ndim == 2 and out.shape[0] == B
        fn = _load().oracle_apply_mask_f32
    elif dtype == "bf16":
        out = np.array(logits, dtype=np.uint16, copy=True, order="C")
        assert out.ndim == 2 and out.shape[0] == B
        fn = _load().oracle_apply_mask_bf16
    else:
        raise ValueError(dtype)
    stride = out.shape[1]
    V = stride if V is None else V
    assert tok_bits.shape[1] == words_for(V)
    fn(_p(out), ctypes.c_int32(B), ctypes.c_int32(V), ctypes.c_int64(stride), _p(tok_bits))
    return out


def map_to_rep(tok, class_of_token, rep_of_class) -> np.ndarray:
    tok = _c(tok, np.int32)
    c = _c(class_of_token, np.int32)
    r = _c(rep_of_class, np.int32)
    out = np.empty(tok.shape[0], dtype=np.int32)
    _load().oracle_map_to_rep(_p(tok), ctypes.c_int32(tok.shape[0]), _p(c),
                              ctypes.c_int32(c.shape[0]), _p(r), ctypes.c_int32(r.shape[0]),
                              _p(out))
    return out


def live_states(table, accept) -> np.ndarray:
    """uint8 [S]: 1 iff an accepting state is reachable from the state."""
    table = _c(table, np.uint16)
    accept = _c(accept, np.uint8)
    S = table.shape[0]
    assert table.shape == (S, 256) and accept.shape == (S,)
    live = np.empty(S, dtype=np.uint8)
    _load().oracle_live_states(_p(table), ctypes.c_int32(S), _p(accept), _p(live))
    return live


def state_masks(sig_rep, live) -> np.ndarray:
    """int32 [S, W(C)]: bit k of row q = live[sig_rep[k][q]]."""
    sig_rep = _c(sig_rep, np.uint16)
    live = _c(live, np.uint8)
    C, S = sig_rep.shape
    out = np.empty((S, words_for(C)), dtype=np.int32)
    _load().oracle_state_masks(_p(sig_rep), ctypes.c_int32(C), ctypes.c_int32(S), _p(live), _p(out))
    return out


def class_masks(state_mask, C: int, states) -> np.ndarray:
    state_mask = _c(state_mask, np.int32)
    states = _c(states, np.int32)
    S = state_mask.shape[0]
    assert state_mask.shape[1] == words_for(C)
    out = np.empty((states.shape[0], words_for(C)), dtype=np.int32)
    _load().oracle_class_masks(_p(state_mask), ctypes.c_int32(S), ctypes.c_int32(C), _p(states),
                               ctypes.c_int32(states.shape[0]), _p(out))
    return out


def advance_states(sig_rep, class_of_token, tok, states) -> np.ndarray:
    """Returns the new states (int32 [B])."""
    sig_rep = _c(sig_rep, np.uint16)
    c = _c(class_of_token, np.int32)
    tok = _c(tok, np.int32)
    out = np.array(states, dtype=np.int32, copy=True)
    C, S = sig_rep.shape
    _load().oracle_advance_states(_p(sig_rep), ctypes.c_int32(C), ctypes.c_int32(S), _p(c),
                                  ctypes.c_int32(c.shape[0]), _p(tok), ctypes.c_int32(tok.shape[0]),
                                  _p(out))
    return out


def signature_hash(sig, seed: int) -> np.ndarray:
    sig = _c(sig, np.uint16)
    V, S = sig.shape
    out = np.empty(V, dtype=np.uint64)
    _load().oracle_hash(_p(sig), ctypes.c_int32(V), ctypes.c_int32(S), ctypes.c_uint64(seed),
                        _p(out))
    return out


def representative_vocabulary(tok_bytes, tok_off, rep):
    """(rep_bytes uint8 [total], rep_off int64 [C + 1]): the representatives' byte strings."""
    tok_bytes = _c(tok_bytes, np.uint8)
    tok_off = _c(tok_off, np.int64)
    rep = _c(rep, np.int32)
    V, C = tok_off.shape[0] - 1, rep.shape[0]
    rep_off = np.empty(C + 1, dtype=np.int64)
    fn = _load().oracle_representative_vocabulary
    fn.restype = ctypes.c_int64
    total = fn(_p(tok_bytes), _p(tok_off), ctypes.c_int32(V), _p(rep), ctypes.c_int32(C), _p(rep_off), None)
    rep_bytes = np.empty(max(int(total), 1), dtype=np.uint8)
    fn(_p(tok_bytes), _p(tok_off), ctypes.c_int32(V), _p(rep), ctypes.c_int32(C), _p(rep_off), _p(rep_bytes))
    return rep_bytes[:total], rep_off


def nfa_signatures(tok_bytes, tok_off, nfa) -> np.ndarray:
    """uint32 [V, S, W]: bit row of the states reachable from q on the bytes of token t, for a
    non-deterministic byte automaton nfa[b][q] = bit row of successors (uint32 [256, S, W])."""
    tok_bytes = _c(tok_bytes, np.uint8)
    tok_off = _c(tok_off, np.int64)
    nfa = _c(nfa, np.uint32)
    V = tok_off.shape[0] - 1
    S = nfa.shape[1]
    W = (S + 31) // 32
    assert nfa.shape == (256, S, W)
    out = np.empty((V, S, W), dtype=np.uint32)
    _load().oracle_nfa_signatures(_p(tok_bytes), _p(tok_off), ctypes.c_int32(V), _p(nfa),
                                  ctypes.c_int32(S), _p(out))
    return out


def nfa_live_states(nfa, accept) -> np.ndarray:
    """uint8 [S]: 1 iff an accepting state can be reached from the state (nfa uint32 [256, S, W])."""
    nfa = _c(nfa, np.uint32)
    accept = _c(accept, np.uint8)
    S = nfa.shape[1]
    live = np.empty(S, dtype=np.uint8)
    _load().oracle_nfa_live_states(_p(nfa), ctypes.c_int32(S), _p(accept), _p(live))
    return live


def nfa_state_masks(rel_rep, live) -> np.ndarray:
    """int32 [S, W(C)]: bit k of row q = the representative of class k leads from q to a live
    state (rel_rep uint32 [C, S, W(S)])."""
    rel_rep = _c(rel_rep, np.uint32)
    live = _c(live, np.uint8)
    C, S = rel_rep.shape[0], rel_rep.shape[1]
    out = np.empty((S, (C + 31) // 32), dtype=np.int32)
    _load().oracle_nfa_state_masks(_p(rel_rep), ctypes.c_int32(C), ctypes.c_int32(S), _p(live), _p(out))
    return out


def nfa_class_masks(state_mask, C, sets) -> np.ndarray:
    """int32 [B, W(C)]: union of the mask rows of the states in each set (sets uint32 [B, W(S)])."""
    state_mask = _c(state_mask, np.int32)
    sets = _c(sets, np.uint32)
    S, B = state_mask.shape[0], sets.shape[0]
    out = np.empty((B, (C + 31) // 32), dtype=np.int32)
    _load().oracle_nfa_class_masks(_p(state_mask), ctypes.c_int32(S), ctypes.c_int32(C), _p(sets),
                                   ctypes.c_int32(B), _p(out))
    return out


def nfa_advance_states(rel_rep, class_of_token, tok, sets) -> np.ndarray:
    """The state sets after each sequence consumed the representative of its token's class."""
    rel_rep = _c(rel_rep, np.uint32)
    c = _c(class_of_token, np.int32)
    tok = _c(tok, np.int32)
    out = _c(sets, np.uint32).copy()
    C, S = rel_rep.shape[0], rel_rep.shape[1]
    _load().oracle_nfa_advance_states(_p(rel_rep), ctypes.c_int32(C), ctypes.c_int32(S), _p(c),
                                      ctypes.c_int32(c.shape[0]), _p(tok), ctypes.c_int32(tok.shape[0]),
                                      _p(out))
    return out


def splitmix64_stream(seed: int, n: int) -> np.ndarray:
    state = ctypes.c_uint64(seed)
    lib = _load()
    return np.array([lib.oracle_splitmix64_next(ctypes.byref(state)) for _ in range(n)],
                    dtype=np.uint64)
