"""ctypes binding of libcfgzip.so.  Argument marshalling only.

Tensors are torch CUDA (ROCm) tensors; they supply device memory and the HIP
stream.  Function names and argument order follow ``include/cfgzip.h``.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "lib", "libcfgzip.so")
_lib: Optional[ctypes.CDLL] = None

DEFAULT_HASH_SEED = 0x5EED_CF62_1234_ABCD

CFGZIP_DTYPE_F32 = 0
CFGZIP_DTYPE_BF16 = 1
CFGZIP_BITS_TOKEN = 0
CFGZIP_BITS_CLASS = 1

_ERRORS = {
    -1: "CFGZIP_E_INVALID (bad argument)",
    -2: "CFGZIP_E_WORKSPACE (workspace missing, misaligned or too small)",
    -3: "CFGZIP_E_HIP (a HIP call failed)",
    -4: "CFGZIP_E_COLLISION (hash collisions not resolved)",
    -5: "CFGZIP_E_TOO_LARGE (beyond what an entry point with built-in scratch memory takes)",
}


class CfgzipError(RuntimeError):
    def __init__(self, fn: str, code: int, hip_error: int = 0):
        self.code = code
        self.hip_error = hip_error
        extra = f", hipError_t={hip_error}" if code == -3 else ""
        super().__init__(f"{fn} failed: {_ERRORS.get(code, code)}{extra}")


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Loads the built HIP library; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2605_29986_amd.build` "
            "(hipcc, gfx950). The CFGzip path has no CPU fallback.")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u64, sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64,
                             ctypes.c_size_t)
    lib.cfgzip_version.restype = ctypes.c_int
    lib.cfgzip_last_hip_error.restype = ctypes.c_int
    lib.cfgzip_signatures_workspace_bytes.restype = sz
    lib.cfgzip_signatures_workspace_bytes.argtypes = [i32, i32]
    lib.cfgzip_signatures.restype = ctypes.c_int
    lib.cfgzip_signatures.argtypes = [vp, vp, i32, vp, i32, vp, vp, u64, vp, sz, vp]
    lib.cfgzip_signatures_composed_workspace_bytes.restype = sz
    lib.cfgzip_signatures_composed_workspace_bytes.argtypes = [i32, i32]
    lib.cfgzip_signatures_composed.restype = ctypes.c_int
    lib.cfgzip_signatures_composed.argtypes = [vp, vp, i32, vp, i32, vp, vp, u64, vp, sz, vp]
    lib.cfgzip_signatures_static.restype = ctypes.c_int
    lib.cfgzip_signatures_static.argtypes = [vp, vp, i32, vp, i32, vp, vp, u64, vp]
    lib.cfgzip_build_classes_workspace_bytes.restype = sz
    lib.cfgzip_build_classes_workspace_bytes.argtypes = [i32, i32]
    lib.cfgzip_build_classes.restype = ctypes.c_int
    lib.cfgzip_build_classes.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cfgzip_expand_mask.restype = ctypes.c_int
    lib.cfgzip_expand_mask.argtypes = [vp, i32, i32, vp, i32, vp, vp]
    lib.cfgzip_apply_mask.restype = ctypes.c_int
    lib.cfgzip_apply_mask.argtypes = [vp, i32, i32, i32, i64, vp, i32, vp, i32, vp, vp]
    lib.cfgzip_map_to_rep.restype = ctypes.c_int
    lib.cfgzip_map_to_rep.argtypes = [vp, i32, vp, i32, vp, i32, vp, vp]
    lib.cfgzip_decode_step.restype = ctypes.c_int
    lib.cfgzip_decode_step.argtypes = [vp, i32, i32, i32, i64, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.cfgzip_state_masks.restype = ctypes.c_int
    lib.cfgzip_state_masks.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.cfgzip_class_masks.restype = ctypes.c_int
    lib.cfgzip_class_masks.argtypes = [vp, i32, i32, vp, i32, vp, vp]
    lib.cfgzip_advance_states.restype = ctypes.c_int
    lib.cfgzip_advance_states.argtypes = [vp, i32, i32, vp, i32, vp, i32, vp, vp]
    lib.cfgzip_engine_step.restype = ctypes.c_int
    lib.cfgzip_engine_step.argtypes = [vp, i32, i32, i32, i64, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.cfgzip_representative_vocabulary.restype = ctypes.c_int
    lib.cfgzip_representative_vocabulary.argtypes = [vp, vp, i32, vp, i32, vp, vp, i64, vp]
    lib.cfgzip_nfa_signatures.restype = ctypes.c_int
    lib.cfgzip_nfa_signatures.argtypes = [vp, vp, i32, vp, i32, vp, vp, u64, vp]
    lib.cfgzip_nfa_state_masks.restype = ctypes.c_int
    lib.cfgzip_nfa_state_masks.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.cfgzip_nfa_class_masks.restype = ctypes.c_int
    lib.cfgzip_nfa_class_masks.argtypes = [vp, i32, i32, vp, i32, vp, vp]
    lib.cfgzip_nfa_advance_states.restype = ctypes.c_int
    lib.cfgzip_nfa_advance_states.argtypes = [vp, i32, i32, vp, i32, vp, i32, vp, vp]
    lib.cfgzip_displacements_workspace_bytes.restype = sz
    lib.cfgzip_displacements_workspace_bytes.argtypes = [i32, i32, i32]
    lib.cfgzip_stack_adjacency.restype = ctypes.c_int
    lib.cfgzip_stack_adjacency.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.cfgzip_displacements.restype = ctypes.c_int
    lib.cfgzip_displacements.argtypes = [vp, vp, i32, vp, vp, vp, vp, i32, i32, i32, vp, i32, vp, vp, u64,
                                         vp, sz, vp]
    _lib = lib
    return lib


def cfgzip_version() -> int:
    return int(load_library().cfgzip_version())


def words_for(n: int) -> int:
    return (int(n) + 31) // 32


def _check(fn: str, rc: int) -> None:
    if rc != 0:
        raise CfgzipError(fn, rc, int(load_library().cfgzip_last_hip_error()))


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a tensor in GPU memory")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _workspace(nbytes: int, device) -> torch.Tensor:
    # torch's caching allocator hands out 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def cfgzip_signatures(tok_bytes: torch.Tensor, tok_off: torch.Tensor, table: torch.Tensor, *,
                      want_sig: bool = True, want_hash: bool = True,
                      hash_seed: int = DEFAULT_HASH_SEED, sig_out: Optional[torch.Tensor] = None,
                      hash_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                      stream=None, composed: bool = False) -> Tuple[Optional[torch.Tensor], Optional[torch.Tensor]]:
    """sig[t][q] = state reached from q on bytes(t) (uint16 [V, S]) and/or its 64-bit hash
    (int64 tensor holding the uint64 bit patterns, [V]).  composed=True calls
    cfgzip_signatures_composed (same results; longer tokens continue the walk of a short token
    that is a prefix of theirs); its workspace is larger."""
    lib = load_library()
    entry = lib.cfgzip_signatures_composed if composed else lib.cfgzip_signatures
    query = lib.cfgzip_signatures_composed_workspace_bytes if composed else lib.cfgzip_signatures_workspace_bytes
    V = tok_off.numel() - 1
    S = table.shape[0]
    dev = tok_off.device
    if want_sig and sig_out is None:
        sig_out = torch.empty((V, S), dtype=torch.uint16, device=dev)
    if want_hash and hash_out is None:
        hash_out = torch.empty((V,), dtype=torch.int64, device=dev)
    need = query(V, S)
    if workspace is None:
        workspace = _workspace(need, dev)
    rc = entry(
        _dev(tok_bytes, torch.uint8, "tok_bytes") if tok_bytes.numel() else None,
        _dev(tok_off, torch.int64, "tok_off"), V,
        _dev(table, torch.uint16, "table"), S,
        _dev(sig_out, torch.uint16, "sig_out") if sig_out is not None else None,
        _dev(hash_out, torch.int64, "hash_out") if hash_out is not None else None,
        ctypes.c_uint64(hash_seed & 0xFFFFFFFFFFFFFFFF),
        workspace.data_ptr(), workspace.numel(), _stream(stream))
    _check("cfgzip_signatures_composed" if composed else "cfgzip_signatures", rc)
    return sig_out, hash_out


STATIC_MAX_STATES = 4096


def cfgzip_signatures_static(tok_bytes: torch.Tensor, tok_off: torch.Tensor, table: torch.Tensor,
                             sig_out: Optional[torch.Tensor], hash_out: Optional[torch.Tensor], *,
                             hash_seed: int = DEFAULT_HASH_SEED, stream=None) -> None:
    """cfgzip_signatures into caller-provided outputs, with the tables in memory that belongs to
    the library: nothing is allocated (at most STATIC_MAX_STATES states)."""
    lib = load_library()
    V = tok_off.numel() - 1
    S = table.shape[0]
    rc = lib.cfgzip_signatures_static(
        _dev(tok_bytes, torch.uint8, "tok_bytes") if tok_bytes.numel() else None,
        _dev(tok_off, torch.int64, "tok_off"), V,
        _dev(table, torch.uint16, "table"), S,
        _dev(sig_out, torch.uint16, "sig_out") if sig_out is not None else None,
        _dev(hash_out, torch.int64, "hash_out") if hash_out is not None else None,
        ctypes.c_uint64(hash_seed & 0xFFFFFFFFFFFFFFFF), _stream(stream))
    _check("cfgzip_signatures_static", rc)


def cfgzip_build_classes(tok_bytes: torch.Tensor, tok_off: torch.Tensor,
                         table: Optional[torch.Tensor],
                         sig: Optional[torch.Tensor], hash: torch.Tensor, *,
                         class_of_token: Optional[torch.Tensor] = None,
                         rep_of_class: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None,
                         signatures_workspace: Optional[torch.Tensor] = None, stream=None):
    """Returns (class_of_token int32 [V], rep_of_class int32 [C] (a view of the first C
    entries), C, collisions).  `signatures_workspace` is the untouched workspace tensor of the
    cfgzip_signatures call that produced `hash` (its compressed signatures are compared
    instead of `sig` rows or a second walk).  With table=None the rows of `sig` (any row
    length) are grouped as they are."""
    lib = load_library()
    V = tok_off.numel() - 1
    S = table.shape[0] if table is not None else (sig.shape[1] if sig is not None else 0)
    dev = tok_off.device
    if class_of_token is None:
        class_of_token = torch.empty((V,), dtype=torch.int32, device=dev)
    if rep_of_class is None:
        rep_of_class = torch.empty((V,), dtype=torch.int32, device=dev)
    need = lib.cfgzip_build_classes_workspace_bytes(V, S)
    if workspace is None:
        workspace = _workspace(need, dev)
    c_host = ctypes.c_int32(0)
    coll_host = ctypes.c_int32(0)
    rc = lib.cfgzip_build_classes(
        _dev(tok_bytes, torch.uint8, "tok_bytes") if tok_bytes.numel() else None,
        _dev(tok_off, torch.int64, "tok_off"), V,
        _dev(table, torch.uint16, "table") if table is not None else None, S,
        _dev(sig, torch.uint16, "sig") if sig is not None else None,
        _dev(hash, torch.int64, "hash"),
        _dev(signatures_workspace, torch.uint8, "signatures_workspace")
        if signatures_workspace is not None else None,
        _dev(class_of_token, torch.int32, "class_of_token"),
        _dev(rep_of_class, torch.int32, "rep_of_class"),
        None, ctypes.addressof(c_host), ctypes.addressof(coll_host),
        workspace.data_ptr(), workspace.numel(), _stream(stream))
    _check("cfgzip_build_classes", rc)
    C = int(c_host.value)
    return class_of_token, rep_of_class[:C], C, int(coll_host.value)


def cfgzip_expand_mask(cls_bits: torch.Tensor, C: int, class_of_token: torch.Tensor, *,
                       tok_bits: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """tok_bits[b] bit i = cls_bits[b] bit class_of_token[i]; int32 [B, W(V)]."""
    lib = load_library()
    B = cls_bits.shape[0]
    V = class_of_token.numel()
    if cls_bits.shape[1] != words_for(C):
        raise ValueError("cls_bits must be [B, ceil(C/32)]")
    if tok_bits is None:
        tok_bits = torch.empty((B, words_for(V)), dtype=torch.int32, device=cls_bits.device)
    rc = lib.cfgzip_expand_mask(_dev(cls_bits, torch.int32, "cls_bits"), B, int(C),
                                _dev(class_of_token, torch.int32, "class_of_token"), V,
                                _dev(tok_bits, torch.int32, "tok_bits"), _stream(stream))
    _check("cfgzip_expand_mask", rc)
    return tok_bits


def cfgzip_apply_mask(logits: torch.Tensor, bits: torch.Tensor, *, V: Optional[int] = None,
                      class_of_token: Optional[torch.Tensor] = None, C: int = 0,
                      tok_bits_out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Masks `logits` ([B, row_stride >= V], float32 or bfloat16) in place.  With
    `class_of_token` given, `bits` is a class-level mask [B, W(C)] gathered through it
    (fused expand + apply, optionally also writing the token-level mask); otherwise
    `bits` is a token-level mask [B, W(V)]."""
    lib = load_library()
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [B, V] with unit column stride")
    B = logits.shape[0]
    V = logits.shape[1] if V is None else int(V)
    if logits.dtype == torch.float32:
        dt = CFGZIP_DTYPE_F32
    elif logits.dtype == torch.bfloat16:
        dt = CFGZIP_DTYPE_BF16
    else:
        raise TypeError("logits must be float32 or bfloat16")
    if not logits.is_cuda:
        raise TypeError("logits must be a tensor in GPU memory")
    kind = CFGZIP_BITS_CLASS if class_of_token is not None else CFGZIP_BITS_TOKEN
    want_words = words_for(C) if kind == CFGZIP_BITS_CLASS else words_for(V)
    if bits.shape[0] != B or bits.shape[1] != want_words:
        raise ValueError("bits has the wrong shape for this mask kind")
    rc = lib.cfgzip_apply_mask(
        logits.data_ptr(), dt, B, V, int(logits.stride(0)),
        _dev(bits, torch.int32, "bits"), kind,
        _dev(class_of_token, torch.int32, "class_of_token") if class_of_token is not None else None,
        int(C),
        _dev(tok_bits_out, torch.int32, "tok_bits_out") if tok_bits_out is not None else None,
        _stream(stream))
    _check("cfgzip_apply_mask", rc)
    return logits


def cfgzip_map_to_rep(tok: torch.Tensor, class_of_token: torch.Tensor, rep_of_class: torch.Tensor,
                      *, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """out[b] = rep_of_class[class_of_token[tok[b]]] (-1 for an id out of range)."""
    lib = load_library()
    B = tok.numel()
    if out is None:
        out = torch.empty((B,), dtype=torch.int32, device=tok.device)
    rc = lib.cfgzip_map_to_rep(_dev(tok, torch.int32, "tok"), B,
                               _dev(class_of_token, torch.int32, "class_of_token"),
                               class_of_token.numel(),
                               _dev(rep_of_class, torch.int32, "rep_of_class"),
                               rep_of_class.numel(), _dev(out, torch.int32, "out"), _stream(stream))
    _check("cfgzip_map_to_rep", rc)
    return out


def cfgzip_decode_step(logits: torch.Tensor, cls_bits: torch.Tensor, class_of_token: torch.Tensor,
                       C: int, tok: torch.Tensor, rep_of_class: torch.Tensor, *,
                       tok_bits_out: Optional[torch.Tensor] = None,
                       rep_out: Optional[torch.Tensor] = None, V: Optional[int] = None,
                       stream=None) -> torch.Tensor:
    """Fused expand + apply on `logits` (in place) and the map of `tok` to representatives, in
    one launch.  Returns rep_out (int32 [B])."""
    lib = load_library()
    if logits.dim() != 2 or logits.stride(1) != 1 or not logits.is_cuda:
        raise ValueError("logits must be a 2-D GPU tensor with unit column stride")
    if logits.dtype == torch.float32:
        dt = CFGZIP_DTYPE_F32
    elif logits.dtype == torch.bfloat16:
        dt = CFGZIP_DTYPE_BF16
    else:
        raise TypeError("logits must be float32 or bfloat16")
    B = logits.shape[0]
    V = logits.shape[1] if V is None else int(V)
    if cls_bits.shape[0] != B or cls_bits.shape[1] != words_for(C) or tok.numel() != B:
        raise ValueError("cls_bits must be [B, ceil(C/32)] and tok [B]")
    if rep_of_class.numel() != C or class_of_token.numel() != V:
        raise ValueError("class_of_token must be [V] and rep_of_class [C]")
    if rep_out is None:
        rep_out = torch.empty((B,), dtype=torch.int32, device=tok.device)
    rc = lib.cfgzip_decode_step(
        logits.data_ptr(), dt, B, V, int(logits.stride(0)), _dev(cls_bits, torch.int32, "cls_bits"),
        _dev(class_of_token, torch.int32, "class_of_token"), int(C),
        _dev(tok_bits_out, torch.int32, "tok_bits_out") if tok_bits_out is not None else None,
        _dev(tok, torch.int32, "tok"), _dev(rep_of_class, torch.int32, "rep_of_class"),
        _dev(rep_out, torch.int32, "rep_out"), _stream(stream))
    _check("cfgzip_decode_step", rc)
    return rep_out


def cfgzip_state_masks(sig_rep: torch.Tensor, live: torch.Tensor, *,
                       state_mask: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """state_mask[q] bit k = live[sig_rep[k][q]]; int32 [S, W(C)] from uint16 [C, S] and uint8 [S]."""
    lib = load_library()
    C, S = sig_rep.shape
    if live.numel() != S:
        raise ValueError("live must have one entry per automaton state")
    if state_mask is None:
        state_mask = torch.empty((S, words_for(C)), dtype=torch.int32, device=sig_rep.device)
    rc = lib.cfgzip_state_masks(_dev(sig_rep, torch.uint16, "sig_rep"), C, S,
                                _dev(live, torch.uint8, "live"),
                                _dev(state_mask, torch.int32, "state_mask"), _stream(stream))
    _check("cfgzip_state_masks", rc)
    return state_mask


def cfgzip_class_masks(state_mask: torch.Tensor, C: int, states: torch.Tensor, *,
                       cls_bits: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """cls_bits[b] = state_mask[states[b]]; int32 [B, W(C)]."""
    lib = load_library()
    S = state_mask.shape[0]
    B = states.numel()
    if state_mask.shape[1] != words_for(C):
        raise ValueError("state_mask must be [S, ceil(C/32)]")
    if cls_bits is None:
        cls_bits = torch.empty((B, words_for(C)), dtype=torch.int32, device=states.device)
    rc = lib.cfgzip_class_masks(_dev(state_mask, torch.int32, "state_mask"), S, int(C),
                                _dev(states, torch.int32, "states"), B,
                                _dev(cls_bits, torch.int32, "cls_bits"), _stream(stream))
    _check("cfgzip_class_masks", rc)
    return cls_bits


def cfgzip_advance_states(sig_rep: torch.Tensor, class_of_token: torch.Tensor, tok: torch.Tensor,
                          states: torch.Tensor, *, stream=None) -> torch.Tensor:
    """states[b] <- sig_rep[class_of_token[tok[b]]][states[b]], in place (-1 when out of range)."""
    lib = load_library()
    C, S = sig_rep.shape
    rc = lib.cfgzip_advance_states(_dev(sig_rep, torch.uint16, "sig_rep"), C, S,
                                   _dev(class_of_token, torch.int32, "class_of_token"),
                                   class_of_token.numel(), _dev(tok, torch.int32, "tok"),
                                   tok.numel(), _dev(states, torch.int32, "states"), _stream(stream))
    _check("cfgzip_advance_states", rc)
    return states


DISP_ROW = 256
DISP_OK, DISP_OVERFLOW, DISP_BAD_GRAMMAR = 0, 1, 2


def _grammar_args(prod_head, prod_byte, prod_body_off, prod_body):
    """Device pointers of a grammar given as flat arrays: heads uint16 [P], terminals uint8 [P],
    body offsets int32 [P + 1], body symbols uint16 [>= body_off[P]] (the count of body symbols
    is the caller's `prod_body.numel()` unless `prod_body` carries padding: see body_total)."""
    P = prod_head.numel()
    if prod_body_off.numel() != P + 1:
        raise ValueError("prod_body_off must have P + 1 entries")
    return (_dev(prod_head, torch.uint16, "prod_head"), _dev(prod_byte, torch.uint8, "prod_byte"),
            _dev(prod_body_off, torch.int32, "prod_body_off"),
            _dev(prod_body, torch.uint16, "prod_body") if prod_body.numel() else None, P)


def cfgzip_stack_adjacency(prod_head: torch.Tensor, prod_byte: torch.Tensor,
                           prod_body_off: torch.Tensor, prod_body: torch.Tensor, N: int, *,
                           body_total: Optional[int] = None,
                           workspace: Optional[torch.Tensor] = None, stream=None):
    """(adj int32 [N, W(N)], invalid int32 [1]): bit Y of row Z <=> (Y, Z) stack-adjacent."""
    lib = load_library()
    dev = prod_head.device
    adj = torch.empty((N, words_for(N)), dtype=torch.int32, device=dev)
    invalid = torch.empty((1,), dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = _workspace(lib.cfgzip_displacements_workspace_bytes(0, N, prod_head.numel()), dev)
    h, b, off, bd, P = _grammar_args(prod_head, prod_byte, prod_body_off, prod_body)
    total = prod_body.numel() if body_total is None else int(body_total)
    rc = lib.cfgzip_stack_adjacency(h, b, off, bd, total, P, N, adj.data_ptr(), invalid.data_ptr(),
                                    workspace.data_ptr(), workspace.numel(), _stream(stream))
    _check("cfgzip_stack_adjacency", rc)
    return adj, invalid


def cfgzip_displacements(tok_bytes: torch.Tensor, tok_off: torch.Tensor, prod_head: torch.Tensor,
                         prod_byte: torch.Tensor, prod_body_off: torch.Tensor, prod_body: torch.Tensor,
                         N: int, *, body_total: Optional[int] = None, row_len: int = DISP_ROW,
                         hash_seed: int = DEFAULT_HASH_SEED,
                         workspace: Optional[torch.Tensor] = None, stream=None):
    """(rows uint16 [V, row_len], hash int64 [V] holding uint64 bit patterns, status int32 [V])."""
    lib = load_library()
    V = tok_off.numel() - 1
    dev = tok_off.device
    rows = torch.empty((V, row_len), dtype=torch.uint16, device=dev)
    hashes = torch.empty((V,), dtype=torch.int64, device=dev)
    status = torch.empty((V,), dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = _workspace(lib.cfgzip_displacements_workspace_bytes(V, N, prod_head.numel()), dev)
    h, b, off, bd, P = _grammar_args(prod_head, prod_byte, prod_body_off, prod_body)
    total = prod_body.numel() if body_total is None else int(body_total)
    rc = lib.cfgzip_displacements(
        _dev(tok_bytes, torch.uint8, "tok_bytes") if tok_bytes.numel() else None,
        _dev(tok_off, torch.int64, "tok_off"), V, h, b, off, bd, total, P, N,
        rows.data_ptr(), row_len, hashes.data_ptr(), status.data_ptr(),
        ctypes.c_uint64(hash_seed & 0xFFFFFFFFFFFFFFFF),
        workspace.data_ptr(), workspace.numel(), _stream(stream))
    _check("cfgzip_displacements", rc)
    return rows, hashes, status


def cfgzip_nfa_signatures(tok_bytes: torch.Tensor, tok_off: torch.Tensor, nfa: torch.Tensor, *,
                          want_hash: bool = True, hash_seed: int = DEFAULT_HASH_SEED, stream=None):
    """(rel int32 [V, S, W(S)], hash int64 [V] or None) for nfa int32 [256, S, W(S)]."""
    lib = load_library()
    V = tok_off.numel() - 1
    S = nfa.shape[1]
    if nfa.shape != (256, S, words_for(S)):
        raise ValueError("nfa must have shape [256, S, W(S)]")
    dev = tok_off.device
    rel = torch.empty((V, S, words_for(S)), dtype=torch.int32, device=dev)
    hashes = torch.empty((V,), dtype=torch.int64, device=dev) if want_hash else None
    rc = lib.cfgzip_nfa_signatures(
        _dev(tok_bytes, torch.uint8, "tok_bytes") if tok_bytes.numel() else None,
        _dev(tok_off, torch.int64, "tok_off"), V, _dev(nfa, torch.int32, "nfa"), S,
        rel.data_ptr(), hashes.data_ptr() if want_hash else None,
        ctypes.c_uint64(hash_seed & 0xFFFFFFFFFFFFFFFF), _stream(stream))
    _check("cfgzip_nfa_signatures", rc)
    return rel, hashes


def cfgzip_nfa_state_masks(rel_rep: torch.Tensor, live: torch.Tensor, *, stream=None) -> torch.Tensor:
    """int32 [S, W(C)] from relations int32 [C, S, W(S)] and live uint8 [S]."""
    lib = load_library()
    C, S, W = rel_rep.shape
    if W != words_for(S) or live.numel() != S:
        raise ValueError("rel_rep must be [C, S, W(S)] and live [S]")
    out = torch.empty((S, words_for(C)), dtype=torch.int32, device=rel_rep.device)
    rc = lib.cfgzip_nfa_state_masks(_dev(rel_rep, torch.int32, "rel_rep"), C, S, _dev(live, torch.uint8, "live"),
                                    out.data_ptr(), _stream(stream))
    _check("cfgzip_nfa_state_masks", rc)
    return out


def cfgzip_nfa_class_masks(state_mask: torch.Tensor, C: int, state_sets: torch.Tensor, *,
                           stream=None) -> torch.Tensor:
    """int32 [B, W(C)]: union of the mask rows of the states in each set (state_sets int32 [B, W(S)])."""
    lib = load_library()
    S = state_mask.shape[0]
    B = state_sets.shape[0]
    if state_sets.shape[1] != words_for(S) or state_mask.shape[1] != words_for(C):
        raise ValueError("state_sets must be [B, W(S)] and state_mask [S, W(C)]")
    out = torch.empty((B, words_for(C)), dtype=torch.int32, device=state_sets.device)
    rc = lib.cfgzip_nfa_class_masks(_dev(state_mask, torch.int32, "state_mask"), S, int(C),
                                    _dev(state_sets, torch.int32, "state_sets"), B, out.data_ptr(),
                                    _stream(stream))
    _check("cfgzip_nfa_class_masks", rc)
    return out


def cfgzip_nfa_advance_states(rel_rep: torch.Tensor, class_of_token: torch.Tensor, tok: torch.Tensor,
                              state_sets: torch.Tensor, *, stream=None) -> torch.Tensor:
    """state_sets (int32 [B, W(S)]) advanced in place on the representatives of tok's classes."""
    lib = load_library()
    C, S, _W = rel_rep.shape
    rc = lib.cfgzip_nfa_advance_states(_dev(rel_rep, torch.int32, "rel_rep"), C, S,
                                       _dev(class_of_token, torch.int32, "class_of_token"),
                                       class_of_token.numel(), _dev(tok, torch.int32, "tok"), tok.numel(),
                                       _dev(state_sets, torch.int32, "state_sets"), _stream(stream))
    _check("cfgzip_nfa_advance_states", rc)
    return state_sets


def cfgzip_representative_vocabulary(tok_bytes: torch.Tensor, tok_off: torch.Tensor,
                                     rep_of_class: torch.Tensor, *, stream=None):
    """(rep_bytes uint8 [capacity], rep_off int64 [C + 1]): the representatives' byte strings in
    class order, CSR like the vocabulary.  rep_off[C] bytes of rep_bytes are meaningful."""
    lib = load_library()
    V = tok_off.numel() - 1
    C = rep_of_class.numel()
    dev = tok_off.device
    capacity = tok_bytes.numel()
    rep_off = torch.empty((C + 1,), dtype=torch.int64, device=dev)
    rep_bytes = torch.empty((max(capacity, 1),), dtype=torch.uint8, device=dev)
    rc = lib.cfgzip_representative_vocabulary(
        _dev(tok_bytes, torch.uint8, "tok_bytes") if capacity else None,
        _dev(tok_off, torch.int64, "tok_off"), V,
        _dev(rep_of_class, torch.int32, "rep_of_class"), C, rep_off.data_ptr(),
        rep_bytes.data_ptr(), capacity, _stream(stream))
    _check("cfgzip_representative_vocabulary", rc)
    return rep_bytes, rep_off


def cfgzip_engine_step(logits: torch.Tensor, state_mask: torch.Tensor, C: int,
                       class_of_token: torch.Tensor, sig_rep: Optional[torch.Tensor],
                       tok_prev: Optional[torch.Tensor], states_in: torch.Tensor, *,
                       states_out: Optional[torch.Tensor] = None,
                       tok_bits_out: Optional[torch.Tensor] = None, V: Optional[int] = None,
                       stream=None) -> torch.Tensor:
    """One decode step of the byte-automaton engine in one launch: advances the states on the
    tokens sampled last (tok_prev, or None at the first step), masks `logits` in place with each
    sequence's class mask, returns the new states (int32 [B], a tensor other than states_in)."""
    lib = load_library()
    if logits.dtype == torch.float32:
        dtype = 0
    elif logits.dtype == torch.bfloat16:
        dtype = 1
    else:
        raise TypeError("logits must be float32 or bfloat16")
    if not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be a 2-D GPU tensor with unit column stride")
    B = logits.shape[0]
    V = int(V) if V is not None else logits.shape[1]
    S = state_mask.shape[0]
    if states_out is None:
        states_out = torch.empty_like(states_in)
    rc = lib.cfgzip_engine_step(
        logits.data_ptr(), dtype, B, V, logits.stride(0), _dev(state_mask, torch.int32, "state_mask"), S, C,
        _dev(class_of_token, torch.int32, "class_of_token"),
        _dev(sig_rep, torch.uint16, "sig_rep") if sig_rep is not None else None,
        _dev(tok_prev, torch.int32, "tok_prev") if tok_prev is not None else None,
        _dev(states_in, torch.int32, "states_in"), _dev(states_out, torch.int32, "states_out"),
        _dev(tok_bits_out, torch.int32, "tok_bits_out") if tok_bits_out is not None else None,
        _stream(stream))
    _check("cfgzip_engine_step", rc)
    return states_out
