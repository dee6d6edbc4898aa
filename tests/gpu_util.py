"""Helpers for the GPU parity tests: numpy <-> device tensors, bit views."""

import numpy as np
import torch


def dev(a: np.ndarray) -> torch.Tensor:
    """Copies a numpy array to the GPU keeping its bit pattern (uint64 travels as int64,
    uint32 as int32)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def vocab_dev(vocab, table):
    return dev(vocab.tok_bytes), dev(vocab.tok_off), dev(table)


def logits_dev(logits: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 values/uint32 patterns -> float32 tensor; uint16 patterns -> bfloat16 tensor."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(logits).view(np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(logits, dtype=np.uint16)).cuda().view(torch.bfloat16)


def logits_bits(t: torch.Tensor) -> np.ndarray:
    """Raw bit patterns of a float32 / bfloat16 tensor as uint32 / uint16."""
    if t.dtype == torch.float32:
        return t.cpu().numpy().view(np.uint32)
    return t.view(torch.uint16).cpu().numpy()


def hash_np(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)
