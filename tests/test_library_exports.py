"""The C-ABI library loads without a GPU and exports every symbol the header
declares; argument validation answers before any device work."""

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cfgzip.h")


@pytest.fixture(scope="module")
def raw():
    from paper_2605_29986_amd import binding, build
    if not os.path.exists(binding.library_path()):
        build.build()
    return ctypes.CDLL(binding.library_path())


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cfgzip_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_five_calls():
    names = _declared_functions()
    for fn in ("cfgzip_signatures", "cfgzip_build_classes", "cfgzip_expand_mask",
               "cfgzip_apply_mask", "cfgzip_map_to_rep"):
        assert fn in names


def test_every_declared_symbol_is_exported(raw):
    for fn in _declared_functions():
        assert hasattr(raw, fn), fn


def test_host_only_queries(raw):
    raw.cfgzip_signatures_workspace_bytes.restype = ctypes.c_size_t
    raw.cfgzip_build_classes_workspace_bytes.restype = ctypes.c_size_t
    assert raw.cfgzip_version() >= 100
    s = raw.cfgzip_signatures_workspace_bytes(128256, 1024)
    # transposed table + room for the compressed signatures (up to 256 uint16 per token)
    assert s >= 256 * 1024 * 2 + 128256 * 256 * 2
    b = raw.cfgzip_build_classes_workspace_bytes(128256, 1024)
    # its own tables for the re-walk + sort buffers and per-position arrays
    assert b > 256 * 1024 * 2 + 128256 * (8 + 8 + 4 + 4)
    assert raw.cfgzip_signatures_workspace_bytes(0, 10) == 0
    assert raw.cfgzip_build_classes_workspace_bytes(10, 70000) == 0


def test_widening_rows_queries_and_argument_checks(raw):
    names = _declared_functions()
    for fn in ("cfgzip_state_masks", "cfgzip_class_masks", "cfgzip_advance_states", "cfgzip_stack_adjacency",
               "cfgzip_displacements", "cfgzip_displacements_workspace_bytes", "cfgzip_nfa_signatures"):
        assert fn in names
    q = raw.cfgzip_displacements_workspace_bytes
    q.restype = ctypes.c_size_t
    assert q(0, 4097, 5) == 0 and q(-1, 10, 5) == 0 and q(0, 0, 5) == 0 and q(0, 10, 0) == 0
    small, large = q(0, 27, 480), q(128256, 27, 480)
    assert small >= 256 * 27 * 4 + 257 * 4          # the (terminal, head) index and the byte offsets
    assert large >= small + 128256 * 4              # plus the list of tokens for the second pass
    assert q(0, 4096, 9000) >= 3 * 4096 * 128 * 4 + 256 * 4096 * 4 + 9000 * 16   # three bit matrices and the index
    u64, sz = ctypes.c_uint64(0), ctypes.c_size_t(0)
    assert raw.cfgzip_displacements(None, None, 1, None, None, None, None, 0, 1, 1, None, 256, None, None, u64,
                                    None, sz, None) == -1
    assert raw.cfgzip_stack_adjacency(None, None, None, None, 0, 1, 1, None, None, None, sz, None) == -1
    assert raw.cfgzip_nfa_signatures(None, None, 1, None, 1, None, None, u64, None) == -1
    # sizes are checked before any pointer is used
    buf = ctypes.create_string_buffer(4096)
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert raw.cfgzip_nfa_signatures(p, p, 1, p, 1025, p, None, u64, None) == -1
    assert raw.cfgzip_displacements(p, p, 1, p, p, p, p, 2, 1, 5000, p, 256, p, None, u64, p, sz, None) == -1
    assert raw.cfgzip_displacements(p, p, 1, p, p, p, p, -1, 1, 5, p, 256, p, None, u64, p, sz, None) == -1
    assert raw.cfgzip_displacements(p, p, 1, p, p, p, None, 2, 1, 5, p, 256, p, None, u64, p, sz, None) == -1
    for bad_row_len in (0, 255, 300, 8192):
        assert raw.cfgzip_displacements(p, p, 1, p, p, p, p, 2, 1, 5, p, bad_row_len, p, None, u64, p, sz,
                                        None) == -1
    assert raw.cfgzip_displacements(p, p, 1, p, p, p, p, 2, 1, 5, p, 256, p, None, u64, None, sz, None) == -2


def test_null_and_range_arguments_are_rejected_without_a_gpu(raw):
    assert raw.cfgzip_expand_mask(None, 1, 1, None, 1, None, None) == -1
    assert raw.cfgzip_apply_mask(None, 0, 1, 1, ctypes.c_int64(1), None, 0, None, 0, None, None) == -1
    assert raw.cfgzip_map_to_rep(None, 1, None, 1, None, 1, None, None) == -1
    assert raw.cfgzip_signatures(None, None, 1, None, 1, None, None, ctypes.c_uint64(0), None,
                                 ctypes.c_size_t(0), None) == -1
    assert raw.cfgzip_build_classes(None, None, 1, None, 1, None, None, None, None, None, None, None,
                                    None, None, ctypes.c_size_t(0), None) == -1


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2605_29986_amd as lib
    with pytest.raises(TypeError):
        lib.cfgzip_map_to_rep(torch.zeros(4, dtype=torch.int32), torch.zeros(4, dtype=torch.int32),
                              torch.zeros(1, dtype=torch.int32))
