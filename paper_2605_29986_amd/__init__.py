"""MI355X-native hot path of CFGzip (token-vocabulary compression for
grammar-constrained decoding): a C-ABI HIP library, ``lib/libcfgzip.so``, and a
thin ctypes binding with the same entry-point names.

The binding only marshals arguments (device pointers of torch tensors, sizes,
the current HIP stream); every step of the path runs in the library's kernels.
There is no CPU fallback: calling anything without the built library raises.
"""

from .binding import (  # noqa: F401
    CfgzipError,
    DISP_BAD_GRAMMAR,
    DISP_OK,
    DISP_OVERFLOW,
    DISP_ROW,
    DEFAULT_HASH_SEED,
    cfgzip_advance_states,
    cfgzip_apply_mask,
    cfgzip_build_classes,
    cfgzip_class_masks,
    cfgzip_decode_step,
    cfgzip_displacements,
    cfgzip_engine_step,
    cfgzip_expand_mask,
    cfgzip_map_to_rep,
    cfgzip_nfa_advance_states,
    cfgzip_nfa_class_masks,
    cfgzip_nfa_signatures,
    cfgzip_nfa_state_masks,
    cfgzip_representative_vocabulary,
    cfgzip_signatures,
    cfgzip_signatures_static,
    cfgzip_stack_adjacency,
    cfgzip_state_masks,
    cfgzip_version,
    library_path,
    load_library,
    words_for,
)
