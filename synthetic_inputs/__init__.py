"""Seeded synthetic inputs for the CFGzip hot path.

This package only *draws inputs* (token vocabularies, byte-level lexer
automata, class bitmasks, logits, sampled ids).  It contains none of the
method's arithmetic: no byte walk, no grouping, no mask expansion.  Both the
CPU oracle's tests and the HIP path's tests/bench draw their inputs here so
that the two sides see byte-identical data.

Every generator takes an explicit integer seed and uses
``numpy.random.Generator(numpy.random.PCG64(seed))`` only.
"""

from .configs import (  # noqa: F401
    CONFIG_SEED_BASE,
    config_seed,
    make_config,
    make_decode_inputs,
    adjust_class_count,
)
from .vocab import Vocab, make_vocab_uniform, make_vocab_mixture  # noqa: F401
from .dfa import make_json_like_dfa, make_lexer_dfa  # noqa: F401
