"""Seeded synthetic inputs: vocabularies, grammar texts, logits, walk policy.

This module is data only.  It holds none of the method's arithmetic (no
automaton, no parser, no mask computation): it writes grammar *text*, token
*bytes*, logits and random choices.  Both the CPU oracle's tests and the GPU
library's tests/bench read the same inputs from here; neither of those two
imports the other.

All randomness is numpy ``Generator(PCG64(seed))``.
"""

from .vocab import make_vocab, Vocab, ARITH_ALPHABET
from .grammars import (
    ARITH_GRAMMAR,
    JSON_GRAMMAR,
    CSQL_GRAMMAR,
    XML_GRAMMAR,
    PYDSL_GRAMMAR,
    make_schema_grammar,
    random_schema,
)
from .logits import make_logits
from .walks import pick_token, pick_tokens, STRUCTURAL_BYTES

__all__ = [
    "make_vocab",
    "Vocab",
    "ARITH_ALPHABET",
    "ARITH_GRAMMAR",
    "JSON_GRAMMAR",
    "CSQL_GRAMMAR",
    "XML_GRAMMAR",
    "PYDSL_GRAMMAR",
    "make_schema_grammar",
    "random_schema",
    "make_logits",
    "pick_token",
    "pick_tokens",
    "STRUCTURAL_BYTES",
]
