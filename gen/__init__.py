"""Seeded synthetic inputs: vocabularies, EBNF grammars, token traces, logits.

This package only *draws inputs*.  It contains no recogniser, no automaton
construction, no mask logic: the CPU oracle and the HIP library both consume
what it produces (byte strings, EBNF text, token-id lists) and share nothing
else.
"""
from .vocab import make_vocab, Vocab            # noqa: F401
from .grammars import (                          # noqa: F401
    Schema, schema_to_ebnf, random_value, render_value,
    tiny_json_schema, nested_schema, tool_schema, repetition_stress_ebnf,
)
from .configs import build_config, CONFIG_NAMES, BASE_SEED   # noqa: F401
from .traces import segment, Segmenter, random_depth_traces   # noqa: F401
