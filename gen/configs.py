"""The five seeded workloads: vocabulary + grammar text + a sentence sampler each.

Index (1-based)  workload
  1  tiny JSON object, V = 2,048
  2  nested JSON schema, V = 32,000
  3  TagDispatch tool calling, 64 tools, V = 128,256
  4  cross-grammar reuse: 256 request grammars over a pool of 512 tools, V = 151,936
  5  runtime stress with bounded repetition, V = 151,936, batch 1024
"""
from __future__ import annotations

import random
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Tuple

from .grammars import (BASIC_RULES, Schema, _ident, _lit, nested_schema, random_value, render_value,
                       repetition_stress_ebnf, schema_to_ebnf, sub_object_type, tiny_json_schema, tool_schema)
from .vocab import Vocab, make_vocab

BASE_SEED = 260104426 * 10
CONFIG_NAMES = {1: "tiny_json", 2: "nested_schema", 3: "tagdispatch_tools", 4: "cross_grammar", 5: "repetition_stress"}
VOCAB_SIZES = {1: 2048, 2: 32000, 3: 128256, 4: 151936, 5: 151936}


@dataclass
class Config:
    index: int
    name: str
    vocab: Vocab
    grammars: List[Tuple[str, str]]                 # (ebnf text, root rule)
    batch: int
    steps: int
    sample_text: Callable[[random.Random, int], bytes]   # (rng, grammar index) -> one full sentence
    notes: dict = field(default_factory=dict)


_FREE = "".join(chr(c) for c in range(0x20, 0x7F) if chr(c) != "<") + "\n"


def _free_text(rng: random.Random, lo=0, hi=40) -> str:
    return "".join(rng.choice(_FREE) for _ in range(rng.randint(lo, hi)))


def _tool_names(rng: random.Random, n: int) -> List[str]:
    names: List[str] = []
    while len(names) < n:
        nm = _ident(rng, 4, 12)
        if nm not in names:
            names.append(nm)
    return names


def _dispatch_grammar(tools: List[Tuple[str, Schema, str]]) -> str:
    """tools: (tool name, argument schema, tool rule name).  Rules of shared sub-schemas are
    emitted once."""
    lines: List[str] = []
    pairs = ", ".join(f'({_lit("<function=" + nm + ">")}, {rule})' for nm, _, rule in tools)
    lines.append(f"root ::= TagDispatch({pairs})")
    seen_rules = set()
    body: List[str] = []
    for nm, sch, rule in tools:
        lines.append(f'{rule} ::= {sch.rule} "</function>"')
        txt = schema_to_ebnf(sch, root_rule="__unused__", with_basic=False)
        for ln in txt.splitlines()[1:]:
            head = ln.split(" ::= ", 1)[0]
            if head not in seen_rules:
                seen_rules.add(head)
                body.append(ln)
    return "\n".join(lines + body) + "\n" + BASIC_RULES


def _dispatch_sampler(tools_per_grammar: List[List[Tuple[str, Schema, str]]]):
    def sample(rng: random.Random, g: int) -> bytes:
        tools = tools_per_grammar[g]
        out = _free_text(rng, 0, 30)
        for _ in range(rng.randint(1, 3)):
            nm, sch, _ = rng.choice(tools)
            out += "<function=" + nm + ">" + render_value(random_value(sch, rng), rng) + "</function>"
            out += _free_text(rng, 0, 30)
        return out.encode("utf-8")
    return sample


def _stress_sentence(rng: random.Random, max_objects: int) -> bytes:
    from .grammars import _STR_ALPHA, _ws
    n = rng.randint(1, min(max_objects, 24))
    objs = []
    for _ in range(n):
        s = "".join(chr(rng.randrange(0x80, 0x800)) if rng.random() < 0.05 else rng.choice(_STR_ALPHA)
                    for _ in range(rng.randint(0, 64)))
        d = ("-" if rng.random() < 0.3 else "") + "".join(rng.choice("0123456789") for _ in range(rng.randint(1, 19)))
        objs.append("{" + _ws(rng) + '"s"' + _ws(rng) + ":" + _ws(rng) + '"' + s + '"' + _ws(rng) + "," + _ws(rng)
                    + '"n"' + _ws(rng) + ":" + _ws(rng) + d + _ws(rng) + "}")
    body = objs[0]
    for o in objs[1:]:
        body += _ws(rng) + "," + _ws(rng) + o
    return ("[" + _ws(rng) + body + _ws(rng) + "]").encode("utf-8")


def build_config(index: int, vocab_size: Optional[int] = None, n_grammars: Optional[int] = None,
                 n_tools: Optional[int] = None, max_objects: int = 1000) -> Config:
    """Config `index` (1..5).  The optional arguments shrink a workload for CPU-sized tests
    without changing its recipe."""
    seed = BASE_SEED + index
    rng = random.Random(seed)
    V = vocab_size or VOCAB_SIZES[index]
    vocab = make_vocab(V, seed ^ 0x5EED, "tiny" if index == 1 else "bpe")
    if index == 1:
        sch = tiny_json_schema()
        ebnf = schema_to_ebnf(sch)
        return Config(1, CONFIG_NAMES[1], vocab, [(ebnf, "root")], 4, 64,
                      lambda r, g: render_value(random_value(sch, r, ascii_only=True), r).encode("utf-8"))
    if index == 2:
        sch = nested_schema(rng, 20, 3)
        ebnf = schema_to_ebnf(sch)
        return Config(2, CONFIG_NAMES[2], vocab, [(ebnf, "root")], 64, 256,
                      lambda r, g: render_value(random_value(sch, r), r).encode("utf-8"))
    if index == 3:
        nt = n_tools or 64
        names = _tool_names(rng, nt)
        tools = [(nm, tool_schema(rng, f"t{i}_"), f"tool{i}") for i, nm in enumerate(names)]
        ebnf = _dispatch_grammar(tools)
        return Config(3, CONFIG_NAMES[3], vocab, [(ebnf, "root")], 256, 512, _dispatch_sampler([tools]),
                      notes={"n_tools": nt})
    if index == 4:
        n_pool = n_tools or 512
        n_req = n_grammars or 256
        subs = [sub_object_type(rng, i) for i in range(64)]
        names = _tool_names(rng, n_pool)
        pool = [(nm, tool_schema(rng, f"t{i}_", subs), f"tool{i}") for i, nm in enumerate(names)]
        per_req = []
        for _ in range(n_req):
            k = rng.randint(8, min(32, n_pool))
            per_req.append(rng.sample(pool, k))
        grammars = [(_dispatch_grammar(ts), "root") for ts in per_req]
        return Config(4, CONFIG_NAMES[4], vocab, grammars, 0, 0, _dispatch_sampler(per_req),
                      notes={"n_pool": n_pool, "n_requests": n_req})
    if index == 5:
        ebnf = repetition_stress_ebnf(max_objects)
        return Config(5, CONFIG_NAMES[5], vocab, [(ebnf, "root")], 1024, 200,
                      lambda r, g: _stress_sentence(r, max_objects), notes={"max_objects": max_objects})
    raise ValueError(index)
