"""Seeded JSON-schema-like structures, their EBNF text, and random conforming documents.

The EBNF is produced by a deterministic converter (same schema -> same text), the way
structure front-ends of constrained-decoding engines do it.  Random documents are drawn
from the *schema*, never from the grammar text, so a trace needs no mask to be made.
"""
from __future__ import annotations

import random
from dataclasses import dataclass, field
from typing import Any, Dict, List, Optional, Tuple

WS_CHARS = " \n\t"

BASIC_RULES = r'''ws ::= [ \n\t]*
string ::= "\"" ([^"\\\x00-\x1F] | "\\" (["\\/bfnrt] | "u" [0-9a-fA-F]{4}))* "\""
integer ::= "-"? ("0" | [1-9] [0-9]*)
number ::= "-"? ("0" | [1-9] [0-9]*) ("." [0-9]+)? ([eE] [+\-]? [0-9]+)?
boolean ::= "true" | "false"
'''


@dataclass
class Schema:
    kind: str                                   # string|integer|number|boolean|enum|object|array
    props: List[Tuple[str, "Schema", bool]] = field(default_factory=list)   # (name, schema, required)
    items: Optional["Schema"] = None
    min_items: int = 0
    max_items: Optional[int] = None
    values: List[str] = field(default_factory=list)                          # enum members
    rule: str = ""                              # rule name for object / array / enum


def _ident(rng: random.Random, lo=3, hi=10) -> str:
    return "".join(rng.choice("abcdefghijklmnopqrstuvwxyz_") for _ in range(rng.randint(lo, hi))).strip("_") or "k"


def _lit(s: str) -> str:
    out = []
    for ch in s:
        if ch == '"':
            out.append('\\"')
        elif ch == "\\":
            out.append("\\\\")
        elif ch == "\n":
            out.append("\\n")
        elif ch == "\t":
            out.append("\\t")
        else:
            out.append(ch)
    return '"' + "".join(out) + '"'


class _Namer:
    def __init__(self, prefix: str):
        self.prefix = prefix
        self.n = 0

    def fresh(self, kind: str) -> str:
        self.n += 1
        return f"{self.prefix}{kind}{self.n}"


def _value_ref(s: Schema) -> str:
    return s.rule if s.kind in ("object", "array", "enum") else s.kind


def _emit(s: Schema, out: List[str], done: set) -> None:
    if s.kind == "enum":
        if s.rule not in done:
            done.add(s.rule)
            out.append(f"{s.rule} ::= " + " | ".join(_lit('"' + v + '"') for v in s.values))
    elif s.kind == "array":
        _emit(s.items, out, done)
        if s.rule not in done:
            done.add(s.rule)
            it = _value_ref(s.items)
            lo, hi = s.min_items, s.max_items
            if hi is None:
                more = f'(ws "," ws {it})' + ("*" if lo <= 1 else f"{{{lo - 1},}}")
            else:
                more = f'(ws "," ws {it}){{{max(lo - 1, 0)},{hi - 1}}}'
            body = f"{it} {more}"
            if lo == 0:
                body = f"({body})?"
            out.append(f'{s.rule} ::= "[" ws {body} ws "]"')
    elif s.kind == "object":
        for _, ps, _ in s.props:
            _emit(ps, out, done)
        if s.rule not in done:
            done.add(s.rule)
            parts = []
            for i, (name, ps, req) in enumerate(s.props):
                kv = f'{_lit(chr(34) + name + chr(34))} ws ":" ws {_value_ref(ps)}'
                if i == 0:
                    parts.append(kv)                      # first property is always required
                elif req:
                    parts.append(f'ws "," ws {kv}')
                else:
                    parts.append(f'(ws "," ws {kv})?')
            out.append(f'{s.rule} ::= "{{" ws ' + " ".join(parts) + ' ws "}"')


def schema_to_ebnf(root: Schema, root_rule: str = "root", with_basic: bool = True) -> str:
    """EBNF text whose `root_rule` derives exactly the documents of `root`."""
    out: List[str] = []
    _emit(root, out, set())
    text = f"{root_rule} ::= {_value_ref(root)}\n" + "\n".join(out) + "\n"
    return text + (BASIC_RULES if with_basic else "")


# ---------------------------------------------------------------- random schemas

def _leaf(rng: random.Random, namer: _Namer, kinds=("string", "integer", "number", "boolean", "enum")) -> Schema:
    k = rng.choice(kinds)
    if k == "enum":
        vals = []
        while len(vals) < rng.randint(4, 16):
            v = _ident(rng)
            if v not in vals:
                vals.append(v)
        return Schema("enum", values=vals, rule=namer.fresh("enum"))
    return Schema(k)


def tiny_json_schema() -> Schema:
    """One object with 3 required properties: string, integer, boolean."""
    return Schema("object", rule="obj", props=[
        ("name", Schema("string"), True), ("age", Schema("integer"), True), ("ok", Schema("boolean"), True)])


def nested_schema(rng: random.Random, n_props: int = 20, depth: int = 3, prefix: str = "") -> Schema:
    """`n_props` properties in total spread over objects nested to `depth`, with enums and
    arrays of objects."""
    namer = _Namer(prefix)
    budget = [n_props]

    def obj(d: int) -> Schema:
        o = Schema("object", rule=namer.fresh("obj"))
        want = max(2, budget[0] // max(1, d)) if d > 1 else budget[0]
        n_here = max(1, min(budget[0], rng.randint(2, max(2, want))))
        names = set()
        for i in range(n_here):
            if budget[0] <= 0:
                break
            name = _ident(rng)
            while name in names:
                name = _ident(rng)
            names.add(name)
            budget[0] -= 1
            r = rng.random()
            if d > 1 and budget[0] >= 2 and r < 0.25:
                ps = obj(d - 1)
            elif d > 1 and budget[0] >= 2 and r < 0.40:
                ps = Schema("array", items=obj(d - 1), rule=namer.fresh("arr"), min_items=rng.choice((0, 1)),
                            max_items=rng.choice((None, 4, 8)))
            else:
                ps = _leaf(rng, namer)
            o.props.append((name, ps, i == 0 or rng.random() < 0.7))
        return o

    root = obj(depth)
    # spend what is left on the root so the total is n_props
    names = {n for n, _, _ in root.props}
    while budget[0] > 0:
        name = _ident(rng)
        if name in names:
            continue
        names.add(name)
        budget[0] -= 1
        root.props.append((name, _leaf(rng, namer), rng.random() < 0.7))
    return root


def tool_schema(rng: random.Random, prefix: str, sub_types: Optional[List[Schema]] = None) -> Schema:
    """A tool's argument object: 5-15 parameters, random types, enums, optional fields;
    with `sub_types`, some parameters are objects from that shared library."""
    namer = _Namer(prefix)
    o = Schema("object", rule=namer.fresh("args"))
    names = set()
    for i in range(rng.randint(5, 15)):
        name = _ident(rng)
        while name in names:
            name = _ident(rng)
        names.add(name)
        if sub_types and rng.random() < 0.4:
            ps = rng.choice(sub_types)
        else:
            ps = _leaf(rng, namer)
        o.props.append((name, ps, i == 0 or rng.random() < 0.5))
    return o


def sub_object_type(rng: random.Random, idx: int) -> Schema:
    namer = _Namer(f"sub{idx}_")
    o = Schema("object", rule=f"sub{idx}")
    names = set()
    for i in range(rng.randint(2, 6)):
        name = _ident(rng)
        while name in names:
            name = _ident(rng)
        names.add(name)
        o.props.append((name, _leaf(rng, namer), i == 0 or rng.random() < 0.6))
    return o


def repetition_stress_ebnf(max_objects: int = 1000) -> str:
    """JSON array of 1..max_objects objects, each with a string of 0..64 characters and an
    integer of 1..19 digits."""
    return (f'root ::= "[" ws item (ws "," ws item){{0,{max_objects - 1}}} ws "]"\n'
            'item ::= "{" ws "\\"s\\"" ws ":" ws str ws "," ws "\\"n\\"" ws ":" ws int ws "}"\n'
            'str ::= "\\"" [^"\\\\\\x00-\\x1F]{0,64} "\\""\n'
            'int ::= "-"? [0-9]{1,19}\n'
            'ws ::= [ \\n\\t]*\n')


# ---------------------------------------------------------------- random documents

_STR_ALPHA = "".join(chr(c) for c in range(0x20, 0x7F) if chr(c) not in '"\\')


def _ws(rng: random.Random) -> str:
    r = rng.random()
    if r < 0.6:
        return ""
    if r < 0.9:
        return rng.choice(WS_CHARS)
    return rng.choice(WS_CHARS) + rng.choice(WS_CHARS)


def _rand_string(rng: random.Random, max_len: int = 12, escapes: bool = True, ascii_only: bool = False) -> str:
    """Rendered JSON string *body* (already escaped)."""
    out = []
    for _ in range(rng.randint(0, max_len)):
        r = rng.random()
        if escapes and r < 0.04:
            out.append("\\" + rng.choice('"\\/bfnrt'))
        elif escapes and r < 0.06:
            out.append("\\u" + "".join(rng.choice("0123456789abcdefABCDEF") for _ in range(4)))
        elif r < 0.10 and not ascii_only:
            cp = rng.choice((rng.randrange(0x80, 0x800), rng.randrange(0x800, 0xD800),
                             rng.randrange(0xE000, 0x10000), rng.randrange(0x10000, 0x110000)))
            out.append(chr(cp))
        else:
            out.append(rng.choice(_STR_ALPHA))
    return "".join(out)


def _rand_int(rng: random.Random) -> str:
    if rng.random() < 0.15:
        return "0"
    s = rng.choice("123456789") + "".join(rng.choice("0123456789") for _ in range(rng.randint(0, 6)))
    return ("-" if rng.random() < 0.3 else "") + s


def random_value(s: Schema, rng: random.Random, ascii_only: bool = False) -> Any:
    """A random document of schema `s` as a nested structure of already-rendered leaves."""
    if s.kind == "string":
        return ("string", _rand_string(rng, ascii_only=ascii_only))
    if s.kind == "integer":
        return ("integer", _rand_int(rng))
    if s.kind == "number":
        t = _rand_int(rng)
        if rng.random() < 0.5:
            t += "." + "".join(rng.choice("0123456789") for _ in range(rng.randint(1, 4)))
        if rng.random() < 0.25:
            t += rng.choice("eE") + rng.choice(("", "+", "-")) + str(rng.randint(0, 30))
        return ("number", t)
    if s.kind == "boolean":
        return ("boolean", rng.choice(("true", "false")))
    if s.kind == "enum":
        return ("enum", rng.choice(s.values))
    if s.kind == "array":
        hi = s.max_items if s.max_items is not None else s.min_items + 3
        n = rng.randint(s.min_items, min(hi, s.min_items + 3))
        return ("array", [random_value(s.items, rng, ascii_only) for _ in range(n)])
    if s.kind == "object":
        kv = []
        for i, (name, ps, req) in enumerate(s.props):
            if i == 0 or req or rng.random() < 0.5:
                kv.append((name, random_value(ps, rng, ascii_only)))
        return ("object", kv)
    raise ValueError(s.kind)


def render_value(v: Any, rng: random.Random) -> str:
    """Text of a document with random whitespace wherever the grammar has `ws`."""
    kind, x = v
    if kind in ("integer", "number", "boolean"):
        return x
    if kind == "string":
        return '"' + x + '"'
    if kind == "enum":
        return '"' + x + '"'
    if kind == "array":
        if not x:
            return "[" + _ws(rng) + _ws(rng) + "]"
        body = render_value(x[0], rng)
        for e in x[1:]:
            body += _ws(rng) + "," + _ws(rng) + render_value(e, rng)
        return "[" + _ws(rng) + body + _ws(rng) + "]"
    if kind == "object":
        parts = []
        for i, (name, pv) in enumerate(x):
            kv = '"' + name + '"' + _ws(rng) + ":" + _ws(rng) + render_value(pv, rng)
            parts.append(kv if i == 0 else _ws(rng) + "," + _ws(rng) + kv)
        return "{" + _ws(rng) + "".join(parts) + _ws(rng) + "}"
    raise ValueError(kind)


def value_to_python(v: Any):
    """The document as json.loads would see it (for cross-checks against the json module)."""
    import json
    kind, x = v
    if kind == "string":
        return json.loads('"' + x + '"')
    if kind == "integer":
        return int(x)
    if kind == "number":
        return float(x)
    if kind == "boolean":
        return x == "true"
    if kind == "enum":
        return x
    if kind == "array":
        return [value_to_python(e) for e in x]
    return {k: value_to_python(pv) for k, pv in x}
