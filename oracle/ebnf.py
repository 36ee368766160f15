r"""CPU ORACLE -- test infrastructure only.

Reader for the EBNF dialect (paper section 2.1 uses EBNF without fixing a syntax; this is the
subset the workloads need) and the TagDispatch intrinsic of section 3.2.

    rule      NAME ::= alternation           a rule ends where the next `NAME ::=` begins
    alternation   sequence ("|" sequence)*
    sequence      term*                      empty sequence = empty string
    term          atom ("*" | "+" | "?" | "{m}" | "{m,n}" | "{m,}")?
    atom          "literal" | [class] | NAME | "(" alternation ")"
    literal / class escapes   \" \\ \n \t \r \/ \xHH \uHHHH \UHHHHHHHH (code points), in classes
                              also \- \] \[ \^
    class         [a-z0-9_], negated [^...] = every Unicode scalar value not listed
    comments      # to end of line
    intrinsic     NAME ::= TagDispatch(("tag", rule), ..., stop_strs=("s", ...))   (whole rule body)

Abstract syntax (tuples):
    ("lit", [code points])  ("cls", negated, [(lo, hi), ...])  ("ref", name)
    ("seq", [nodes])  ("alt", [nodes])  ("rep", node, m, n_or_None)
    ("tagdispatch", [(tag_bytes, rule_name)], [stop_bytes])
"""
from __future__ import annotations

from typing import Dict, List, Tuple


class EBNFError(ValueError):
    pass


_NAME_START = set("abcdefghijklmnopqrstuvwxyzABCDEFGHIJKLMNOPQRSTUVWXYZ_")
_NAME_CONT = _NAME_START | set("0123456789.-")


class _P:
    def __init__(self, text: str):
        self.s = text
        self.i = 0

    def err(self, msg):
        line = self.s.count("\n", 0, self.i) + 1
        raise EBNFError(f"line {line}: {msg}")

    def skip(self):
        while self.i < len(self.s):
            c = self.s[self.i]
            if c in " \t\r\n":
                self.i += 1
            elif c == "#":
                while self.i < len(self.s) and self.s[self.i] != "\n":
                    self.i += 1
            else:
                break

    def peek(self):
        self.skip()
        return self.s[self.i] if self.i < len(self.s) else ""

    def name(self):
        self.skip()
        j = self.i
        if j < len(self.s) and self.s[j] in _NAME_START:
            j += 1
            while j < len(self.s) and self.s[j] in _NAME_CONT:
                j += 1
            nm = self.s[self.i:j]
            self.i = j
            return nm
        return None

    def at_rule_head(self):
        """True if what follows is `NAME ::=`."""
        save = self.i
        nm = self.name()
        ok = False
        if nm is not None:
            self.skip()
            ok = self.s.startswith("::=", self.i)
        self.i = save
        return ok

    def escape(self, in_class: bool) -> int:
        c = self.s[self.i]
        self.i += 1
        simple = {'"': 34, "\\": 92, "n": 10, "t": 9, "r": 13, "/": 47, "'": 39}
        if in_class:
            simple.update({"-": 45, "]": 93, "[": 91, "^": 94})
        if c in simple:
            return simple[c]
        width = {"x": 2, "u": 4, "U": 8}.get(c)
        if width is None:
            self.err(f"unknown escape \\{c}")
        h = self.s[self.i:self.i + width]
        if len(h) != width or any(ch not in "0123456789abcdefABCDEF" for ch in h):
            self.err("bad hex escape")
        self.i += width
        cp = int(h, 16)
        if cp > 0x10FFFF or 0xD800 <= cp <= 0xDFFF:
            self.err("escape is not a Unicode scalar value")
        return cp

    def literal(self) -> List[int]:
        assert self.s[self.i] == '"'
        self.i += 1
        out = []
        while True:
            if self.i >= len(self.s):
                self.err("unterminated literal")
            c = self.s[self.i]
            if c == '"':
                self.i += 1
                return out
            if c == "\\":
                self.i += 1
                out.append(self.escape(False))
            else:
                out.append(ord(c))
                self.i += 1

    def cls(self):
        assert self.s[self.i] == "["
        self.i += 1
        neg = False
        if self.i < len(self.s) and self.s[self.i] == "^":
            neg = True
            self.i += 1
        ranges = []

        def one():
            if self.i >= len(self.s):
                self.err("unterminated class")
            c = self.s[self.i]
            if c == "\\":
                self.i += 1
                return self.escape(True)
            self.i += 1
            return ord(c)
        while True:
            if self.i >= len(self.s):
                self.err("unterminated class")
            if self.s[self.i] == "]":
                self.i += 1
                break
            lo = one()
            hi = lo
            if self.i + 1 < len(self.s) and self.s[self.i] == "-" and self.s[self.i + 1] != "]":
                self.i += 1
                hi = one()
                if hi < lo:
                    self.err("reversed range in class")
            ranges.append((lo, hi))
        return ("cls", neg, ranges)

    def number(self) -> int:
        self.skip()
        j = self.i
        while j < len(self.s) and self.s[j].isdigit():
            j += 1
        if j == self.i:
            self.err("number expected")
        v = int(self.s[self.i:j])
        self.i = j
        return v

    def atom(self):
        c = self.peek()
        if c == '"':
            return ("lit", self.literal())
        if c == "[":
            return self.cls()
        if c == "(":
            self.i += 1
            n = self.alternation()
            if self.peek() != ")":
                self.err("')' expected")
            self.i += 1
            return n
        nm = self.name()
        if nm is None:
            self.err(f"unexpected character {c!r}")
        return ("ref", nm)

    def term(self):
        a = self.atom()
        while True:
            c = self.peek()
            if c == "*":
                self.i += 1
                a = ("rep", a, 0, None)
            elif c == "+":
                self.i += 1
                a = ("rep", a, 1, None)
            elif c == "?":
                self.i += 1
                a = ("rep", a, 0, 1)
            elif c == "{":
                self.i += 1
                m = self.number()
                n = m
                if self.peek() == ",":
                    self.i += 1
                    n = None if self.peek() == "}" else self.number()
                if self.peek() != "}":
                    self.err("'}' expected")
                self.i += 1
                if n is not None and n < m:
                    self.err("repetition bounds reversed")
                a = ("rep", a, m, n)
            else:
                return a

    def sequence(self):
        items = []
        while True:
            c = self.peek()
            if c == "" or c in "|)" or self.at_rule_head():
                break
            items.append(self.term())
        return items[0] if len(items) == 1 else ("seq", items)

    def alternation(self):
        alts = [self.sequence()]
        while self.peek() == "|":
            self.i += 1
            alts.append(self.sequence())
        return alts[0] if len(alts) == 1 else ("alt", alts)

    def expect(self, tok):
        self.skip()
        if not self.s.startswith(tok, self.i):
            self.err(f"{tok!r} expected")
        self.i += len(tok)

    def tagdispatch(self):
        self.expect("(")
        pairs, stops = [], []
        while True:
            c = self.peek()
            if c == "(":
                self.i += 1
                if self.peek() != '"':
                    self.err("tag literal expected")
                tag = self.literal()
                self.expect(",")
                nm = self.name()
                if nm is None:
                    self.err("rule name expected")
                self.expect(")")
                pairs.append((_utf8(tag), nm))
            elif self.s.startswith("stop_strs", self.i):
                self.i += len("stop_strs")
                self.expect("=")
                self.expect("(")
                while self.peek() == '"':
                    stops.append(_utf8(self.literal()))
                    if self.peek() == ",":
                        self.i += 1
                self.expect(")")
            else:
                self.err("tag pair or stop_strs expected")
            if self.peek() == ",":
                self.i += 1
                continue
            break
        self.expect(")")
        return ("tagdispatch", pairs, stops)


def _utf8(cps: List[int]) -> bytes:
    return "".join(chr(c) for c in cps).encode("utf-8")


def parse_ebnf(text: str) -> Tuple[List[str], Dict[str, tuple]]:
    """-> (rule names in declaration order, {name: abstract syntax})."""
    p = _P(text)
    order: List[str] = []
    rules: Dict[str, tuple] = {}
    while p.peek() != "":
        nm = p.name()
        if nm is None:
            p.err("rule name expected")
        p.expect("::=")
        p.skip()
        save = p.i
        head = p.name()
        if head == "TagDispatch" and p.peek() == "(":
            body = p.tagdispatch()
        else:
            p.i = save
            body = p.alternation()
        if p.peek() != "" and not p.at_rule_head():
            p.err("unexpected text after rule body")
        if nm in rules:
            p.err(f"rule {nm} defined twice")
        order.append(nm)
        rules[nm] = body
    _check_refs(order, rules)
    return order, rules


def _check_refs(order, rules):
    def walk(n):
        k = n[0]
        if k == "ref":
            if n[1] not in rules:
                raise EBNFError(f"undefined rule {n[1]}")
        elif k in ("seq", "alt"):
            for c in n[1]:
                walk(c)
        elif k == "rep":
            walk(n[1])
        elif k == "tagdispatch":
            for _, r in n[1]:
                if r not in rules:
                    raise EBNFError(f"undefined rule {r}")
    for nm in order:
        walk(rules[nm])
