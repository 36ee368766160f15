"""CPU ORACLE -- test infrastructure only.

Per-rule finite-state machines (paper section 3.3: every rule is one FSM whose edges are
character edges, rule-reference edges or epsilon edges; "we attempt to transform most FSMs
into DFAs", appendix "More Explanation of the Hash Algorithm").

Here every rule body is read as a regular expression over the alphabet
    {byte 0..255}  U  {one symbol per rule name},
and its FSM is THE minimal partial DFA of that regular language (unique up to renaming),
renamed canonically: breadth-first from the start state, out-edges visited by ascending byte
value and then by ascending declaration index of the referenced rule.  A cache position is
(rule, canonical state) with at least one byte edge (section 3.4: only scannable states are
cached).

Characters are Unicode scalar values matched byte-wise on their UTF-8 encoding; a negated
class is the complement over all scalar values.
"""
from __future__ import annotations

from collections import deque
from typing import Dict, List, Optional, Tuple

FULL = (1 << 256) - 1


def _mask_range(lo: int, hi: int) -> int:
    return ((1 << (hi + 1)) - 1) ^ ((1 << lo) - 1)


def scalar_ranges(neg: bool, ranges: List[Tuple[int, int]]) -> List[Tuple[int, int]]:
    """Sorted disjoint ranges of Unicode scalar values (no surrogates) denoted by a class."""
    rs = sorted(ranges)
    merged: List[List[int]] = []
    for lo, hi in rs:
        if merged and lo <= merged[-1][1] + 1:
            merged[-1][1] = max(merged[-1][1], hi)
        else:
            merged.append([lo, hi])
    if neg:
        out, prev = [], 0
        for lo, hi in merged:
            if lo > prev:
                out.append([prev, lo - 1])
            prev = hi + 1
        if prev <= 0x10FFFF:
            out.append([prev, 0x10FFFF])
        merged = out
    final = []
    for lo, hi in merged:                       # cut out the surrogate block
        hi = min(hi, 0x10FFFF)
        if lo > hi:
            continue
        if hi < 0xD800 or lo > 0xDFFF:
            final.append((lo, hi))
        else:
            if lo < 0xD800:
                final.append((lo, 0xD7FF))
            if hi > 0xDFFF:
                final.append((0xE000, hi))
    return final


def utf8_groups(ranges: List[Tuple[int, int]]) -> Dict[bytes, int]:
    """{all-but-last bytes of the encoding: set of last bytes}, by encoding with Python's own
    UTF-8 encoder one block of <= 64 consecutive scalars (same leading bytes) at a time."""
    groups: Dict[bytes, int] = {}
    for lo, hi in ranges:
        cp = lo
        while cp <= hi:
            if cp < 0x80:
                end = min(hi, 0x7F)
                prefix, first = b"", cp
            else:
                end = min(hi, cp | 0x3F)
                enc = chr(cp).encode("utf-8")
                prefix, first = enc[:-1], enc[-1]
            groups[prefix] = groups.get(prefix, 0) | _mask_range(first, first + (end - cp))
            cp = end + 1
    return groups


class NFA:
    def __init__(self):
        self.edges: List[List[Tuple[object, int]]] = []   # label: int mask | ("r", idx) | None

    def new(self) -> int:
        self.edges.append([])
        return len(self.edges) - 1

    def add(self, a: int, label, b: int):
        self.edges[a].append((label, b))


class DFA:
    """bedges[s] = [(mask, target)] with disjoint masks, redges[s] = {rule index: target}."""

    def __init__(self):
        self.bedges: List[List[Tuple[int, int]]] = []
        self.redges: List[Dict[int, int]] = []
        self.final: List[bool] = []
        self.start = 0

    def new(self, final=False) -> int:
        self.bedges.append([])
        self.redges.append({})
        self.final.append(final)
        return len(self.final) - 1

    @property
    def n(self):
        return len(self.final)


def _build(node, nfa: NFA, rule_index: Dict[str, int]) -> Tuple[int, int]:
    k = node[0]
    s, e = nfa.new(), nfa.new()
    if k == "lit":
        cur = s
        data = "".join(chr(c) for c in node[1]).encode("utf-8")
        for b in data:
            nx = nfa.new()
            nfa.add(cur, 1 << b, nx)
            cur = nx
        nfa.add(cur, None, e)
    elif k == "cls":
        d = class_dfa(node[1], tuple(node[2]))          # small: copy it in as a fragment
        st = [nfa.new() for _ in range(d.n)]
        nfa.add(s, None, st[d.start])
        for q in range(d.n):
            for mask, t in d.bedges[q]:
                nfa.add(st[q], mask, st[t])
            if d.final[q]:
                nfa.add(st[q], None, e)
    elif k == "ref":
        nfa.add(s, ("r", rule_index[node[1]]), e)
    elif k == "seq":
        cur = s
        for c in node[1]:
            a, b = _build(c, nfa, rule_index)
            nfa.add(cur, None, a)
            cur = b
        nfa.add(cur, None, e)
    elif k == "alt":
        for c in node[1]:
            a, b = _build(c, nfa, rule_index)
            nfa.add(s, None, a)
            nfa.add(b, None, e)
    elif k == "rep":
        _, x, m, n = node
        cur = s
        for _ in range(m):
            a, b = _build(x, nfa, rule_index)
            nfa.add(cur, None, a)
            cur = b
        if n is None:
            a, b = _build(x, nfa, rule_index)
            nfa.add(cur, None, a)
            nfa.add(b, None, cur)
            nfa.add(cur, None, e)
        else:
            nfa.add(cur, None, e)
            for _ in range(n - m):
                a, b = _build(x, nfa, rule_index)
                nfa.add(cur, None, a)
                cur = b
                nfa.add(cur, None, e)
    else:
        raise ValueError(k)
    return s, e


_CLASS_CACHE: Dict[tuple, "DFA"] = {}


def class_dfa(neg: bool, ranges: tuple) -> "DFA":
    """Minimal DFA over bytes of the UTF-8 encodings of one character class: a trie over the
    encodings (grouped by all-but-last byte), minimised."""
    key = (neg, ranges)
    if key not in _CLASS_CACHE:
        nfa = NFA()
        s, e = nfa.new(), nfa.new()
        trie: Dict[bytes, int] = {b"": s}
        for prefix, mask in sorted(utf8_groups(scalar_ranges(neg, list(ranges))).items()):
            for i in range(1, len(prefix) + 1):
                if prefix[:i] not in trie:
                    trie[prefix[:i]] = nfa.new()
                    nfa.add(trie[prefix[:i - 1]], 1 << prefix[i - 1], trie[prefix[:i]])
            nfa.add(trie[prefix], mask, e)
        _CLASS_CACHE[key] = minimize(nfa_to_dfa(nfa, s, e))
    return _CLASS_CACHE[key]


def _atoms(masks) -> List[int]:
    """Coarsest partition of the bytes covered by `masks` such that every mask is a union of parts."""
    parts: List[int] = []
    for m in masks:
        rest = m
        nxt = []
        for p in parts:
            i = p & m
            if i:
                nxt.append(i)
                if p & ~m:
                    nxt.append(p & ~m)
                rest &= ~p
            else:
                nxt.append(p)
        if rest:
            nxt.append(rest)
        parts = nxt
    return parts


def nfa_to_dfa(nfa: NFA, start: int, end: int) -> DFA:
    def closure(states):
        seen = set(states)
        stack = list(states)
        while stack:
            q = stack.pop()
            for lab, d in nfa.edges[q]:
                if lab is None and d not in seen:
                    seen.add(d)
                    stack.append(d)
        return frozenset(seen)

    dfa = DFA()
    s0 = closure([start])
    ids = {s0: dfa.new(end in s0)}
    work = deque([s0])
    while work:
        S = work.popleft()
        sid = ids[S]
        bmasks, rlabels = [], set()
        for q in S:
            for lab, d in nfa.edges[q]:
                if isinstance(lab, int):
                    bmasks.append(lab)
                elif lab is not None:
                    rlabels.add(lab[1])
        targets = []
        for atom in _atoms(sorted(set(bmasks))):
            T = closure([d for q in S for lab, d in nfa.edges[q] if isinstance(lab, int) and lab & atom])
            targets.append(("b", atom, T))
        for r in sorted(rlabels):
            T = closure([d for q in S for lab, d in nfa.edges[q] if lab == ("r", r)])
            targets.append(("r", r, T))
        for kind, lab, T in targets:
            if T not in ids:
                ids[T] = dfa.new(end in T)
                work.append(T)
            if kind == "b":
                dfa.bedges[sid].append((lab, ids[T]))
            else:
                dfa.redges[sid][lab] = ids[T]
    return dfa


def tagdispatch_dfa(pairs: List[Tuple[bytes, int]], stops: List[bytes]) -> DFA:
    """Section 3.2 read as a regular language over bytes and rule symbols, built the naive way:
    a dispatching-mode state is the longest suffix of the text since the last return that is a
    proper prefix of a tag or stop string; each byte either completes a pattern (a tag: go through
    the tag's rule and return to the empty-suffix state; a stop string: exit) or moves to the state
    of the new longest suffix.  Any byte is free text.  Without stop strings the construct may end
    at any moment of the dispatching mode; with stop strings only right after one."""
    patterns = [t for t, _ in pairs] + list(stops)
    if any(len(p) == 0 for p in patterns):
        raise ValueError("empty tag or stop string")
    for i, a in enumerate(patterns):
        for j, b in enumerate(patterns):
            if i != j and a in b:
                raise ValueError("a tag or stop string occurs inside another one")
    prefixes = sorted({p[:i] for p in patterns for i in range(len(p))})
    dfa = DFA()
    st = {u: dfa.new(final=(len(stops) == 0)) for u in [b""] + [u for u in prefixes if u]}
    after_tag = []
    for _, rule in pairs:
        x = dfa.new(False)
        dfa.redges[x][rule] = st[b""]
        after_tag.append(x)
    stop_state = dfa.new(True) if stops else None
    for u in st:
        by_target: Dict[int, int] = {}
        for c in range(256):
            w = u + bytes([c])
            tgt = None
            for k, p in enumerate(patterns):
                if w.endswith(p):
                    tgt = after_tag[k] if k < len(pairs) else stop_state
            if tgt is None:
                for cut in range(len(w) + 1):             # longest suffix first
                    if w[cut:] in st:
                        tgt = st[w[cut:]]
                        break
            by_target[tgt] = by_target.get(tgt, 0) | (1 << c)
        dfa.bedges[st[u]] = [(m, t) for t, m in by_target.items()]
    dfa.start = st[b""]
    return dfa


def minimize(dfa: DFA) -> DFA:
    """Hopcroft's partition refinement on the trimmed automaton, then removal of states that
    cannot reach a final state.  Bytes that behave alike in every state are handled as one symbol."""
    n = dfa.n
    # reachable part
    reach = [False] * n
    reach[dfa.start] = True
    stack = [dfa.start]
    while stack:
        q = stack.pop()
        for _, t in dfa.bedges[q]:
            if not reach[t]:
                reach[t] = True
                stack.append(t)
        for t in dfa.redges[q].values():
            if not reach[t]:
                reach[t] = True
                stack.append(t)
    # co-reachable part (can reach a final state)
    rev: List[List[int]] = [[] for _ in range(n)]
    for q in range(n):
        for _, t in dfa.bedges[q]:
            rev[t].append(q)
        for t in dfa.redges[q].values():
            rev[t].append(q)
    live = [False] * n
    stack = [q for q in range(n) if dfa.final[q]]
    for q in stack:
        live[q] = True
    while stack:
        q = stack.pop()
        for p in rev[q]:
            if not live[p]:
                live[p] = True
                stack.append(p)
    keep = [q for q in range(n) if reach[q] and live[q]]
    if dfa.start not in keep:
        raise ValueError("rule has an empty language")
    keepset = set(keep)
    atoms = _atoms(sorted({m for q in keep for m, t in dfa.bedges[q] if t in keepset}))
    rules = sorted({r for q in keep for r, t in dfa.redges[q].items() if t in keepset})
    nsym = len(atoms) + len(rules)
    # delta[q][sym] = target or None, inverse lists per symbol
    delta: Dict[int, List[Optional[int]]] = {}
    inv: List[Dict[int, List[int]]] = [dict() for _ in range(nsym)]
    for q in keep:
        row: List[Optional[int]] = [None] * nsym
        for m, t in dfa.bedges[q]:
            if t in keepset:
                for ai, a in enumerate(atoms):
                    if a & m:
                        row[ai] = t
        for r, t in dfa.redges[q].items():
            if t in keepset:
                row[len(atoms) + rules.index(r)] = t
        delta[q] = row
        for sy, t in enumerate(row):
            if t is not None:
                inv[sy].setdefault(t, []).append(q)
    fin = {q for q in keep if dfa.final[q]}
    non = keepset - fin
    blocks: List[set] = [b for b in (fin, non) if b]
    block_of = {q: i for i, b in enumerate(blocks) for q in b}
    work = deque((i, sy) for i in range(len(blocks)) for sy in range(nsym))
    inwork = set(work)
    while work:
        bi, sy = work.popleft()
        inwork.discard((bi, sy))
        pre: Dict[int, List[int]] = {}
        for t in list(blocks[bi]):
            for q in inv[sy].get(t, ()):
                pre.setdefault(block_of[q], []).append(q)
        for bj, members in pre.items():
            if len(members) == len(blocks[bj]):
                continue
            mem = set(members)
            rest = blocks[bj] - mem
            small, large = (mem, rest) if len(mem) <= len(rest) else (rest, mem)
            blocks[bj] = large
            blocks.append(small)
            nb = len(blocks) - 1
            for q in small:
                block_of[q] = nb
            # Hopcroft: if (bj, s) is still queued both halves must be (bj keeps the larger half and
            # stays queued); otherwise the smaller half alone suffices.  Either way: queue the new block.
            for s2 in range(nsym):
                work.append((nb, s2))
                inwork.add((nb, s2))
    out = DFA()
    for _ in blocks:
        out.new(False)
    for bi, b in enumerate(blocks):
        q = next(iter(b))
        out.final[bi] = dfa.final[q]
        by_t: Dict[int, int] = {}
        for ai, a in enumerate(atoms):
            t = delta[q][ai]
            if t is not None:
                by_t[block_of[t]] = by_t.get(block_of[t], 0) | a
        out.bedges[bi] = [(m, t) for t, m in by_t.items()]
        for ri, r in enumerate(rules):
            t = delta[q][len(atoms) + ri]
            if t is not None:
                out.redges[bi][r] = block_of[t]
    out.start = block_of[dfa.start]
    return out


def canonical(dfa: DFA) -> DFA:
    """Rename states breadth-first: by ascending byte, then ascending rule index."""
    order = [dfa.start]
    ident = {dfa.start: 0}
    i = 0
    while i < len(order):
        q = order[i]
        i += 1
        nxt = sorted(((m & -m).bit_length() - 1, t) for m, t in dfa.bedges[q])
        nxt_r = sorted(dfa.redges[q].items())
        for _, t in nxt + nxt_r:
            if t not in ident:
                ident[t] = len(order)
                order.append(t)
    out = DFA()
    for q in order:
        out.new(dfa.final[q])
    for q in order:
        c = ident[q]
        out.bedges[c] = sorted(((m, ident[t]) for m, t in dfa.bedges[q]), key=lambda e: (e[0] & -e[0]))
        out.redges[c] = {r: ident[t] for r, t in sorted(dfa.redges[q].items())}
    out.start = 0
    return out


def rule_dfa(node, rule_index: Dict[str, int]) -> DFA:
    if node[0] == "tagdispatch":
        raw = tagdispatch_dfa([(t, rule_index[r]) for t, r in node[1]], node[2])
    else:
        nfa = NFA()
        s, e = _build(node, nfa, rule_index)
        raw = nfa_to_dfa(nfa, s, e)
    return canonical(minimize(raw))


class Lowered:
    """All rules reachable from the root as canonical minimal DFAs."""

    def __init__(self, order: List[str], rules: Dict[str, tuple], root: str):
        if root not in rules:
            raise ValueError(f"unknown root rule {root}")
        self.order = order
        self.index = {nm: i for i, nm in enumerate(order)}
        self.root = root
        self.dfa: Dict[str, DFA] = {}
        todo = [root]
        while todo:
            nm = todo.pop()
            if nm in self.dfa:
                continue
            d = rule_dfa(rules[nm], self.index)
            self.dfa[nm] = d
            for q in range(d.n):
                for r in d.redges[q]:
                    todo.append(order[r])
        self.reachable = [nm for nm in order if nm in self.dfa]

    def positions(self) -> List[Tuple[str, int]]:
        return [(nm, q) for nm in self.reachable for q in range(self.dfa[nm].n) if self.dfa[nm].bedges[q]]
