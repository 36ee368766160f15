"""CPU ORACLE -- test infrastructure only.

Plain BNF (productions over byte-set terminals and nonterminals) for the Earley recogniser,
obtained two independent ways from the same EBNF:

  direct_bnf   textbook desugaring of the syntax tree: one fresh nonterminal per group,
               alternation = several productions, X* = (empty | X X*), X{m,n} = m copies and
               n-m nested options; TagDispatch = the naive (un-minimised) dispatch automaton
               written as a right-linear grammar.
  fsm_bnf      the canonical minimal DFAs of `fsm.Lowered`, one nonterminal per (rule, state):
               N(R,q) -> [bytes] N(R,q') | N(Q,0) N(R,q') | empty (q final).

Both describe the same language; the tests check that they agree, which pins the automaton
construction and minimisation used to name cache positions.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

from . import fsm as F


class BNF:
    def __init__(self):
        self.n_nt = 0
        self.prods: List[Tuple[int, List[int]]] = []
        self.tsets: List[int] = []
        self._tset_id: Dict[int, int] = {}
        self.names: Dict[object, int] = {}

    def nt(self, key=None) -> int:
        if key is not None and key in self.names:
            return self.names[key]
        i = self.n_nt
        self.n_nt += 1
        if key is not None:
            self.names[key] = i
        return i

    def term(self, mask: int) -> int:
        if mask not in self._tset_id:
            self._tset_id[mask] = len(self.tsets)
            self.tsets.append(mask)
        return self._tset_id[mask]

    def add(self, lhs: int, rhs: List[int]):
        self.prods.append((lhs, list(rhs)))


def _dfa_to_right_linear(b: BNF, d: F.DFA, key_of_state, rule_start_nt) -> None:
    for q in range(d.n):
        lhs = b.nt(key_of_state(q))
        for mask, t in d.bedges[q]:
            b.add(lhs, [b.term(mask), ~b.nt(key_of_state(t))])
        for r, t in d.redges[q].items():
            b.add(lhs, [~rule_start_nt(r), ~b.nt(key_of_state(t))])
        if d.final[q]:
            b.add(lhs, [])


def fsm_bnf(low: F.Lowered) -> BNF:
    b = BNF()
    for nm in low.reachable:
        d = low.dfa[nm]
        _dfa_to_right_linear(b, d, lambda q, nm=nm: (nm, q), lambda r: b.nt((low.order[r], 0)))
    return b


def add_follow(b: BNF, low: F.Lowered) -> None:
    """Follow languages as extra nonterminals ("follow", R): whatever can come after an instance of rule R
    in a sentential form of the root.  follow(R) -> N(Q, x) follow(Q) for every edge  s --R--> x  of a
    rule Q;  follow(root) -> empty  as well."""
    for nm in low.reachable:
        b.nt(("follow", nm))
    b.add(b.nt(("follow", low.root)), [])
    for q_rule in low.reachable:
        d = low.dfa[q_rule]
        seen = set()
        for q in range(d.n):
            for r, x in d.redges[q].items():
                if (r, x) in seen:
                    continue
                seen.add((r, x))
                b.add(b.nt(("follow", low.order[r])), [~b.nt((q_rule, x)), ~b.nt(("follow", q_rule))])


def direct_bnf(order: List[str], rules: Dict[str, tuple], root: str) -> BNF:
    b = BNF()
    index = {nm: i for i, nm in enumerate(order)}
    cls_cache: Dict[tuple, int] = {}
    reachable: List[str] = []

    def sym(node) -> int:
        """A single grammar symbol deriving exactly the language of `node`."""
        k = node[0]
        if k == "lit":
            data = "".join(chr(c) for c in node[1]).encode("utf-8")
            if len(data) == 1:
                return b.term(1 << data[0])
            n = b.nt()
            b.add(n, [b.term(1 << x) for x in data])
            return ~n
        if k == "cls":
            key = (node[1], tuple(node[2]))
            if key not in cls_cache:
                d = F.class_dfa(node[1], tuple(node[2]))
                tag = ("cls", len(cls_cache))
                _dfa_to_right_linear(b, d, lambda q, tag=tag: (tag, q), lambda r: 0)
                cls_cache[key] = b.nt((tag, d.start))
            return ~cls_cache[key]
        if k == "ref":
            if node[1] not in reachable:
                reachable.append(node[1])
            return ~b.nt(("rule", node[1]))
        if k == "seq":
            n = b.nt()
            b.add(n, [sym(c) for c in node[1]])
            return ~n
        if k == "alt":
            n = b.nt()
            for c in node[1]:
                b.add(n, [sym(c)])
            return ~n
        if k == "rep":
            _, x, m, hi = node
            xs = sym(x)
            n = b.nt()
            if hi is None:
                star = b.nt()
                b.add(star, [])
                b.add(star, [xs, ~star])
                b.add(n, [xs] * m + [~star])
            else:
                tail = b.nt()
                b.add(tail, [])                      # zero further copies
                for _ in range(hi - m):
                    outer = b.nt()
                    b.add(outer, [])
                    b.add(outer, [xs, ~tail])
                    tail = outer
                b.add(n, [xs] * m + [~tail])
            return ~n
        raise ValueError(k)

    def define(nm: str):
        node = rules[nm]
        lhs = b.nt(("rule", nm))
        if node[0] == "tagdispatch":
            pairs = [(t, index[r]) for t, r in node[1]]
            for _, r in node[1]:
                if r not in reachable:
                    reachable.append(r)
            d = F.tagdispatch_dfa(pairs, node[2])
            _dfa_to_right_linear(b, d, lambda q, nm=nm: ("td", nm, q), lambda r: b.nt(("rule", order[r])))
            b.add(lhs, [~b.nt(("td", nm, d.start))])
        else:
            b.add(lhs, [sym(node)])

    reachable.append(root)
    i = 0
    while i < len(reachable):
        define(reachable[i])
        i += 1
    return b
