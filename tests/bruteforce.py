"""Brute-force language enumeration for tiny grammars -- the yardstick the oracle is pinned to.

Grammars are given here as Python data (not as EBNF text, so that nothing of the oracle's
reader or automata is used):

    ("lit", b"ab")  ("set", b"abc")  ("seq", x, y, ...)  ("alt", x, y, ...)
    ("star", x)  ("opt", x)  ("rep", x, m, n)  ("ref", "rule")

`languages(rules, N)` returns, per rule, the set of all its sentences of length <= N (least
fixed point of the obvious set equations, truncated at N).
"""
from __future__ import annotations

from itertools import product
from typing import Dict, Set


def _cat(a: Set[bytes], b: Set[bytes], N: int) -> Set[bytes]:
    return {x + y for x in a for y in b if len(x) + len(y) <= N}


def _lang(e, env: Dict[str, Set[bytes]], N: int) -> Set[bytes]:
    k = e[0]
    if k == "lit":
        return {e[1]} if len(e[1]) <= N else set()
    if k == "set":
        return {bytes([c]) for c in e[1]} if N >= 1 else set()
    if k == "ref":
        return env[e[1]]
    if k == "seq":
        cur = {b""}
        for c in e[1:]:
            cur = _cat(cur, _lang(c, env, N), N)
        return cur
    if k == "alt":
        out: Set[bytes] = set()
        for c in e[1:]:
            out |= _lang(c, env, N)
        return out
    if k == "opt":
        return {b""} | _lang(e[1], env, N)
    if k == "star":
        base = _lang(e[1], env, N)
        out = {b""}
        while True:
            nxt = out | _cat(out, base, N)
            if nxt == out:
                return out
            out = nxt
    if k == "rep":
        _, x, m, n = e
        base = _lang(x, env, N)
        cur = {b""}
        for _ in range(m):
            cur = _cat(cur, base, N)
        out = set(cur)
        for _ in range(n - m):
            cur = _cat(cur, base, N)
            out |= cur
        return out
    raise ValueError(k)


def languages(rules: Dict[str, tuple], N: int) -> Dict[str, Set[bytes]]:
    env: Dict[str, Set[bytes]] = {nm: set() for nm in rules}
    while True:
        new = {nm: _lang(body, env, N) for nm, body in rules.items()}
        if new == env:
            return env
        env = new


def prefixes(lang: Set[bytes]) -> Set[bytes]:
    return {s[:i] for s in lang for i in range(len(s) + 1)}


def all_strings(alphabet: bytes, max_len: int):
    for n in range(max_len + 1):
        for tup in product(alphabet, repeat=n):
            yield bytes(tup)
