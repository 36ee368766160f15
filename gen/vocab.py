"""Seeded synthetic vocabularies shaped like byte-level BPE vocabularies.

Token id 0 is always the end-of-sequence token (no bytes, special).
"""
from __future__ import annotations

import random
from dataclasses import dataclass, field
from typing import List

STRUCTURAL = b'{}[]:,"\\ \t\n\r'          # 12 structural / whitespace bytes
PRINTABLE = bytes(range(0x20, 0x7F))


@dataclass
class Vocab:
    tokens: List[bytes]                    # tokens[id] = byte string
    eos_id: int = 0
    special_ids: List[int] = field(default_factory=lambda: [0])

    @property
    def size(self) -> int:
        return len(self.tokens)

    def csr(self):
        """(bytes blob, offsets[V+1]) in token-id order."""
        offs = [0]
        for t in self.tokens:
            offs.append(offs[-1] + len(t))
        return b"".join(self.tokens), offs


def _weighted_alphabet() -> List[int]:
    pool: List[int] = []
    for b in PRINTABLE:
        pool.extend([b] * (3 if b in STRUCTURAL else 1))
    for b in b"\t\n\r":
        pool.extend([b] * 3)
    return pool


def _utf8_scalar(rng: random.Random) -> bytes:
    n = rng.choice((2, 3, 4))
    while True:
        if n == 2:
            cp = rng.randrange(0x80, 0x800)
        elif n == 3:
            cp = rng.randrange(0x800, 0x10000)
            if 0xD800 <= cp <= 0xDFFF:
                continue
        else:
            cp = rng.randrange(0x10000, 0x110000)
        return chr(cp).encode("utf-8")


def make_vocab(size: int, seed: int, style: str) -> Vocab:
    """style 'tiny': lengths uniform 1..8 over weighted printable ASCII, every
    printable byte and tab/newline/CR present as a single-byte token.
    style 'bpe': lengths geometric (p=1/4, mean 4) clamped to 16, 5 % of the
    tokens forced to hold a structural byte, 2 % are one UTF-8 encoded scalar of
    2-4 bytes, all 256 single bytes present.  Strings are unique."""
    rng = random.Random(seed)
    pool = _weighted_alphabet()
    toks: List[bytes] = [b""]              # id 0 = EOS
    seen = {b""}
    if style == "tiny":
        singles = list(PRINTABLE) + [9, 10, 13]
    else:
        singles = list(range(256))
    singles_b = [bytes([b]) for b in singles]
    rng.shuffle(singles_b)
    if size < len(singles_b) + 1:
        raise ValueError("vocabulary too small for its guaranteed single-byte tokens")
    body: List[bytes] = []
    seen.update(singles_b)
    need = size - 1 - len(singles_b)
    while len(body) < need:
        if style == "tiny":
            n = rng.randint(1, 8)
            t = bytes(rng.choice(pool) for _ in range(n))
        else:
            u = rng.random()
            if u < 0.02:
                t = _utf8_scalar(rng)
            else:
                n = 1
                while n < 16 and rng.random() >= 0.25:
                    n += 1
                t = bytearray(rng.choice(pool) for _ in range(n))
                if u < 0.07:
                    t[rng.randrange(n)] = rng.choice(STRUCTURAL)
                t = bytes(t)
        if t in seen:
            continue
        seen.add(t)
        body.append(t)
    rest = singles_b + body
    rng.shuffle(rest)
    toks.extend(rest)
    return Vocab(tokens=toks, eos_id=0, special_ids=[0])
