"""Token traces: random segmentation of a byte string into vocabulary tokens."""
from __future__ import annotations

import random
from typing import Dict, List

from .vocab import Vocab


class Segmenter:
    def __init__(self, vocab: Vocab):
        self.by_bytes: Dict[bytes, int] = {}
        self.max_len = 1
        special = set(vocab.special_ids)
        for i, t in enumerate(vocab.tokens):
            if t and i not in special and t not in self.by_bytes:
                self.by_bytes[t] = i
                self.max_len = max(self.max_len, len(t))

    def segment(self, text: bytes, rng: random.Random) -> List[int]:
        """A random split of `text` into tokens of the vocabulary (every needed single byte
        must be a token).  Longer matches are preferred two times out of three."""
        out: List[int] = []
        pos = 0
        n = len(text)
        while pos < n:
            cands = []
            for ln in range(1, min(self.max_len, n - pos) + 1):
                tid = self.by_bytes.get(text[pos:pos + ln])
                if tid is not None:
                    cands.append((ln, tid))
            if not cands:
                raise ValueError(f"byte {text[pos]:#x} is not a token of the vocabulary")
            if rng.random() < 0.67:
                ln, tid = cands[-1]
            else:
                ln, tid = rng.choice(cands)
            out.append(tid)
            pos += ln
        return out


def segment(vocab: Vocab, text: bytes, rng: random.Random) -> List[int]:
    return Segmenter(vocab).segment(text, rng)
