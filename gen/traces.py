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


def random_depth_traces(cfg, seg: Segmenter, batch: int, rng: random.Random, grammar: int = 0):
    """`batch` sentences of workload `cfg` cut into tokens, each with a depth drawn uniformly over its own length:
    the state "concurrent matchers at random depths" starts from.  Returns (traces, depths); a trace ends with the
    end-of-sequence token, and depth < len(trace) - 1 (at least the last text token and the end are still to come)."""
    traces, depths = [], []
    for _ in range(batch):
        ids = seg.segment(cfg.sample_text(rng, grammar), rng) + [cfg.vocab.eos_id]
        traces.append(ids)
        depths.append(rng.randrange(0, max(1, len(ids) - 1)))
    return traces, depths
