"""Shared by the GPU parity tests: load a workload on both sides."""
from __future__ import annotations

import numpy as np

import gen
import oracle


def planes_of(orc: oracle.Oracle, pos, va, threads: int = 0):
    cls = orc.classes(pos, va, threads=threads)
    return oracle.pack_bitmask(cls == oracle.ACCEPTED), oracle.pack_bitmask(cls == oracle.UNCERTAIN)


def load(index: int, **kw):
    import paper_2601_04426_amd as xg
    cfg = gen.build_config(index, **kw)
    vocab = xg.Vocab(cfg.vocab.tokens, cfg.vocab.eos_id, cfg.vocab.special_ids)
    va = oracle.VocabArrays(cfg.vocab.tokens, cfg.vocab.eos_id, cfg.vocab.special_ids)
    return cfg, vocab, va


def diff_words(got: np.ndarray, want: np.ndarray, tokens, limit: int = 5):
    """Human-readable list of the first differing token ids."""
    x = (got.view(np.uint32) ^ want.view(np.uint32))
    out = []
    for w in np.nonzero(x)[0]:
        for b in range(32):
            if (int(x[w]) >> b) & 1:
                tid = int(w) * 32 + b
                out.append((tid, tokens[tid] if tid < len(tokens) else None, bool((int(got.view(np.uint32)[w]) >> b) & 1)))
                if len(out) >= limit:
                    return out
    return out
