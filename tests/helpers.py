"""Shared by the GPU parity tests: load a workload on both sides."""
from __future__ import annotations

import numpy as np

import gen
import oracle


def planes_of(orc: oracle.Oracle, pos, va, parent=None, follow=False, threads: int = 0):
    cls = orc.classes(pos, va, threads=threads, parent=parent, follow=follow)
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


def all_contexts(orc: oracle.Oracle, depth: int):
    """Every (position, parent) combination a cache of the given context depth must serve: at depth 1 each
    position alone; at depth 2 each position of the root rule alone plus each position of a rule with each
    state a referencing rule continues in."""
    out = []
    sites = {}
    for q_rule in orc.low.reachable:
        d = orc.low.dfa[q_rule]
        for q in range(d.n):
            for r, x in d.redges[q].items():
                sites.setdefault(orc.order[r], set()).add((q_rule, x))
    for pos in orc.positions():
        if depth == 1 or pos[0] == orc.root:
            out.append((pos, None))
        if depth == 2:
            for parent in sorted(sites.get(pos[0], ())):
                out.append((pos, parent))
    return out
