"""Invariants of the CPU oracle on the seeded workloads (reduced sizes where needed).

 * the two independent grammar lowerings (textbook desugaring vs canonical minimal automata)
   give the same masks along real traces;
 * every sampled sentence, cut into vocabulary tokens any way, is allowed token by token and
   end-of-sequence is allowed exactly at its end;
 * masks are prefix-closed inside the vocabulary and never empty while a matcher is alive;
 * random walks over allowed tokens end in sentences (checked with the json module where the
   workload is JSON);
 * combining the cached classes of the scannable frontier the way the paper's runtime does
   reproduces the plain-definition mask (this is what justifies reading "uncertain" as
   "leaves the rule after at least one byte").
"""
import json
import random

import numpy as np
import pytest

import gen
import oracle


def _setup(index, **kw):
    cfg = gen.build_config(index, **kw)
    ebnf, root = cfg.grammars[0]
    o = oracle.Oracle(ebnf, root)
    va = oracle.VocabArrays(cfg.vocab.tokens, cfg.vocab.eos_id, cfg.vocab.special_ids)
    return cfg, o, va


SMALL = {1: {}, 2: {"vocab_size": 3000}, 3: {"vocab_size": 3000, "n_tools": 4}, 5: {"vocab_size": 3000, "max_objects": 6}}


@pytest.mark.parametrize("index", [1, 2, 3, 5])
def test_sentences_are_accepted_token_by_token(index):
    cfg, o, va = _setup(index, **SMALL[index])
    seg = gen.Segmenter(cfg.vocab)
    rng = random.Random(100 + index)
    cls_cache = {}
    for trial in range(3):
        text = cfg.sample_text(rng, 0)
        assert o.accepts(text) and o.accepts(text, direct=True)
        ids = seg.segment(text, rng)
        hist = b""
        for step, tid in enumerate(ids + [cfg.vocab.eos_id]):
            m = o.mask(hist, va)
            assert m.any()
            assert m[tid], (hist, cfg.vocab.tokens[tid])
            if step % 7 == 0 or tid == cfg.vocab.eos_id:
                assert np.array_equal(m, o.mask(hist, va, direct=True)), hist
                # prefix closure inside the vocabulary
                allowed = {cfg.vocab.tokens[i] for i in np.nonzero(m)[0] if i != cfg.vocab.eos_id}
                by_bytes = {t: i for i, t in enumerate(cfg.vocab.tokens)}
                for t in list(allowed)[:300]:
                    for k in range(1, len(t)):
                        if t[:k] in by_bytes:
                            assert t[:k] in allowed
                # runtime combination of cached classes == plain definition
                acc = np.zeros(va.V, dtype=bool)
                unc = np.zeros(va.V, dtype=bool)
                for p in o.frontier(hist):
                    if p not in cls_cache:
                        cls_cache[p] = o.classes(p, va)
                    acc |= cls_cache[p] == oracle.ACCEPTED
                    unc |= cls_cache[p] == oracle.UNCERTAIN
                body = m.copy()
                body[cfg.vocab.eos_id] = False
                assert not (acc & ~body).any(), "an accepted token is not a viable continuation"
                assert not (body & ~(acc | unc)).any(), "a viable token is neither accepted nor uncertain anywhere"
            if tid != cfg.vocab.eos_id:
                hist += cfg.vocab.tokens[tid]
        assert hist == text


def test_random_walks_end_in_valid_json():
    cfg, o, va = _setup(1)
    rng = random.Random(5)
    done = 0
    for trial in range(6):
        hist = b""
        for step in range(120):
            m = o.mask(hist, va)
            allowed = np.nonzero(m)[0]
            assert len(allowed) > 0
            if m[cfg.vocab.eos_id] and (rng.random() < 0.9 or len(allowed) == 1):
                break
            # prefer structure over endless whitespace / string growth
            short = [i for i in allowed if i != cfg.vocab.eos_id and not cfg.vocab.tokens[i].isspace()]
            tid = rng.choice(short if short and rng.random() < 0.9 else [i for i in allowed if i != cfg.vocab.eos_id])
            hist += cfg.vocab.tokens[tid]
        if o.accepts(hist):
            doc = json.loads(hist.decode("utf-8"))
            assert list(doc.keys()) == ["name", "age", "ok"]
            assert isinstance(doc["name"], str) and isinstance(doc["age"], int) and isinstance(doc["ok"], bool)
            done += 1
    assert done >= 1


def test_sampled_documents_load_with_json_module():
    for index in (1, 2):
        cfg = gen.build_config(index, **SMALL[index])
        o = oracle.Oracle(*cfg.grammars[0])
        rng = random.Random(9)
        for _ in range(20):
            text = cfg.sample_text(rng, 0)
            json.loads(text.decode("utf-8"))
            assert o.accepts(text)
            # a damaged document the json module rejects must not be a sentence either
            k = rng.randrange(len(text))
            broken = text[:k] + text[k + 1:]
            try:
                json.loads(broken.decode("utf-8"))
            except Exception:
                assert not o.accepts(broken), broken


def test_everything_grammar_allows_exactly_the_utf8_prefixes():
    """root ::= [^] * (any scalar, any number of times): a token is allowed iff it is a prefix of
    well-formed UTF-8 -- compare with Python's incremental decoder."""
    import codecs
    cfg = gen.build_config(2, vocab_size=6000)
    o = oracle.Oracle("root ::= [\\x00-\\U0010FFFF]*\n")
    va = oracle.VocabArrays(cfg.vocab.tokens, 0, [0])
    m = o.mask(b"", va)
    assert m[0]                                             # empty history is a sentence
    for i, t in enumerate(cfg.vocab.tokens):
        if i == 0:
            continue
        dec = codecs.getincrementaldecoder("utf-8")()
        try:
            dec.decode(t, final=False)
            ok = True
        except UnicodeDecodeError:
            ok = False
        assert m[i] == ok, t
    cls = o.classes(("root", 0), va)
    assert not (cls == oracle.UNCERTAIN).any()              # root never "leaves" early for a viable token...
    assert np.array_equal(cls == oracle.ACCEPTED, np.r_[False, m[1:]])


def test_classes_partition_and_specials():
    cfg, o, va = _setup(1)
    for p in o.positions():
        c = o.classes(p, va)
        assert set(np.unique(c)) <= {oracle.REJECTED, oracle.ACCEPTED, oracle.UNCERTAIN}
        assert c[cfg.vocab.eos_id] == oracle.REJECTED
    # a string-content position: tokens without quote/backslash/control bytes are accepted,
    # tokens that close the string and go on are uncertain
    pos = [p for p in o.positions() if p[0] == "string"]
    c = o.classes(pos[1], va)
    for i, t in enumerate(cfg.vocab.tokens):
        if i and all(b >= 0x20 and b not in b'"\\' for b in t):
            assert c[i] == oracle.ACCEPTED
        if i and t.endswith(b'"') and t.count(b'"') == 1 and b"\\" not in t and all(b >= 0x20 for b in t):
            assert c[i] == oracle.ACCEPTED
        if i and len(t) >= 2 and t[0:1] == b'"' and b"\\" not in t[:1]:
            assert c[i] == oracle.UNCERTAIN
