"""The fill entry point that allocates nothing, through the C ABI, against the ordinary one (and the oracle).

Collected last: the name sorts after the other test files.
"""
import random

import numpy as np
import pytest

import gen
import oracle
from helpers import diff_words, load

pytestmark = pytest.mark.gpu


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def test_fill_without_allocation_matches_the_ordinary_fill():
    """Nested-schema workload (V = 32,000): 64 matchers some tokens into their sentences.  Two calls in a row of the
    entry point that works in the library's fixed scratch array, the second on a smaller batch (20 other matchers, so
    the array still holds the first call's rows): each bitmask equals the ordinary entry point's, bit for bit, and
    sampled rows equal the oracle's plain-definition mask.  A batch beyond the stated maximum is refused."""
    import torch
    import paper_2601_04426_amd as xg
    assert torch.cuda.is_available()
    cfg, vocab, va = load(2)
    ebnf, root = cfg.grammars[0]
    W = vocab.words
    cache = xg.compile_grammar(vocab, ebnf, root, stream=_stream())
    orc = oracle.Oracle(ebnf, root)
    rng = random.Random(7007)
    seg = gen.Segmenter(cfg.vocab)
    B = 64
    traces, depth = gen.random_depth_traces(cfg, seg, B, rng)
    matchers = [xg.Matcher(cache) for _ in range(B)]
    hist = []
    for b in range(B):
        for t in traces[b][:depth[b]]:
            assert matchers[b].accept_token(t)
        hist.append(b"".join(cfg.vocab.tokens[t] for t in traces[b][:depth[b]]))
    dev = torch.device("cuda:0")
    for rows in (list(range(B)), [3, 5, 8, 13, 21, 34, 55] + list(range(40, 53))):
        ms = [matchers[b] for b in rows]
        want = torch.full((len(rows), W), -1, dtype=torch.int32, device=dev)
        got = torch.full((len(rows), W), 0x5A5A5A5A, dtype=torch.int32, device=dev)
        xg.fill_next_token_bitmask(ms, want.data_ptr(), W, _stream())
        torch.cuda.synchronize()
        xg.fill_next_token_bitmask_noalloc(ms, got.data_ptr(), W, _stream())
        torch.cuda.synchronize()
        assert not xg.fill_last_status()[1]
        got_h, want_h = got.cpu().numpy(), want.cpu().numpy()
        for i, b in enumerate(rows):
            assert np.array_equal(got_h[i], want_h[i]), (b, hist[b][-30:], diff_words(got_h[i], want_h[i], cfg.vocab.tokens))
        for i in range(0, len(rows), 5):
            plain = oracle.pack_bitmask(orc.mask(hist[rows[i]], va))
            assert np.array_equal(got_h[i], plain), (rows[i], diff_words(got_h[i], plain, cfg.vocab.tokens))
        # a decode step between the two calls: the second call sees other parser states than the first left behind
        for b in rows:
            t = traces[b][depth[b]]
            if t != cfg.vocab.eos_id:
                assert matchers[b].accept_token(t)
                hist[b] += cfg.vocab.tokens[t]
                depth[b] += 1
    # beyond the fixed scratch: 1,100 rows x 1,000 words > 2^20 mask words
    many = [xg.Matcher(cache) for _ in range(1100)]
    big = torch.zeros((1100, W), dtype=torch.int32, device=dev)
    with pytest.raises(xg.Xg2Error) as err:
        xg.fill_next_token_bitmask_noalloc(many, big.data_ptr(), W, _stream())
    assert err.value.code == -4 and "fixed scratch" in str(err.value)
    # a cache compiled just in time has planes that are not built: refused, nothing enqueued
    lazy = xg.compile_grammar(vocab, ebnf, root, stream=_stream(), jit=True, jit_prebuild=0)
    with pytest.raises(xg.Xg2Error) as err:
        xg.fill_next_token_bitmask_noalloc([xg.Matcher(lazy)], big.data_ptr(), W, _stream())
    assert err.value.code == -1
