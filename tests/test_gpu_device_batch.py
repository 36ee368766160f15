"""Matchers that live on the device: accept and fill without the host, against the oracle's plain-definition masks.

All calls go through the C ABI (ctypes binding).  Tolerance 0.
"""
import random

import numpy as np
import pytest

import gen
import oracle
from helpers import diff_words, load

pytestmark = pytest.mark.gpu

OK, EINVAL, EREJECTED, EOVERFLOW = 0, -1, -3, -4


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def run_batch_decode(xg, cfg, vocab, va, cache, orc, batch, steps, seed, check_every, depths=False):
    """`batch` slots follow seeded sentences token by token through the accept kernel; masks of sampled (row, step)
    pairs equal the oracle's; at every step one slot is offered a token its mask forbids (rejected, state unchanged);
    sentences end with the end-of-sequence token (slot terminated: end-of-sequence only) and restart with a reset."""
    import torch
    dev = torch.device("cuda:0")
    W = vocab.words
    rng = random.Random(seed)
    seg = gen.Segmenter(cfg.vocab)
    B = batch
    db = xg.DeviceBatch(vocab, B)
    db.assign(cache, stream=_stream())
    if depths:
        traces, cursor = gen.random_depth_traces(cfg, seg, B, rng)
    else:
        traces = [seg.segment(cfg.sample_text(rng, 0), rng) + [cfg.vocab.eos_id] for _ in range(B)]
        cursor = [0] * B
    ids = torch.zeros(B, dtype=torch.int32, device=dev)
    status = torch.full((B,), 99, dtype=torch.int32, device=dev)
    # advance to the starting depths, one accept launch per step
    for d in range(max(cursor) if depths else 0):
        ids.copy_(torch.tensor([traces[b][d] if d < cursor[b] else -1 for b in range(B)], dtype=torch.int32))
        db.accept_tokens(ids.data_ptr(), status.data_ptr(), _stream())
        assert not status.cpu().numpy().any(), ("advance", d)
    hist = [b"".join(cfg.vocab.tokens[t] for t in traces[b][:cursor[b]]) for b in range(B)]
    terminated = [False] * B
    bitmask = torch.full((B, W), -1, dtype=torch.int32, device=dev)
    n_checked = n_rejected = n_ended = 0
    for step in range(steps):
        db.fill_next_token_bitmask(bitmask.data_ptr(), W, _stream())
        torch.cuda.synchronize()
        assert not xg.fill_last_status()[1]
        got = bitmask.cpu().numpy()
        for b in range(B):
            if (step * B + b) % check_every:
                continue
            if terminated[b]:
                want = np.zeros(vocab.size, dtype=bool)
                want[cfg.vocab.eos_id] = True
            else:
                want = orc.mask(hist[b], va)
            want = oracle.pack_bitmask(want)
            assert np.array_equal(got[b], want), (step, b, hist[b][-40:], diff_words(got[b], want, cfg.vocab.tokens))
            n_checked += 1
        # a forbidden token for one live slot first: rejected, nothing changes
        live = [b for b in range(B) if not terminated[b]]
        if live:
            b = rng.choice(live)
            row = got[b].view(np.uint32)
            forbidden = next((t for t in rng.sample(range(1, vocab.size), 400) if not (int(row[t // 32]) >> (t % 32)) & 1), None)
            if forbidden is not None:                                # (free text of a dispatch grammar allows nearly everything)
                probe = np.full(B, -1, dtype=np.int32)
                probe[b] = forbidden
                ids.copy_(torch.from_numpy(probe))
                db.accept_tokens(ids.data_ptr(), status.data_ptr(), _stream())
                st = status.cpu().numpy()
                assert st[b] == EREJECTED and not np.delete(st, b).any()
                n_rejected += 1
        # then every slot's own next token (a terminated slot starts a new sentence)
        nxt = np.zeros(B, dtype=np.int32)
        for b in range(B):
            nxt[b] = -2 if terminated[b] else traces[b][cursor[b]]
        ids.copy_(torch.from_numpy(nxt))
        db.accept_tokens(ids.data_ptr(), status.data_ptr(), _stream())
        st = status.cpu().numpy()
        assert not st.any(), (step, np.nonzero(st)[0][:5], st[np.nonzero(st)[0][:5]])
        for b in range(B):
            if terminated[b]:
                terminated[b] = False
                traces[b] = seg.segment(cfg.sample_text(rng, 0), rng) + [cfg.vocab.eos_id]
                cursor[b] = 0
                hist[b] = b""
                continue
            tid = int(nxt[b])
            cursor[b] += 1
            if tid == cfg.vocab.eos_id:
                terminated[b] = True
                n_ended += 1
            else:
                hist[b] += cfg.vocab.tokens[tid]
    for b in range(0, B, max(1, B // 8)):
        info = db.row_info(b)
        assert info["error"] == 0 and info["terminated"] == int(terminated[b]) and info["cache"] == 0
    return n_checked, n_rejected, n_ended


@pytest.fixture(scope="module")
def xg():
    import torch
    assert torch.cuda.is_available()
    import paper_2601_04426_amd as xg
    return xg


def test_device_batch_tiny_json_every_mask(xg):
    cfg, vocab, va = load(1)
    ebnf, root = cfg.grammars[0]
    cache = xg.compile_grammar(vocab, ebnf, root, stream=_stream())
    orc = oracle.Oracle(ebnf, root)
    n, rej, ended = run_batch_decode(xg, cfg, vocab, va, cache, orc, batch=cfg.batch, steps=cfg.steps * 2, seed=101, check_every=1)
    assert n == cfg.batch * cfg.steps * 2 and rej > 100 and ended >= 2


def test_device_batch_nested_schema(xg):
    cfg, vocab, va = load(2)
    ebnf, root = cfg.grammars[0]
    cache = xg.compile_grammar(vocab, ebnf, root, stream=_stream())
    orc = oracle.Oracle(ebnf, root)
    n, rej, ended = run_batch_decode(xg, cfg, vocab, va, cache, orc, batch=64, steps=256, seed=102, check_every=3)
    assert n > 5000 and ended >= 10


def test_device_batch_tagdispatch(xg):
    cfg, vocab, va = load(3)
    ebnf, root = cfg.grammars[0]
    cache = xg.compile_grammar(vocab, ebnf, root, stream=_stream())
    orc = oracle.Oracle(ebnf, root)
    n, rej, ended = run_batch_decode(xg, cfg, vocab, va, cache, orc, batch=256, steps=96, seed=103, check_every=29)
    assert n > 800


def test_device_batch_repetition_stress_1024_at_random_depths(xg):
    """The benchmark's state through the device path: 1024 slots advanced to seeded random depths by the accept kernel,
    then 40 steps of fill and accept; one in 31 of the (row, step) masks against the plain definition."""
    cfg, vocab, va = load(5)
    ebnf, root = cfg.grammars[0]
    cache = xg.compile_grammar(vocab, ebnf, root, stream=_stream())
    orc = oracle.Oracle(ebnf, root)
    n, rej, ended = run_batch_decode(xg, cfg, vocab, va, cache, orc, batch=1024, steps=40, seed=105, check_every=31, depths=True)
    assert n > 1300 and rej >= 30


def test_device_batch_slots_of_different_grammars_and_errors(xg):
    import torch
    cfg, vocab, va = load(1)
    grammars = [cfg.grammars[0],
                ('root ::= "[" ws (num (ws "," ws num)*)? ws "]"\nnum ::= "-"? [0-9]{1,4}\nws ::= [ \t\n]*\n', "root"),
                ('root ::= item+\nitem ::= "<" [a-z]{1,8} ">" | [A-Z ]\n', "root")]
    caches = [xg.compile_grammar(vocab, e, r, stream=_stream()) for e, r in grammars]
    orcs = [oracle.Oracle(e, r) for e, r in grammars]
    rng = random.Random(606)
    B = 24
    which = [b % 3 for b in range(B)]
    db = xg.DeviceBatch(vocab, B)
    dev = torch.device("cuda:0")
    ids = torch.zeros(B, dtype=torch.int32, device=dev)
    status = torch.zeros(B, dtype=torch.int32, device=dev)
    bitmask = torch.zeros((B, vocab.words), dtype=torch.int32, device=dev)
    with pytest.raises(xg.Xg2Error):                                  # slots without a cache
        db.fill_next_token_bitmask(bitmask.data_ptr(), vocab.words, _stream())
    for g in range(3):
        db.assign(caches[g], rows=[b for b in range(B) if which[b] == g], stream=_stream())
    lazy = xg.compile_grammar(vocab, grammars[1][0], "root", stream=_stream(), jit=True, jit_prebuild=0)
    with pytest.raises(xg.Xg2Error):                                  # a cache compiled just in time has planes missing
        db.assign(lazy, rows=[0], stream=_stream())
    hist = [b""] * B
    done = [False] * B
    for step in range(24):
        db.fill_next_token_bitmask(bitmask.data_ptr(), vocab.words, _stream())
        torch.cuda.synchronize()
        got = bitmask.cpu().numpy()
        nxt = np.full(B, -1, dtype=np.int32)
        for b in range(B):
            if done[b]:
                want = np.zeros(vocab.size, dtype=bool)
                want[cfg.vocab.eos_id] = True
            else:
                want = orcs[which[b]].mask(hist[b], va)
                allowed = np.nonzero(want)[0]
                assert len(allowed) > 0
                nxt[b] = int(rng.choice(list(allowed)))
            assert np.array_equal(got[b], oracle.pack_bitmask(want)), (step, b, which[b], hist[b])
        ids.copy_(torch.from_numpy(nxt))
        db.accept_tokens(ids.data_ptr(), status.data_ptr(), _stream())
        assert not status.cpu().numpy().any()
        for b in range(B):
            if nxt[b] == cfg.vocab.eos_id:
                done[b] = True
            elif nxt[b] > 0:
                hist[b] += cfg.vocab.tokens[nxt[b]]
    # a terminated slot answers XG2_EINVAL to a further token; an id out of range too
    if any(done):
        b = done.index(True)
        probe = np.full(B, -1, dtype=np.int32)
        probe[b] = 5
        probe[(b + 1) % B] = vocab.size + 7
        ids.copy_(torch.from_numpy(probe))
        db.accept_tokens(ids.data_ptr(), status.data_ptr(), _stream())
        st = status.cpu().numpy()
        assert st[b] == EINVAL and st[(b + 1) % B] == EINVAL


def test_device_batch_slot_overflow_is_reported_not_masked(xg):
    """A right-recursive rule makes every token add a reachable item set: after 240 the slot's capacity is exceeded.
    The accept answers XG2_EOVERFLOW, the slot stays unusable (sticky) until it is reset, and up to that point every
    mask equals the oracle's."""
    import torch
    toks = [b"", b"x", b"y", b"xx"]
    vocab = xg.Vocab(toks, 0, [0])
    va = oracle.VocabArrays(toks, 0, [0])
    ebnf = 'root ::= a\na ::= "x" a | "y"\n'
    cache = xg.compile_grammar(vocab, ebnf, "root", stream=_stream())
    orc = oracle.Oracle(ebnf, "root")
    db = xg.DeviceBatch(vocab, 2)
    db.assign(cache, stream=_stream())
    dev = torch.device("cuda:0")
    ids = torch.tensor([1, -1], dtype=torch.int32, device=dev)
    status = torch.zeros(2, dtype=torch.int32, device=dev)
    bm = torch.zeros((2, 1), dtype=torch.int32, device=dev)
    hist = b""
    overflow_at = None
    for step in range(300):
        if step % 37 == 0:
            db.fill_next_token_bitmask(bm.data_ptr(), 1, _stream())
            torch.cuda.synchronize()
            assert np.array_equal(bm.cpu().numpy()[0], oracle.pack_bitmask(orc.mask(hist, va))), step
        db.accept_tokens(ids.data_ptr(), status.data_ptr(), _stream())
        st = status.cpu().numpy()
        if st[0] == EOVERFLOW:
            overflow_at = step
            break
        assert st[0] == OK
        hist += b"x"
    assert overflow_at is not None and 200 < overflow_at <= 245
    assert db.row_info(0)["error"] == 1 and db.row_info(1)["error"] == 0
    db.accept_tokens(ids.data_ptr(), status.data_ptr(), _stream())
    assert status.cpu().numpy()[0] == EOVERFLOW                       # sticky
    ids.copy_(torch.tensor([-2, -1], dtype=torch.int32))
    db.accept_tokens(ids.data_ptr(), status.data_ptr(), _stream())     # reset
    assert status.cpu().numpy()[0] == OK and db.row_info(0)["error"] == 0
    db.fill_next_token_bitmask(bm.data_ptr(), 1, _stream())
    torch.cuda.synchronize()
    assert np.array_equal(bm.cpu().numpy()[0], oracle.pack_bitmask(orc.mask(b"", va)))
