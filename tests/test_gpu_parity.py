"""GPU parity: every plane, bitmask and masked logit equal to the CPU oracle's, bit for bit.

All calls go through the C ABI (ctypes binding).  Tolerance 0.
"""
import random

import numpy as np
import pytest

import gen
import oracle
from helpers import diff_words, load, planes_of

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xg():
    import torch
    assert torch.cuda.is_available()
    import paper_2601_04426_amd as xg
    return xg


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def check_planes(xg, cfg, vocab, va, ebnf, root, positions=None, pool=None):
    cache = xg.compile_grammar(vocab, ebnf, root, pool=pool, stream=_stream())
    orc = oracle.Oracle(ebnf, root)
    n = cache.num_positions()
    assert sorted(cache.position(p) for p in range(n)) == sorted(orc.positions())
    todo = range(n) if positions is None else positions
    for p in todo:
        acc, unc = cache.get_planes(p)
        want_a, want_u = planes_of(orc, cache.position(p), va)
        assert np.array_equal(acc, want_a), ("accepted", cache.position(p), diff_words(acc, want_a, cfg.vocab.tokens))
        assert np.array_equal(unc, want_u), ("uncertain", cache.position(p), diff_words(unc, want_u, cfg.vocab.tokens))
    return cache, orc


def run_decode(xg, cfg, vocab, va, cache, orc, batch, steps, seed, check_every=1):
    import torch
    dev = torch.device("cuda:0")
    W = vocab.words
    rng = random.Random(seed)
    seg = gen.Segmenter(cfg.vocab)
    matchers = [xg.Matcher(cache) for _ in range(batch)]
    traces = [seg.segment(cfg.sample_text(rng, 0), rng) + [cfg.vocab.eos_id] for _ in range(batch)]
    cursor = [0] * batch
    hist = [b""] * batch
    bitmask = torch.full((batch, W), -1, dtype=torch.int32, device=dev)
    n_checked = 0
    for step in range(steps):
        xg.fill_next_token_bitmask(matchers, bitmask.data_ptr(), W, _stream())
        torch.cuda.synchronize()
        got = bitmask.cpu().numpy()
        for b in range(batch):
            if (step * batch + b) % check_every == 0:
                if matchers[b].is_terminated():
                    want = np.zeros(vocab.size, dtype=bool)
                    want[cfg.vocab.eos_id] = True
                else:
                    want = orc.mask(hist[b], va)
                want = oracle.pack_bitmask(want)
                assert np.array_equal(got[b], want), (step, b, hist[b][-40:], diff_words(got[b], want, cfg.vocab.tokens))
                n_checked += 1
            if matchers[b].is_terminated():
                matchers[b].reset()
                traces[b] = seg.segment(cfg.sample_text(rng, 0), rng) + [cfg.vocab.eos_id]
                cursor[b] = 0
                hist[b] = b""
                continue
            tid = traces[b][cursor[b]]
            assert (int(got[b][tid // 32]) >> (tid % 32)) & 1, "the trace's own next token must be allowed"
            assert matchers[b].accept_token(tid)
            cursor[b] += 1
            if tid != cfg.vocab.eos_id:
                hist[b] += cfg.vocab.tokens[tid]
    return n_checked


def test_config1_planes_and_decode(xg):
    cfg, vocab, va = load(1)
    ebnf, root = cfg.grammars[0]
    cache, orc = check_planes(xg, cfg, vocab, va, ebnf, root)
    st = cache.stats
    assert st.positions == len(orc.positions()) and st.built == st.unique <= st.positions
    assert st.checks == st.built * (cfg.vocab.size - 1)
    n = run_decode(xg, cfg, vocab, va, cache, orc, batch=cfg.batch, steps=cfg.steps, seed=11)
    assert n == cfg.batch * cfg.steps


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,V,pad", [(2, 2048, 0), (3, 1000, 24), (1, 37, 3), (4, 151936, 0), (2, 4099, 5)])
def test_apply_matches_oracle(xg, dtype, B, V, pad):
    import torch
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(B * 1000 + V)
    stride = V + pad
    W = (V + 31) // 32
    if dtype == "f32":
        bits = rng.integers(0, 2 ** 32, size=(B, stride), dtype=np.uint64).astype(np.uint32)
        bits[0, :6] = [0x7FC00001, 0xFFC12345, 0x80000000, 0x7F800000, 0xFF800000, 0x00000001]
        t = torch.from_numpy(bits.view(np.int32)).to(dev)
    else:
        bits = rng.integers(0, 2 ** 16, size=(B, stride), dtype=np.uint64).astype(np.uint16)
        bits[0, :6] = [0x7FC1, 0xFFC1, 0x8000, 0x7F80, 0xFF80, 0x0001]
        t = torch.from_numpy(bits.view(np.int16)).to(dev)
    density = [0.0, 1.0, 0.5, 0.02, 0.98]
    allow = np.stack([rng.random(V) < density[b % len(density)] for b in range(B)])
    bm = np.stack([oracle.pack_bitmask(allow[b]) for b in range(B)])
    bm_t = torch.from_numpy(bm).to(dev)
    xg.apply_token_bitmask(t.data_ptr(), xg.XG2_F32 if dtype == "f32" else xg.XG2_BF16, B, V, stride, bm_t.data_ptr(), W, _stream())
    torch.cuda.synchronize()
    want = bits.copy()
    if dtype == "f32":
        oracle.apply_f32(want[:, :V], bm)
        got = t.cpu().numpy().view(np.uint32)
    else:
        oracle.apply_bf16(want[:, :V], bm)
        got = t.cpu().numpy().view(np.uint16)
    assert np.array_equal(got, want)          # also: the padding between rows is untouched


def test_apply_unaligned_base(xg):
    import torch
    dev = torch.device("cuda:0")
    V, B = 777, 2
    base = torch.randn(B * V + 8, dtype=torch.float32, device=dev)
    view = base[1:1 + B * V].view(B, V)            # 4-byte aligned only
    before = view.cpu().numpy().view(np.uint32).copy()
    allow = np.random.default_rng(1).random((B, V)) < 0.4
    bm = np.stack([oracle.pack_bitmask(allow[b]) for b in range(B)])
    bm_t = torch.from_numpy(bm).to(dev)
    xg.apply_token_bitmask(view.data_ptr(), xg.XG2_F32, B, V, V, bm_t.data_ptr(), bm.shape[1], _stream())
    torch.cuda.synchronize()
    oracle.apply_f32(before, bm)
    assert np.array_equal(view.cpu().numpy().view(np.uint32), before)
