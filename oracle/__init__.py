"""CPU ORACLE -- test infrastructure only.

Slow, plain reference for what the token-mask cache path computes.  Only `tests/`, the
smoke check and the CPU-baseline leg of the benchmark may import this package; the library
under `paper_2601_04426_amd/` never does, and this package imports nothing from it.

What it defines (paper sections 2.1, 3.2, 3.4 and the appendices on the adaptive token mask
cache and on Earley parsing):

  Oracle.mask(history)      next-token mask by the plain definition: token t is allowed iff
                            history.bytes(t) is a prefix of a sentence of the grammar; the
                            end-of-sequence token iff history is a sentence; other special
                            tokens and empty tokens never.
  Oracle.classes(position)  accepted / uncertain / rejected sets of one cache position
                            (rule, canonical FSM state): accepted iff t is a prefix of a string
                            of the position's suffix language, else uncertain iff a proper
                            non-empty prefix of t is a complete string of it, else rejected.
  Oracle.frontier(history)  scannable positions of the closed Earley set after history.
  pack_bitmask / apply_*    bit v%32 of int32 word v/32 (1 = allowed); masked logits = -inf.

Parity status: every function here is pinned by tests/test_oracle_*.py (brute-force
enumeration, closed forms, library routines, invariants); nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import bnf as _bnf
from . import fsm as _fsm
from .ebnf import EBNFError, parse_ebnf   # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libearley_oracle.so")
_lib = None

REJECTED, ACCEPTED, UNCERTAIN = 0, 1, 2


def build_c(force: bool = False) -> str:
    src = os.path.join(_HERE, "earley.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build_c()
        L = ctypes.CDLL(_LIB_PATH)
        L.eo_grammar_new.restype = ctypes.c_void_p
        L.eo_grammar_new.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
        L.eo_grammar_free.argtypes = [ctypes.c_void_p]
        L.eo_productive.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        L.eo_is_nullable.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        L.eo_scan_vocab.restype = ctypes.c_int32
        L.eo_scan_vocab.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32]
        L.eo_accepts.restype = ctypes.c_int32
        L.eo_accepts.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64]
        L.eo_apply_f32.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                   ctypes.c_void_p, ctypes.c_int64]
        L.eo_apply_bf16.argtypes = L.eo_apply_f32.argtypes
        _lib = L
    return _lib


class CGrammar:
    """A BNF handed to the C recogniser."""

    def __init__(self, b: _bnf.BNF):
        L = _load()
        self.bnf = b
        lhs = np.array([p[0] for p in b.prods], dtype=np.int32)
        off = np.zeros(len(b.prods) + 1, dtype=np.int32)
        syms: List[int] = []
        for i, (_, rhs) in enumerate(b.prods):
            syms.extend(rhs)
            off[i + 1] = len(syms)
        syms_a = np.array(syms if syms else [0], dtype=np.int32)
        ts = np.zeros((max(1, len(b.tsets)), 8), dtype=np.uint32)
        for i, m in enumerate(b.tsets):
            for w in range(8):
                ts[i, w] = (m >> (32 * w)) & 0xFFFFFFFF
        self._keep = (lhs, off, syms_a, ts)
        self.h = L.eo_grammar_new(b.n_nt, len(b.prods), lhs.ctypes.data, off.ctypes.data, syms_a.ctypes.data,
                                  len(b.tsets), ts.ctypes.data)
        self.prod_lhs = lhs
        self.prod_off = off
        self.prod_syms = syms_a

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.eo_grammar_free(self.h)
            self.h = None

    def productive(self) -> np.ndarray:
        out = np.zeros(self.bnf.n_nt, dtype=np.uint8)
        _load().eo_productive(self.h, out.ctypes.data)
        return out

    def accepts(self, start_nt: int, text: bytes) -> bool:
        buf = np.frombuffer(text, dtype=np.uint8) if text else np.zeros(1, dtype=np.uint8)
        return bool(_load().eo_accepts(self.h, start_nt, buf.ctypes.data, len(text)))

    def scan_vocab(self, start_nt: int, history: bytes, blob: np.ndarray, offs: np.ndarray, threads: int = 0,
                   want_items: bool = False, start2_nt: int = -1, follow_nt: int = -1):
        """-> (status, viable[V] u8, early[V] u8, items or None); status -1 dead, 1 complete, 0 otherwise."""
        V = len(offs) - 1
        viable = np.zeros(V, dtype=np.uint8)
        early = np.zeros(V, dtype=np.uint8)
        hist = np.frombuffer(history, dtype=np.uint8) if history else np.zeros(1, dtype=np.uint8)
        cap = 4096
        items = np.zeros(3 * cap, dtype=np.int32)
        n_items = ctypes.c_int32(0)
        st = _load().eo_scan_vocab(self.h, start_nt, start2_nt, follow_nt, hist.ctypes.data, len(history), blob.ctypes.data,
                                   offs.ctypes.data, V, viable.ctypes.data, early.ctypes.data,
                                   items.ctypes.data, cap, ctypes.byref(n_items), threads)
        it = None
        if want_items and st >= 0:
            if n_items.value > cap:
                raise RuntimeError("item export buffer too small")
            it = items[:3 * n_items.value].reshape(-1, 3).copy()
        return st, viable, early, it


class VocabArrays:
    """Vocabulary as the C recogniser wants it (token-id order, nothing sorted)."""

    def __init__(self, tokens: Sequence[bytes], eos_id: int, special_ids: Sequence[int]):
        self.tokens = list(tokens)
        self.eos_id = eos_id
        self.special = np.zeros(len(tokens), dtype=bool)
        for s in special_ids:
            self.special[s] = True
        self.special[eos_id] = True
        blob = b"".join(self.tokens)
        self.blob = np.frombuffer(blob if blob else b"\0", dtype=np.uint8).copy()
        offs = np.zeros(len(tokens) + 1, dtype=np.int64)
        np.cumsum([len(t) for t in self.tokens], out=offs[1:])
        self.offs = offs
        self.V = len(tokens)


class Oracle:
    def __init__(self, ebnf_text: str, root: str = "root", check_reduced: bool = True):
        self.order, self.rules = parse_ebnf(ebnf_text)
        self.root = root
        self.low = _fsm.Lowered(self.order, self.rules, root)
        self.fsm_bnf = _bnf.fsm_bnf(self.low)
        _bnf.add_follow(self.fsm_bnf, self.low)
        self.cg = CGrammar(self.fsm_bnf)
        self.root_nt = self.fsm_bnf.names[(root, 0)]
        self._nt_key = {v: k for k, v in self.fsm_bnf.names.items()}
        if check_reduced:
            prod = self.cg.productive()
            bad = [self._nt_key[i] for i in range(self.fsm_bnf.n_nt) if not prod[i]]
            if bad:
                raise ValueError(f"grammar is not reduced; unproductive: {bad[:5]}")
        self._direct: Optional[CGrammar] = None

    # -- positions -------------------------------------------------------------------------
    def positions(self) -> List[Tuple[str, int]]:
        return self.low.positions()

    # -- plain definition of the next-token mask --------------------------------------------
    def mask(self, history: bytes, vocab: VocabArrays, threads: int = 0, direct: bool = False) -> np.ndarray:
        """bool[V]; raises if history is not a viable prefix."""
        cg, start = (self.direct(), self._direct_root) if direct else (self.cg, self.root_nt)
        st, viable, _, _ = cg.scan_vocab(start, history, vocab.blob, vocab.offs, threads)
        if st < 0:
            raise ValueError("history is not a viable prefix of the grammar")
        m = viable.astype(bool)
        m[vocab.special] = False
        m[vocab.eos_id] = (st == 1)
        return m

    def accepts(self, text: bytes, direct: bool = False) -> bool:
        if direct:
            return self.direct().accepts(self._direct_root, text)
        return self.cg.accepts(self.root_nt, text)

    def direct(self) -> CGrammar:
        if self._direct is None:
            b = _bnf.direct_bnf(self.order, self.rules, self.root)
            self._direct = CGrammar(b)
            self._direct_root = b.names[("rule", self.root)]
        return self._direct

    # -- cache classes of one position ------------------------------------------------------
    def classes(self, pos: Tuple[str, int], vocab: VocabArrays, threads: int = 0,
                parent: Optional[Tuple[str, int]] = None, follow: bool = False) -> np.ndarray:
        """u8[V]: ACCEPTED / UNCERTAIN / REJECTED; special and empty tokens are REJECTED.
        With `parent` = the state the referencing rule continues in once this rule instance ends, the
        suffix language is Suf(pos) . Suf(parent) (one level of context).
        With `follow`, a token that leaves the (outermost) rule after t[0:i] stays uncertain only if the
        rest t[i:] is a viable prefix of what can follow that rule somewhere in the grammar (the follow
        language: the union over the rule's reference sites of Suf(site) . follow(site's rule); the root
        rule may also be followed by nothing); otherwise no context can accept it and it is REJECTED."""
        start = self.fsm_bnf.names[pos]
        start2 = self.fsm_bnf.names[parent] if parent is not None else -1
        outer = parent[0] if parent is not None else pos[0]
        fnt = self.fsm_bnf.names[("follow", outer)] if follow else -1
        st, viable, early, _ = self.cg.scan_vocab(start, b"", vocab.blob, vocab.offs, threads, start2_nt=start2, follow_nt=fnt)
        assert st >= 0
        cls = np.where(viable.astype(bool), ACCEPTED, np.where(early.astype(bool), UNCERTAIN, REJECTED)).astype(np.uint8)
        cls[vocab.special] = REJECTED
        return cls

    # -- scannable frontier -----------------------------------------------------------------
    def frontier(self, history: bytes, vocab: Optional[VocabArrays] = None) -> List[Tuple[str, int]]:
        """Positions (rule, state) of the items of the closed Earley set after `history` whose
        next symbol is a terminal."""
        empty_blob = np.zeros(1, dtype=np.uint8)
        empty_offs = np.zeros(1, dtype=np.int64)
        st, _, _, items = self.cg.scan_vocab(self.root_nt, history, empty_blob, empty_offs, 1, want_items=True)
        if st < 0:
            raise ValueError("history is not a viable prefix of the grammar")
        out = set()
        n_prod = len(self.fsm_bnf.prods)
        for prod, dot, _ in items:
            if prod == n_prod:
                continue
            lhs, rhs = self.fsm_bnf.prods[prod]
            if dot < len(rhs) and rhs[dot] >= 0:
                out.add(self._nt_key[lhs])
        return sorted(out)


def pack_bitmask(mask: np.ndarray) -> np.ndarray:
    """bool[V] -> int32[ceil(V/32)], bit v%32 of word v/32, pad bits 0."""
    V = mask.shape[-1]
    W = (V + 31) // 32
    words = np.zeros(W, dtype=np.uint32)
    idx = np.nonzero(mask)[0]
    np.bitwise_or.at(words, idx // 32, (np.uint32(1) << (idx % 32).astype(np.uint32)))
    return words.view(np.int32)


def apply_f32(logits_bits: np.ndarray, bitmask: np.ndarray) -> None:
    """In place on the uint32 view of fp32 logits [B, V]; bitmask int32 [B, W]."""
    assert logits_bits.dtype == np.uint32 and bitmask.dtype == np.int32
    B, V = logits_bits.shape
    _load().eo_apply_f32(logits_bits.ctypes.data, B, V, logits_bits.strides[0] // 4, bitmask.ctypes.data,
                         bitmask.strides[0] // 4)


def apply_bf16(logits_bits: np.ndarray, bitmask: np.ndarray) -> None:
    """In place on the uint16 view of bf16 logits [B, V]; bitmask int32 [B, W]."""
    assert logits_bits.dtype == np.uint16 and bitmask.dtype == np.int32
    B, V = logits_bits.shape
    _load().eo_apply_bf16(logits_bits.ctypes.data, B, V, logits_bits.strides[0] // 2, bitmask.ctypes.data,
                          bitmask.strides[0] // 4)
