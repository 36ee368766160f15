"""Thin ctypes binding over libxg2mask.so: argument marshalling only.

Same names as the C ABI (include/xg2mask.h).  Device buffers are passed as integers
(`tensor.data_ptr()`), streams as `torch.cuda.current_stream().cuda_stream`.  Nothing here
computes a mask; if the library is missing the import fails loudly.
"""
from __future__ import annotations

import ctypes
import json
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libxg2mask.so")

XG2_OK, XG2_EINVAL, XG2_EPARSE, XG2_EREJECTED, XG2_EOVERFLOW, XG2_EHIP = 0, -1, -2, -3, -4, -5
XG2_F32, XG2_BF16 = 0, 1

EXPORTS = [
    "xg2_last_error", "xg2_vocab_create", "xg2_vocab_destroy", "xg2_grammar_create", "xg2_grammar_destroy",
    "xg2_grammar_describe", "xg2_grammar_num_positions", "xg2_pool_create", "xg2_pool_destroy", "xg2_pool_stats",
    "xg2_compile_grammar", "xg2_mask_cache_destroy", "xg2_mask_cache_stats", "xg2_mask_cache_num_positions", "xg2_mask_cache_num_planes", "xg2_mask_cache_jit_stats",
    "xg2_mask_cache_plane_info", "xg2_mask_cache_find_plane", "xg2_mask_cache_get_planes", "xg2_matcher_create", "xg2_matcher_create_host", "xg2_matcher_destroy",
    "xg2_matcher_accept_token", "xg2_matcher_accept_tokens", "xg2_matcher_reset", "xg2_matcher_is_terminated", "xg2_matcher_frontier",
    "xg2_fill_next_token_bitmask", "xg2_fill_next_token_bitmask_noalloc", "xg2_fill_resolve_overflow", "xg2_debug_set_large_capacity", "xg2_debug_set_build_fusion",
    "xg2_fill_last_device_us", "xg2_fill_last_status", "xg2_fill_last_recheck_tokens",
    "xg2_apply_token_bitmask", "xg2_batch_create", "xg2_batch_destroy", "xg2_batch_assign", "xg2_batch_accept_tokens",
    "xg2_batch_fill_next_token_bitmask", "xg2_batch_row_info",
]


class Xg2Error(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"xg2 error {code}: {msg}")
        self.code = code


class CompileStats(ctypes.Structure):
    _fields_ = [("positions", ctypes.c_int64), ("unique", ctypes.c_int64), ("built", ctypes.c_int64), ("partial_hits", ctypes.c_int64),
                ("checks", ctypes.c_int64), ("executed_checks", ctypes.c_int64), ("executed_token_bytes", ctypes.c_int64),
                ("slow_path", ctypes.c_int64),
                ("n_accepted", ctypes.c_int64), ("n_uncertain", ctypes.c_int64),
                ("host_lower_ms", ctypes.c_double), ("device_ms", ctypes.c_double), ("kernel_ms", ctypes.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class CompileOpts(ctypes.Structure):
    _fields_ = [("context_depth", ctypes.c_int32), ("merge_equivalent", ctypes.c_int32), ("follow_filter", ctypes.c_int32),
                ("jit", ctypes.c_int32), ("jit_prebuild", ctypes.c_int32), ("partial_hits", ctypes.c_int32), ("time_kernel", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    try:
        # PyTorch wheels ship their own HIP runtime; load it first so that the process has one runtime,
        # whichever of the two is imported first.
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2601_04426_amd/build.py` "
                          "(there is no fallback implementation)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    pvp = ctypes.POINTER(ctypes.c_void_p)
    L.xg2_last_error.restype = ctypes.c_char_p
    L.xg2_vocab_create.argtypes = [vp, vp, i32, i32, vp, i32, pvp]
    L.xg2_vocab_destroy.argtypes = [vp]
    L.xg2_grammar_create.argtypes = [ctypes.c_char_p, sz, ctypes.c_char_p, pvp]
    L.xg2_grammar_destroy.argtypes = [vp]
    L.xg2_grammar_describe.argtypes = [vp, ctypes.c_char_p, sz, ctypes.POINTER(sz)]
    L.xg2_grammar_num_positions.argtypes = [vp, ctypes.POINTER(i32)]
    L.xg2_pool_create.argtypes = [sz, pvp]
    L.xg2_pool_destroy.argtypes = [vp]
    L.xg2_pool_stats.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.xg2_compile_grammar.argtypes = [vp, ctypes.c_char_p, sz, ctypes.c_char_p, ctypes.POINTER(CompileOpts), vp, vp, pvp,
                                      ctypes.POINTER(CompileStats)]
    L.xg2_mask_cache_destroy.argtypes = [vp]
    L.xg2_mask_cache_stats.argtypes = [vp, ctypes.POINTER(CompileStats)]
    L.xg2_mask_cache_num_positions.argtypes = [vp, ctypes.POINTER(i32)]
    L.xg2_mask_cache_num_planes.argtypes = [vp, ctypes.POINTER(i32)]
    L.xg2_mask_cache_jit_stats.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_double)]
    L.xg2_mask_cache_plane_info.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(i32),
                                            ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(i32)]
    L.xg2_mask_cache_find_plane.argtypes = [vp, ctypes.c_char_p, i32, ctypes.c_char_p, i32, ctypes.POINTER(i32)]
    L.xg2_mask_cache_get_planes.argtypes = [vp, i32, vp, vp]
    L.xg2_matcher_create.argtypes = [vp, pvp]
    L.xg2_matcher_create_host.argtypes = [vp, vp, pvp]
    L.xg2_matcher_destroy.argtypes = [vp]
    L.xg2_matcher_accept_token.argtypes = [vp, i32]
    L.xg2_matcher_accept_tokens.argtypes = [vp, vp, i32, vp]
    L.xg2_matcher_reset.argtypes = [vp]
    L.xg2_matcher_is_terminated.argtypes = [vp, ctypes.POINTER(i32)]
    L.xg2_matcher_frontier.argtypes = [vp, vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.xg2_fill_next_token_bitmask.argtypes = [vp, i32, vp, i64, vp]
    L.xg2_fill_next_token_bitmask_noalloc.argtypes = [vp, i32, vp, i64, vp]
    L.xg2_fill_resolve_overflow.argtypes = [vp, i32, vp, i64, ctypes.POINTER(i32)]
    L.xg2_debug_set_large_capacity.argtypes = [i32, i32]
    L.xg2_debug_set_build_fusion.argtypes = [i32]
    L.xg2_fill_last_device_us.argtypes = [ctypes.POINTER(ctypes.c_float)]
    L.xg2_fill_last_status.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.xg2_fill_last_recheck_tokens.argtypes = [vp, i32, ctypes.POINTER(i32)]
    L.xg2_apply_token_bitmask.argtypes = [vp, i32, i32, i32, i64, vp, i64, vp]
    L.xg2_batch_create.argtypes = [vp, i32, pvp]
    L.xg2_batch_destroy.argtypes = [vp]
    L.xg2_batch_assign.argtypes = [vp, vp, i32, vp, vp]
    L.xg2_batch_accept_tokens.argtypes = [vp, vp, vp, vp]
    L.xg2_batch_fill_next_token_bitmask.argtypes = [vp, vp, i64, vp]
    L.xg2_batch_row_info.argtypes = [vp, i32, vp]
    for name in EXPORTS:
        if name not in ("xg2_last_error",) and not name.endswith("_destroy"):
            getattr(L, name).restype = i32
    return L


lib = _load()


def _check(code: int) -> None:
    if code != XG2_OK:
        raise Xg2Error(code, lib.xg2_last_error().decode("utf-8", "replace"))


class Vocab:
    def __init__(self, tokens: Sequence[bytes], eos_id: int, special_ids: Sequence[int] = ()):
        blob = b"".join(tokens)
        offs = np.zeros(len(tokens) + 1, dtype=np.uint64)
        np.cumsum([len(t) for t in tokens], out=offs[1:])
        buf = np.frombuffer(blob if blob else b"\0", dtype=np.uint8)
        sp = np.array(list(special_ids), dtype=np.int32)
        self.size = len(tokens)
        self.words = (self.size + 31) // 32
        self.eos_id = eos_id
        self.h = ctypes.c_void_p()
        _check(lib.xg2_vocab_create(buf.ctypes.data, offs.ctypes.data, len(tokens), eos_id,
                                    sp.ctypes.data if len(sp) else None, len(sp), ctypes.byref(self.h)))

    def __del__(self):
        if getattr(self, "h", None):
            lib.xg2_vocab_destroy(self.h)
            self.h = None


class Grammar:
    """Host-only lowering of an EBNF text (no device needed)."""

    def __init__(self, ebnf: str, root: str = "root"):
        data = ebnf.encode("utf-8")
        self.h = ctypes.c_void_p()
        _check(lib.xg2_grammar_create(data, len(data), root.encode(), ctypes.byref(self.h)))

    def describe(self) -> dict:
        need = ctypes.c_size_t(0)
        _check(lib.xg2_grammar_describe(self.h, None, 0, ctypes.byref(need)))
        buf = ctypes.create_string_buffer(need.value)
        _check(lib.xg2_grammar_describe(self.h, buf, need.value, ctypes.byref(need)))
        return json.loads(buf.value.decode("utf-8"))

    def num_positions(self) -> int:
        n = ctypes.c_int32(0)
        _check(lib.xg2_grammar_num_positions(self.h, ctypes.byref(n)))
        return n.value

    def __del__(self):
        if getattr(self, "h", None):
            lib.xg2_grammar_destroy(self.h)
            self.h = None


class Pool:
    def __init__(self, max_bytes: int = 0):
        self.h = ctypes.c_void_p()
        _check(lib.xg2_pool_create(max_bytes, ctypes.byref(self.h)))

    def stats(self) -> Tuple[int, int]:
        n, b = ctypes.c_int64(0), ctypes.c_int64(0)
        _check(lib.xg2_pool_stats(self.h, ctypes.byref(n), ctypes.byref(b)))
        return n.value, b.value

    def __del__(self):
        if getattr(self, "h", None):
            lib.xg2_pool_destroy(self.h)
            self.h = None


class MaskCache:
    def __init__(self, h, vocab: Vocab, stats: CompileStats, pool: Optional[Pool]):
        self.h, self.vocab, self.host_stats, self.pool = h, vocab, stats, pool
        self._stats = None

    @property
    def stats(self) -> CompileStats:
        """Full statistics of the compile call; the first access waits for the build (and raises if it failed)."""
        if self._stats is None:
            st = CompileStats()
            _check(lib.xg2_mask_cache_stats(self.h, ctypes.byref(st)))
            self._stats = st
        return self._stats

    def num_positions(self) -> int:
        n = ctypes.c_int32(0)
        _check(lib.xg2_mask_cache_num_positions(self.h, ctypes.byref(n)))
        return n.value

    def jit_stats(self) -> Tuple[int, int, float]:
        """(planes built so far, build launches issued by fill calls, their summed device time in ms)."""
        n, calls, ms = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_double(0)
        _check(lib.xg2_mask_cache_jit_stats(self.h, ctypes.byref(n), ctypes.byref(calls), ctypes.byref(ms)))
        return n.value, calls.value, ms.value

    def num_planes(self) -> int:
        n = ctypes.c_int32(0)
        _check(lib.xg2_mask_cache_num_planes(self.h, ctypes.byref(n)))
        return n.value

    def plane_info(self, k: int):
        """-> ((rule, state), parent) with parent = (rule, state) or None: the representative plane k was built for."""
        name, st, pname, pst = ctypes.c_char_p(), ctypes.c_int32(0), ctypes.c_char_p(), ctypes.c_int32(0)
        _check(lib.xg2_mask_cache_plane_info(self.h, k, ctypes.byref(name), ctypes.byref(st), ctypes.byref(pname), ctypes.byref(pst)))
        parent = (pname.value.decode(), pst.value) if pname.value is not None else None
        return (name.value.decode(), st.value), parent

    def find_plane(self, pos: Tuple[str, int], parent: Optional[Tuple[str, int]] = None) -> int:
        k = ctypes.c_int32(-1)
        _check(lib.xg2_mask_cache_find_plane(self.h, pos[0].encode(), pos[1], parent[0].encode() if parent else None,
                                             parent[1] if parent else -1, ctypes.byref(k)))
        return k.value

    def get_planes(self, k: int) -> Tuple[np.ndarray, np.ndarray]:
        acc = np.zeros(self.vocab.words, dtype=np.int32)
        unc = np.zeros(self.vocab.words, dtype=np.int32)
        _check(lib.xg2_mask_cache_get_planes(self.h, k, acc.ctypes.data, unc.ctypes.data))
        return acc, unc

    def __del__(self):
        if getattr(self, "h", None):
            lib.xg2_mask_cache_destroy(self.h)
            self.h = None


def compile_grammar(vocab: Vocab, ebnf: str, root: str = "root", pool: Optional[Pool] = None, stream: int = 0,
                    context_depth: int = 2, merge_equivalent: bool = True, follow_filter: bool = True,
                    jit: bool = False, jit_prebuild: int = 0, partial_hits: bool = True, time_kernel: bool = False) -> MaskCache:
    data = ebnf.encode("utf-8")
    h = ctypes.c_void_p()
    stats = CompileStats()
    opts = CompileOpts(context_depth, 1 if merge_equivalent else 0, 1 if follow_filter else 0, 1 if jit else 0, jit_prebuild, 1 if partial_hits else 0, 1 if time_kernel else 0)
    _check(lib.xg2_compile_grammar(vocab.h, data, len(data), root.encode(), ctypes.byref(opts), pool.h if pool else None,
                                   ctypes.c_void_p(stream), ctypes.byref(h), ctypes.byref(stats)))
    return MaskCache(h, vocab, stats, pool)


class Matcher:
    def __init__(self, cache: Optional[MaskCache] = None, grammar: Optional[Grammar] = None, vocab: Optional[Vocab] = None):
        self.h = ctypes.c_void_p()
        self._keep = (cache, grammar, vocab)
        if cache is not None:
            _check(lib.xg2_matcher_create(cache.h, ctypes.byref(self.h)))
        else:
            _check(lib.xg2_matcher_create_host(grammar.h, vocab.h, ctypes.byref(self.h)))

    def accept_token(self, token_id: int) -> bool:
        code = lib.xg2_matcher_accept_token(self.h, token_id)
        if code == XG2_EREJECTED:
            return False
        _check(code)
        return True

    def reset(self) -> None:
        _check(lib.xg2_matcher_reset(self.h))

    def is_terminated(self) -> bool:
        out = ctypes.c_int32(0)
        _check(lib.xg2_matcher_is_terminated(self.h, ctypes.byref(out)))
        return bool(out.value)

    def frontier(self) -> Tuple[List[int], bool]:
        cap = 256
        while True:
            buf = np.zeros(cap, dtype=np.int32)
            n, end = ctypes.c_int32(0), ctypes.c_int32(0)
            _check(lib.xg2_matcher_frontier(self.h, buf.ctypes.data, cap, ctypes.byref(n), ctypes.byref(end)))
            if n.value <= cap:
                return list(buf[:n.value]), bool(end.value)
            cap = n.value

    def __del__(self):
        if getattr(self, "h", None):
            lib.xg2_matcher_destroy(self.h)
            self.h = None


class MatcherBatch:
    """A fixed list of matchers with its handle array marshalled once."""

    def __init__(self, matchers: Sequence[Matcher]):
        self.matchers = list(matchers)
        self.arr = (ctypes.c_void_p * len(self.matchers))(*[m.h for m in self.matchers])

    def __len__(self):
        return len(self.matchers)

    def accept_tokens(self, token_ids) -> np.ndarray:
        """One token per matcher (negative = skip); returns the int32 status of every matcher."""
        ids = np.ascontiguousarray(token_ids, dtype=np.int32)
        if ids.shape != (len(self.matchers),):
            raise ValueError("one token id per matcher expected")
        status = np.zeros(len(self.matchers), dtype=np.int32)
        _check(lib.xg2_matcher_accept_tokens(self.arr, ids.ctypes.data, len(self.matchers), status.ctypes.data))
        return status


class DeviceBatch:
    """B matcher slots in device memory (argument marshalling only)."""

    def __init__(self, vocab: Vocab, batch: int):
        self.h = ctypes.c_void_p()
        self.vocab, self.batch, self._caches = vocab, batch, []
        _check(lib.xg2_batch_create(vocab.h, batch, ctypes.byref(self.h)))

    def assign(self, cache: "MaskCache", rows: Optional[Sequence[int]] = None, stream: int = 0) -> None:
        self._caches.append(cache)
        if rows is None:
            _check(lib.xg2_batch_assign(self.h, None, 0, cache.h, ctypes.c_void_p(stream)))
        else:
            arr = np.ascontiguousarray(rows, dtype=np.int32)
            _check(lib.xg2_batch_assign(self.h, arr.ctypes.data, len(arr), cache.h, ctypes.c_void_p(stream)))

    def accept_tokens(self, token_ids_ptr: int, status_ptr: int = 0, stream: int = 0) -> None:
        _check(lib.xg2_batch_accept_tokens(self.h, ctypes.c_void_p(token_ids_ptr), ctypes.c_void_p(status_ptr) if status_ptr else None,
                                           ctypes.c_void_p(stream)))

    def fill_next_token_bitmask(self, bitmask_ptr: int, row_stride_words: int, stream: int = 0) -> None:
        _check(lib.xg2_batch_fill_next_token_bitmask(self.h, ctypes.c_void_p(bitmask_ptr), row_stride_words, ctypes.c_void_p(stream)))

    def row_info(self, row: int) -> dict:
        out = np.zeros(8, dtype=np.int32)
        _check(lib.xg2_batch_row_info(self.h, row, out.ctypes.data))
        keys = ("can_end", "terminated", "error", "sets", "items", "wait_entries", "planes", "cache")
        return dict(zip(keys, (int(v) for v in out)))

    def __del__(self):
        if getattr(self, "h", None):
            lib.xg2_batch_destroy(self.h)
            self.h = None


def fill_next_token_bitmask(matchers, bitmask_ptr: int, row_stride_words: int, stream: int = 0) -> None:
    """matchers: a sequence of Matcher or a MatcherBatch."""
    if isinstance(matchers, MatcherBatch):
        arr = matchers.arr
    else:
        arr = (ctypes.c_void_p * len(matchers))(*[m.h for m in matchers])
    _check(lib.xg2_fill_next_token_bitmask(arr, len(matchers), ctypes.c_void_p(bitmask_ptr), row_stride_words,
                                           ctypes.c_void_p(stream)))


def fill_next_token_bitmask_noalloc(matchers, bitmask_ptr: int, row_stride_words: int, stream: int = 0) -> None:
    """The variant that allocates nothing (fixed device scratch, bounded batch)."""
    if isinstance(matchers, MatcherBatch):
        arr = matchers.arr
    else:
        arr = (ctypes.c_void_p * len(matchers))(*[m.h for m in matchers])
    _check(lib.xg2_fill_next_token_bitmask_noalloc(arr, len(matchers), ctypes.c_void_p(bitmask_ptr), row_stride_words,
                                                   ctypes.c_void_p(stream)))


def fill_resolve_overflow(matchers, bitmask_ptr: int, row_stride_words: int) -> int:
    """Decides on the host what the latest fill's large-capacity re-check left undecided; returns the number of pairs."""
    arr = matchers.arr if isinstance(matchers, MatcherBatch) else (ctypes.c_void_p * len(matchers))(*[m.h for m in matchers])
    n = ctypes.c_int32(0)
    _check(lib.xg2_fill_resolve_overflow(arr, len(matchers), ctypes.c_void_p(bitmask_ptr), row_stride_words, ctypes.byref(n)))
    return n.value


def debug_set_build_fusion(on: bool = True) -> None:
    _check(lib.xg2_debug_set_build_fusion(1 if on else 0))


def debug_set_large_capacity(items: int = 0, wait_entries: int = 0) -> None:
    _check(lib.xg2_debug_set_large_capacity(items, wait_entries))


def fill_last_status() -> Tuple[int, bool]:
    """(pairs re-checked by the large-capacity kernel, whether one of them overflowed even that) of the latest fill."""
    n, over = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib.xg2_fill_last_status(ctypes.byref(n), ctypes.byref(over)))
    return n.value, bool(over.value)


def fill_last_recheck_tokens(batch: int) -> np.ndarray:
    """Per row of the latest fill: how many candidate tokens went through the full-context re-check."""
    out = np.zeros(batch, dtype=np.int32)
    n = ctypes.c_int32(0)
    _check(lib.xg2_fill_last_recheck_tokens(out.ctypes.data, batch, ctypes.byref(n)))
    return out[:min(batch, n.value)]


def fill_last_device_us() -> float:
    out = ctypes.c_float(0)
    _check(lib.xg2_fill_last_device_us(ctypes.byref(out)))
    return out.value


def apply_token_bitmask(logits_ptr: int, dtype: int, B: int, V: int, row_stride_elems: int, bitmask_ptr: int,
                        bm_row_stride_words: int, stream: int = 0) -> None:
    _check(lib.xg2_apply_token_bitmask(ctypes.c_void_p(logits_ptr), dtype, B, V, row_stride_elems,
                                       ctypes.c_void_p(bitmask_ptr), bm_row_stride_words, ctypes.c_void_p(stream)))
