"""xg2mask: MI355X-native token-mask cache for grammar-constrained decoding (HIP kernels behind a C ABI)."""
from .binding import (  # noqa: F401
    XG2_BF16, XG2_F32, CompileOpts, CompileStats, DeviceBatch, Grammar, MaskCache, Matcher, MatcherBatch, Pool, Vocab, Xg2Error, apply_token_bitmask,
    compile_grammar, fill_last_device_us, fill_last_recheck_tokens, fill_last_status, fill_next_token_bitmask, fill_next_token_bitmask_noalloc, fill_resolve_overflow, debug_set_large_capacity, debug_set_build_fusion, lib, LIB_PATH, EXPORTS,
)
