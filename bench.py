#!/usr/bin/env python3
"""Benchmark of the token-mask cache hot path on one MI355X.

A step is one pass of the whole path over one batch of the "runtime stress" workload
(V = 151,936, 1024 concurrent matchers): build the mask cache of the grammar (every position x
every token), fill the batch's next-token bitmask (cached planes + re-check of uncertain tokens),
apply it to bf16 logits and to fp32 logits, then advance every matcher by one token on the host.

Prints ONE JSON line.  `value` = (position, token) checks per second of the cache build, from the
build's device time (HIP events inside the library: clearing of the rows and table upload to last
plane written); the fill+apply microseconds per step, the host times and the wall-clock per step are
given beside it.  `roofline` counts only the pairs a lane actually stepped through (tokens skipped by
their first byte or copied from another plane move no bytes and are not counted).  After the timed
steps, one cache build of the TagDispatch workload (config 3, a millisecond-scale launch of the same
kernel) is measured the same way and reported under `build_tagdispatch`.
"""
from __future__ import annotations

import argparse
import json
import os
import random
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (counter values per dispatch, default workload and
# batch; k_build_tagdispatch: the one build of the TagDispatch workload), valid only for the kernel sources they were taken
# with.  The same counters read 303,890 (FETCH_SIZE) and 607,744 (WRITE_SIZE) for a device-to-device copy of 607,744 KiB,
# hence the scale factors to KiB.  The summaries under profiles/ hold the commands and the full tables.
PMC = {
    "sources_sha256": "236e9418d43ccc896bf41a1fa618f043c5f6b0f15c010edf8f2233fc1ca770e9",
    "fetch_scale": 2.00, "write_scale": 1.00,
    "k_build": (11030.4, 4800.5),
    "k_fill": (3308.2, 19191.9),
    "k_apply_vec<8>": (97590.3, 303872.0),
    "k_apply_vec<4>": (180438.0, 605533.3),
    "k_build_tagdispatch": (144657.9, 689897.5),
    # wave instructions of one k_build launch (rocprofv3 --pmc SQ_INSTS_VALU; SQ_INSTS_SALU + SQ_INSTS_SMEM + SQ_INSTS_BRANCH)
    "k_build_valu_instructions": 12898560.0, "k_build_scalar_and_branch_instructions": 17288610.0,
    "k_build_tagdispatch_valu_instructions": 848041696.0, "k_build_tagdispatch_scalar_and_branch_instructions": 1115408341.0,
}
KERNEL_SOURCES = ("csrc/kernels.hip", "csrc/earley_core.hpp", "csrc/device.hpp", "build.py")   # code and compiler flags


def kernel_sources_sha256() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2601_04426_amd", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(kernel: str, default_workload: bool):
    """Bytes per launch, or None when the kernels or the workload differ from what the counters were taken on."""
    if not default_workload or kernel not in PMC or kernel_sources_sha256() != PMC["sources_sha256"]:
        return None
    fetch_kib, write_kib = PMC[kernel]
    return (fetch_kib * PMC["fetch_scale"] + write_kib * PMC["write_scale"]) * 1024.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload index (5 = runtime stress, the metric's configuration)")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-host-matchers", action="store_true", help="skip the comparison leg with the parsers on the host")
    ap.add_argument("--no-tagdispatch-build", action="store_true", help="skip the one build of the TagDispatch workload after the timed steps")
    ap.add_argument("--cross-grammar", type=int, default=0, metavar="N",
                    help="also compile the first N grammars of the cross-grammar workload (config 4; 256 = all) into one pool and "
                         "report planes built once versus positions, and checks/s (adds build launches of other sizes)")
    ap.add_argument("--no-jit", action="store_true", help="skip the just-in-time leg (128 decode steps on a cache compiled just in time and on the "
                                                          "fully built one: per-step fill latency median / P99 / max)")
    ap.add_argument("--build-only", action="store_true",
                    help="time cache builds of --config only (steps = builds; no decode, no oracle): the command the build kernel's profiles are taken with")
    ap.add_argument("--cpu-positions", type=int, default=4096, help="positions in the oracle's timed sample")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU; --gpus above 1 is not supported (no sharding, no collectives)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import gen
    import paper_2601_04426_amd as xg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream().cuda_stream

    cfg = gen.build_config(args.config)
    ebnf, root = cfg.grammars[0]
    B = args.batch or cfg.batch or 256
    V = cfg.vocab.size
    vocab = xg.Vocab(cfg.vocab.tokens, cfg.vocab.eos_id, cfg.vocab.special_ids)
    W = vocab.words
    n_checkable = sum(1 for i, t in enumerate(cfg.vocab.tokens) if t and i not in cfg.vocab.special_ids)
    tok_bytes = sum(len(t) for i, t in enumerate(cfg.vocab.tokens) if t and i not in cfg.vocab.special_ids)

    if args.build_only:
        def roof(stats, k_ms):
            b = int(stats.executed_token_bytes) + 4.25 * int(stats.executed_checks)
            return {"kernel": "k_build", "bound": "hbm", "achieved": b / (k_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": b / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None, "algorithmic_bytes_per_launch": b}
        ks, ds, hs = [], [], []
        t_begin = None
        for it in range(args.warmup + args.steps):
            if it == args.warmup:
                torch.cuda.synchronize()
                t_begin = time.perf_counter()
            c = xg.compile_grammar(vocab, ebnf, root, stream=stream)
            st = c.stats
            if it >= args.warmup:
                ds.append(st.device_ms); hs.append(st.host_lower_ms)
            del c
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_begin
        for it in range(args.steps):                                 # the same builds with events around the classification kernel
            c = xg.compile_grammar(vocab, ebnf, root, stream=stream, time_kernel=True)
            ks.append(c.stats.kernel_ms)
            del c
        k_ms, d_ms = sum(ks) / len(ks), sum(ds) / len(ds)
        print(json.dumps({"metric": "mask-cache build (position x token) checks/s", "value": int(st.checks) / (d_ms * 1e-3), "unit": "checks/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True,
                          "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
                          "config": {"workload": cfg.name + " (cache builds only)", "config_index": cfg.index, "vocab": V, "positions": int(st.positions),
                                     "built_positions": int(st.built), "checks_per_build": int(st.checks), "executed_checks": int(st.executed_checks)},
                          "build": {"device_ms": d_ms, "kernel_ms": k_ms, "host_lower_ms": sum(hs) / len(hs),
                                    "executed_pairs_per_s": int(st.executed_checks) / (k_ms * 1e-3)},
                          "roofline": roof(st, k_ms)}))
        return 0

    # matchers at random depths of their own sentences (set-up, untimed): B slots in device memory, advanced by the accept kernel
    cache0 = xg.compile_grammar(vocab, ebnf, root, stream=stream)
    rng = random.Random(gen.BASE_SEED + 100 + args.config)
    seg = gen.Segmenter(cfg.vocab)
    traces, cursor = gen.random_depth_traces(cfg, seg, B, rng)
    db = xg.DeviceBatch(vocab, B)
    db.assign(cache0, stream=stream)
    ids_host = torch.zeros(B, dtype=torch.int32).pin_memory()
    ids_dev = torch.zeros(B, dtype=torch.int32, device=dev)
    status_dev = torch.zeros(B, dtype=torch.int32, device=dev)
    ids_np = ids_host.numpy()
    for d in range(max(cursor)):
        for b in range(B):
            ids_np[b] = traces[b][d] if d < cursor[b] else -1
        ids_dev.copy_(ids_host)
        db.accept_tokens(ids_dev.data_ptr(), status_dev.data_ptr(), stream)
    assert not status_dev.cpu().numpy().any(), "a trace token was rejected during set-up"
    ended = [False] * B

    g = torch.Generator(device="cpu").manual_seed(1234)
    logits32_src = torch.randn((B, V), generator=g, dtype=torch.float32).to(dev)
    logits16_src = logits32_src.to(torch.bfloat16)
    logits32 = torch.empty_like(logits32_src)
    logits16 = torch.empty_like(logits16_src)
    bitmask = torch.zeros((B, W), dtype=torch.int32, device=dev)

    def next_tokens():
        # what the sampler would hand over: here the next token of each slot's own sentence; a slot whose sentence has
        # ended starts a fresh one (-2)
        for b in range(B):
            if ended[b]:
                ids_np[b] = -2
                traces[b] = seg.segment(cfg.sample_text(rng, 0), rng) + [cfg.vocab.eos_id]
                cursor[b] = 0
                ended[b] = False
            else:
                ids_np[b] = traces[b][cursor[b]]
                cursor[b] += 1
                ended[b] = cursor[b] >= len(traces[b])              # the end-of-sequence token goes in now

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    acc = {"build_device_ms": [], "build_kernel_ms": [], "build_host_ms": [], "fill_us": [], "apply_bf16_us": [],
           "apply_f32_us": [], "fill_device_us": [], "fill_call_ms": [], "accept_call_ms": [], "accept_us": []}
    last_stats = None

    def step(record: bool):
        nonlocal last_stats
        # logits of this step (untimed refresh: apply works in place)
        logits16.copy_(logits16_src)
        logits32.copy_(logits32_src)
        cache = xg.compile_grammar(vocab, ebnf, root, stream=stream)          # a2: builds every position afresh
        st = cache.stats
        t0 = time.perf_counter()
        ev[0].record()
        db.fill_next_token_bitmask(bitmask.data_ptr(), W, stream)             # a3 + a4, nothing uploaded
        t1 = time.perf_counter()
        ev[1].record()
        xg.apply_token_bitmask(logits16.data_ptr(), xg.XG2_BF16, B, V, V, bitmask.data_ptr(), W, stream)   # a5
        ev[2].record()
        xg.apply_token_bitmask(logits32.data_ptr(), xg.XG2_F32, B, V, V, bitmask.data_ptr(), W, stream)
        ev[3].record()
        next_tokens()
        ids_dev.copy_(ids_host, non_blocking=True)
        t2 = time.perf_counter()
        ev[4].record()
        db.accept_tokens(ids_dev.data_ptr(), status_dev.data_ptr(), stream)   # a6, on the device
        ev[5].record()
        t3 = time.perf_counter()
        ev[5].synchronize()
        assert not status_dev.cpu().numpy().any(), "a trace token was rejected"
        fill_dev_us = xg.fill_last_device_us()
        if record:
            last_stats = st
            acc["fill_device_us"].append(fill_dev_us)
            acc["build_device_ms"].append(st.device_ms)
            acc["build_host_ms"].append(st.host_lower_ms)
            acc["fill_us"].append(ev[0].elapsed_time(ev[1]) * 1e3)
            acc["apply_bf16_us"].append(ev[1].elapsed_time(ev[2]) * 1e3)
            acc["apply_f32_us"].append(ev[2].elapsed_time(ev[3]) * 1e3)
            acc["accept_us"].append(ev[4].elapsed_time(ev[5]) * 1e3)
            acc["fill_call_ms"].append((t1 - t0) * 1e3)
            acc["accept_call_ms"].append((t3 - t2) * 1e3)
        del cache

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    # the classification kernel alone: the same builds once more, with events around the kernel (they sit between the
    # kernels of a build and would lengthen the device time that `value` is taken from)
    for _ in range(args.steps):
        ck = xg.compile_grammar(vocab, ebnf, root, stream=stream, time_kernel=True)
        acc["build_kernel_ms"].append(ck.stats.kernel_ms)
        del ck

    # the last step's bitmask: fraction of logits masked, and the bytes the apply kernel moves for it (a 16-byte vector of
    # logits whose tokens are all allowed is neither read nor written, one whose tokens are all masked is written
    # without a read, a mixed one is read and written back)
    bm = bitmask.cpu().numpy().view(np.uint32)
    bm_bytes = bm.view(np.uint8).reshape(B, W * 4)[:, :V // 8]       # one byte = the 8 tokens of one bf16 vector
    allowed = int(np.unpackbits(bm.view(np.uint8)).sum())
    masked = B * V - allowed
    moved = {}
    n8_zero, n8_full = int((bm_bytes == 0).sum()), int((bm_bytes == 0xFF).sum())
    moved[2] = B * W * 4 + 16 * n8_zero + 32 * (bm_bytes.size - n8_zero - n8_full) + 2 * B * (V % 8)
    nib = np.stack([bm_bytes & 0xF, bm_bytes >> 4])
    n4_zero, n4_full = int((nib == 0).sum()), int((nib == 0xF).sum())
    moved[4] = B * W * 4 + 16 * n4_zero + 32 * (nib.size - n4_zero - n4_full) + 4 * B * (V % 8)

    mean = lambda xs: float(sum(xs) / len(xs))
    med = lambda xs: float(sorted(xs)[len(xs) // 2])
    st = last_stats
    build_ms = mean(acc["build_device_ms"])
    kernel_ms = mean(acc["build_kernel_ms"])
    host_ms = mean(acc["build_host_ms"])
    checks = int(st.checks)
    value = checks / (build_ms * 1e-3)

    def build_roofline(stats, k_ms):
        """HBM roofline of one launch of the build kernel: bytes of the pairs a lane stepped through (token bytes + 4 bytes
        of offset in, 2 bits out) over the kernel's duration.  The logical figure (every built plane x every token, skipped
        or not) is kept beside it under its own name."""
        executed_bytes = int(stats.executed_token_bytes) + 4.25 * int(stats.executed_checks)
        logical_bytes = int(stats.built) * (tok_bytes_of[id(stats)] + 4.25 * n_checkable_of[id(stats)])
        gbs = executed_bytes / (k_ms * 1e-3) / 1e9
        return {"kernel": "k_build", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                "traffic": None, "algorithmic_bytes_per_launch": executed_bytes, "executed_pairs_per_launch": int(stats.executed_checks),
                "kernel_ms": k_ms, "executed_pairs_per_s": int(stats.executed_checks) / (k_ms * 1e-3),
                "logical_checks_accounting": {"bytes_per_launch": logical_bytes, "achieved": logical_bytes / (k_ms * 1e-3) / 1e9,
                                              "note": "every (built plane, token) pair counted, also the ones skipped by their first byte or copied from "
                                                      "another plane: not a bandwidth figure, kept for comparison with earlier lines"},
                "note": "the kernel is bound by instruction issue and load latency of a divergent interpreter, not by HBM: the HBM target of 40 % is not met by the build"}

    tok_bytes_of, n_checkable_of = {id(st): tok_bytes}, {id(st): n_checkable}
    default_workload = args.config == 5 and B == 1024
    roof = build_roofline(st, kernel_ms)
    roof["traffic"] = measured_traffic("k_build", default_workload)
    out = {
        "metric": "mask-cache build (position x token) checks/s; batch-%d mask fill+apply us/step" % B,
        "value": value,
        "unit": "checks/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": cfg.name, "config_index": cfg.index, "vocab": V, "batch": B, "positions": int(st.positions),
                   "unique_positions": int(st.unique), "built_positions": int(st.built), "checks_per_build": checks,
                   "executed_checks": int(st.executed_checks), "slow_path_checks": int(st.slow_path),
                   "value_basis": "logical (built plane, token) pairs over the device time of one cache build (HIP events: clearing of the rows and "
                                  "table upload to last plane); executed pairs and the end-to-end rate with host lowering are under `build`"},
        "build": {"device_ms": build_ms, "kernel_ms": kernel_ms, "host_lower_ms": host_ms,
                  "executed_checks_per_s_device": int(st.executed_checks) / (build_ms * 1e-3),
                  "checks_per_s_end_to_end": checks / ((build_ms + host_ms) * 1e-3),
                  "executed_checks_per_s_end_to_end": int(st.executed_checks) / ((build_ms + host_ms) * 1e-3),
                  "n_accepted_bits": int(st.n_accepted), "n_uncertain_bits": int(st.n_uncertain)},
        "decode": {"matchers": "device-resident (accept kernel, fill without upload)",
                   "fill_us": med(acc["fill_device_us"]), "apply_bf16_us": med(acc["apply_bf16_us"]), "apply_f32_us": med(acc["apply_f32_us"]),
                   "accept_us": med(acc["accept_us"]),
                   "fill_apply_bf16_us": med(acc["fill_device_us"]) + med(acc["apply_bf16_us"]),
                   "fill_apply_f32_us": med(acc["fill_device_us"]) + med(acc["apply_f32_us"]),
                   "fill_between_events_us": med(acc["fill_us"]),
                   "fill_call_host_us": med(acc["fill_call_ms"]) * 1e3, "accept_call_host_us": med(acc["accept_call_ms"]) * 1e3,
                   "masked_fraction_last_step": masked / float(B * V)},
        "roofline": roof,
    }
    # the build kernel is an interpreter: what bounds it is the rate at which the SIMDs issue vector instructions
    # (256 CUs x 4 SIMDs of 16 lanes at 2.4 GHz: a vector instruction of a 64-lane wave occupies its SIMD for 4 cycles);
    # scalar and branch instructions issue on ports of their own and are reported beside, not against that peak
    valu_peak = 256 * 4 * 2.4e9 / 4
    counted = default_workload and kernel_sources_sha256() == PMC["sources_sha256"]
    n_valu = PMC["k_build_valu_instructions"] if counted else None
    out["roofline_alu"] = {"kernel": "k_build", "bound": "alu", "achieved": (n_valu / (kernel_ms * 1e-3)) if n_valu else None,
                           "peak": valu_peak, "unit": "vector wave-instructions/s",
                           "frac": (n_valu / (kernel_ms * 1e-3) / valu_peak) if n_valu else None, "traffic": None,
                           "scalar_and_branch_instructions_per_launch": PMC["k_build_scalar_and_branch_instructions"] if counted else None,
                           "note": "instruction counts from rocprofv3 SQ counters, valid for the kernel sources they were taken with (null otherwise)"}
    for name, key, e in (("roofline_apply_bf16", "apply_bf16_us", 2), ("roofline_apply_f32", "apply_f32_us", 4)):
        t = med(acc[key]) * 1e-6
        gbs = moved[e] / t / 1e9
        out[name] = {"kernel": "k_apply_vec", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": measured_traffic("k_apply_vec<8>" if e == 2 else "k_apply_vec<4>", default_workload),
                     "algorithmic_bytes_per_launch": moved[e],
                     "accounting": "bytes the kernel has to move for this bitmask: bitmask read + 16 B written per fully masked vector + 32 B read and "
                                   "written per mixed vector (last step's bitmask)",
                     "achieved_read_modify_write_accounting": (B * W * 4 + 2 * B * V * e) / t / 1e9,
                     "achieved_store_only_accounting": (B * W * 4 + masked * e) / t / 1e9}
    tf = med(acc["fill_device_us"]) * 1e-6
    out["roofline_fill"] = {"kernel": "k_fill + k_recheck_slow", "bound": "hbm", "achieved": B * W * 4 / tf / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": B * W * 4 / tf / 1e9 / HBM_PEAK_GBS, "traffic": measured_traffic("k_fill", default_workload),
                            "accounting": "bitmask write only, over the whole device time of fill (upload, union, re-check)"}
    # fill + apply as one unit (the decode half of the metric): bitmask written once, then what apply moves
    for name, key, e in (("roofline_fill_apply_bf16", "apply_bf16_us", 2), ("roofline_fill_apply_f32", "apply_f32_us", 4)):
        t = (med(acc["fill_device_us"]) + med(acc[key])) * 1e-6
        gbs = (B * W * 4 + moved[e]) / t / 1e9
        out[name] = {"kernel": "k_fill + k_recheck_slow + k_apply_vec", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": None, "us_per_step": t * 1e6,
                     "accounting": "bitmask write + the bytes apply moves (see roofline_apply_*), over fill's and apply's device time"}

    if not args.no_tagdispatch_build:
        # one cache build of the TagDispatch workload (64 tools, V = 128,256): a millisecond-scale launch of the same kernel
        cfg3 = gen.build_config(3)
        vocab3 = xg.Vocab(cfg3.vocab.tokens, cfg3.vocab.eos_id, cfg3.vocab.special_ids)
        ebnf3, root3 = cfg3.grammars[0]
        xg.compile_grammar(vocab3, ebnf3, root3, stream=stream)               # first use: vocabulary upload, allocations
        k3 = xg.compile_grammar(vocab3, ebnf3, root3, stream=stream, time_kernel=True).stats.kernel_ms
        c3 = xg.compile_grammar(vocab3, ebnf3, root3, stream=stream)
        s3 = c3.stats
        tok_bytes_of[id(s3)] = sum(len(t) for i, t in enumerate(cfg3.vocab.tokens) if t and i not in cfg3.vocab.special_ids)
        n_checkable_of[id(s3)] = sum(1 for i, t in enumerate(cfg3.vocab.tokens) if t and i not in cfg3.vocab.special_ids)
        out["build_tagdispatch"] = {"workload": cfg3.name, "vocab": cfg3.vocab.size, "positions": int(s3.positions), "planes_built": int(s3.built),
                                    "checks": int(s3.checks), "executed_checks": int(s3.executed_checks), "slow_path_checks": int(s3.slow_path),
                                    "device_ms": s3.device_ms, "kernel_ms": k3, "host_lower_ms": s3.host_lower_ms,
                                    "checks_per_s_device": int(s3.checks) / (s3.device_ms * 1e-3),
                                    "roofline": build_roofline(s3, k3)}
        counted3 = kernel_sources_sha256() == PMC["sources_sha256"]
        if counted3:
            f3, w3 = PMC["k_build_tagdispatch"]
            out["build_tagdispatch"]["roofline"]["traffic"] = (f3 * PMC["fetch_scale"] + w3 * PMC["write_scale"]) * 1024.0
        n3 = PMC["k_build_tagdispatch_valu_instructions"] if counted3 else None
        out["build_tagdispatch"]["roofline_alu"] = {
            "kernel": "k_build", "bound": "alu", "achieved": (n3 / (k3 * 1e-3)) if n3 else None, "peak": valu_peak,
            "unit": "vector wave-instructions/s", "frac": (n3 / (k3 * 1e-3) / valu_peak) if n3 else None, "traffic": None,
            "scalar_and_branch_instructions_per_launch": PMC["k_build_tagdispatch_scalar_and_branch_instructions"] if counted3 else None}
        del c3, vocab3

    if not args.no_host_matchers:
        # the same decode step with the parsers on the host (one Earley chart per matcher, frontier and context uploaded by
        # every fill call), for comparison: 10 steps from the state the timed loop ended in
        hm = [xg.Matcher(cache0) for _ in range(B)]
        for b in range(B):
            if not ended[b]:
                for t in traces[b][:cursor[b]]:
                    assert hm[b].accept_token(t)
        hbatch = xg.MatcherBatch(hm)
        h_fill, h_fill_dev, h_acc = [], [], []
        nxt = np.zeros(B, dtype=np.int32)
        for _ in range(10):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            xg.fill_next_token_bitmask(hbatch, bitmask.data_ptr(), W, stream)
            h_fill.append((time.perf_counter() - t0) * 1e6)
            h_fill_dev.append(xg.fill_last_device_us())
            for b in range(B):
                if ended[b] or cursor[b] >= len(traces[b]):
                    nxt[b] = -1
                else:
                    nxt[b] = traces[b][cursor[b]]
                    cursor[b] += 1
            t0 = time.perf_counter()
            stt = hbatch.accept_tokens(nxt)
            h_acc.append((time.perf_counter() - t0) * 1e6)
            assert not stt.any()
        out["decode_host_matchers"] = {"fill_call_host_us": med(h_fill), "fill_device_us": med(h_fill_dev), "accept_call_host_us": med(h_acc),
                                       "note": "host Earley parsers; fill uploads the frontier planes and context slices of all rows every step"}
        del hbatch, hm

    if args.cross_grammar:
        cfg4 = gen.build_config(4)
        vocab4 = xg.Vocab(cfg4.vocab.tokens, cfg4.vocab.eos_id, cfg4.vocab.special_ids)
        n_tok4 = sum(1 for i, t in enumerate(cfg4.vocab.tokens) if t and i not in cfg4.vocab.special_ids)
        pool4 = xg.Pool()
        tot = {"positions": 0, "planes_used": 0, "planes_built": 0, "device_ms": 0.0, "host_ms": 0.0, "executed": 0}
        t4 = time.perf_counter()
        keep = []
        for ebnf4, root4 in cfg4.grammars[:args.cross_grammar]:
            c4 = xg.compile_grammar(vocab4, ebnf4, root4, pool=pool4, stream=stream)
            s4 = c4.stats
            tot["positions"] += s4.positions; tot["planes_used"] += s4.unique; tot["planes_built"] += s4.built
            tot["device_ms"] += s4.device_ms; tot["host_ms"] += s4.host_lower_ms; tot["executed"] += s4.executed_checks
            tot["partial_hits"] = tot.get("partial_hits", 0) + s4.partial_hits
            keep.append(c4)
        wall4 = time.perf_counter() - t4
        out["cross_grammar"] = {"grammars": len(keep), "vocab": cfg4.vocab.size, "positions": tot["positions"], "planes_used": tot["planes_used"],
                                "planes_built_once": tot["planes_built"], "pool_rows": pool4.stats()[0], "pool_device_bytes": pool4.stats()[1],
                                "device_ms": tot["device_ms"], "host_lower_ms": tot["host_ms"], "wall_s": wall4,
                                "checks_per_s_device": tot["planes_built"] * n_tok4 / (tot["device_ms"] * 1e-3),
                                "checks_per_s_served_device": tot["planes_used"] * n_tok4 / (tot["device_ms"] * 1e-3),
                                "executed_checks": tot["executed"], "partial_hits": tot.get("partial_hits", 0)}
        del keep, pool4

    if not args.no_jit:
        # per-step latency of fill (host + device, synchronised) along 128 decode steps of B fresh sentences: on a cache
        # compiled just in time (nothing pre-built) and, for reference, on the fully built one
        def step_latencies(c):
            ms_ = [xg.Matcher(c) for _ in range(B)]
            batch_ = xg.MatcherBatch(ms_)
            rng_ = random.Random(4242)
            tr = [seg.segment(cfg.sample_text(rng_, 0), rng_) + [cfg.vocab.eos_id] for _ in range(B)]
            lat = []
            for stp in range(128):
                torch.cuda.synchronize()
                tj = time.perf_counter()
                xg.fill_next_token_bitmask(batch_, bitmask.data_ptr(), W, stream)
                torch.cuda.synchronize()
                lat.append((time.perf_counter() - tj) * 1e3)
                batch_.accept_tokens([t[stp] if stp < len(t) else -1 for t in tr])
            return sorted(lat)
        pct = lambda v, q: v[min(len(v) - 1, int(q * len(v)))]
        flat = step_latencies(cache0)
        out["jit"] = {"note": "fill-step latency (host call + device, synchronised) over 128 decode steps of %d fresh sentences, host matchers; "
                              "K = planes built at compile time (the costliest first), the rest by the fill calls that reach them, on the library's own stream" % B,
                      "fully_built_cache": {"fill_step_ms": {"mean": mean(flat), "median": pct(flat, 0.5), "p99": pct(flat, 0.99), "max": flat[-1]}},
                      "K": {}}
        for K in (0, 5, 10):
            jit_cache = xg.compile_grammar(vocab, ebnf, root, stream=stream, jit=True, jit_prebuild=K)
            compile_ms = jit_cache.stats.device_ms
            compile_host_ms = jit_cache.stats.host_lower_ms
            jlat = step_latencies(jit_cache)
            jbuilt, jlaunches, jms = jit_cache.jit_stats()
            out["jit"]["K"][str(K)] = {"compile_device_ms": compile_ms, "compile_host_ms": compile_host_ms, "planes_total": jit_cache.num_planes(),
                                       "planes_built_after_128_steps": jbuilt, "build_launches_in_fill": jlaunches, "build_device_ms_in_fill": jms,
                                       "fill_step_ms": {"mean": mean(jlat), "median": pct(jlat, 0.5), "p99": pct(jlat, 0.99), "max": jlat[-1]}}
            del jit_cache

    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.Oracle(ebnf, root)
        va = oracle.VocabArrays(cfg.vocab.tokens, cfg.vocab.eos_id, cfg.vocab.special_ids)
        pos = orc.positions()
        prng = random.Random(7)
        sample = prng.sample(pos, min(args.cpu_positions, len(pos)))
        threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))
        t0 = time.perf_counter()
        for p in sample:
            orc.classes(p, va, threads=threads)
        dt = time.perf_counter() - t0
        # the same on one core (the paper's timings are single-threaded), on a smaller seeded sample
        one = prng.sample(pos, min(96, len(pos)))
        t0 = time.perf_counter()
        for p in one:
            orc.classes(p, va, threads=1)
        dt1 = time.perf_counter() - t0
        # decode side: the plain-definition mask of a few rows of the batch, and a plain masking loop over one row of logits
        rows_sample = [b for b in range(0, B, max(1, B // 4))][:4]
        hist = [b"".join(cfg.vocab.tokens[t] for t in traces[b][:cursor[b]] if t != cfg.vocab.eos_id) for b in rows_sample]
        t0 = time.perf_counter()
        for h in hist:
            orc.mask(h, va, threads=threads)
        dtm = (time.perf_counter() - t0) / len(hist)
        bits = np.ascontiguousarray(logits32_src[0].cpu().numpy()).view(np.uint32).reshape(1, V).copy()
        bm_row = bitmask[:1].cpu().numpy()
        t0 = time.perf_counter()
        oracle.apply_f32(bits, bm_row)
        dta = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": len(sample) * n_checkable / dt, "unit": "checks/s", "cores": threads, "kind": "oracle",
                               "sample": "%d of %d positions (seeded sample) x all %d tokens, textbook Earley per pair, %.1f s"
                                         % (len(sample), len(pos), n_checkable, dt),
                               "value_one_core": len(one) * n_checkable / dt1,
                               "decode_mask_us_per_row": dtm * 1e6, "apply_f32_us_per_row": dta * 1e6,
                               "decode_note": "plain-definition mask of one row (oracle, %d threads) and masking of one fp32 row; the GPU figures above are for %d rows" % (threads, B)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
