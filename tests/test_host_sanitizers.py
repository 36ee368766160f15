"""Host-side C++ under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The lowering (EBNF -> canonical automata -> packed tables, bounded classes, follow signatures), the host Earley parser,
and the recogniser and accept cores that the kernels run per lane are built with `-fsanitize=address,undefined` into
one executable (`tests/hostcheck/sanitize_main`) and run over the workloads' grammars with sampled vocabularies: the
same cross-checks as `test_recogniser_core.py`, with every out-of-bounds access, use after free, signed overflow or
misaligned access turned into a failure.  Device code and the HIP calls of `api.cpp` are not covered (no GPU sanitizer
on this pool).
"""
from __future__ import annotations

import os
import random
import struct
import subprocess

import pytest

import gen

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2601_04426_amd", "csrc")
HC = os.path.join(HERE, "hostcheck")
EXE = os.path.join(HC, "sanitize_main")


@pytest.fixture(scope="module")
def exe():
    srcs = [os.path.join(HC, "sanitize_main.cpp"), os.path.join(HC, "hostcheck.cpp"), os.path.join(CSRC, "grammar.cpp"), os.path.join(CSRC, "tables.cpp")]
    deps = srcs + [os.path.join(CSRC, f) for f in ("earley_core.hpp", "accept_core.hpp", "device.hpp", "tables.hpp", "grammar.hpp")]
    if not os.path.exists(EXE) or any(os.path.getmtime(d) > os.path.getmtime(EXE) for d in deps):
        cmd = ["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
               "-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__", "-o", EXE] + srcs
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout[-3000:]
    return EXE


def run(exe, tmp_path, ebnf, root, tokens, seq):
    (tmp_path / "g.ebnf").write_text(ebnf)
    (tmp_path / "tokens.bin").write_bytes(b"".join(struct.pack("<I", len(t)) + t for t in tokens))
    (tmp_path / "seq.bin").write_bytes(b"".join(struct.pack("<i", s) for s in seq))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    env.pop("LD_PRELOAD", None)
    res = subprocess.run([exe, str(tmp_path / "g.ebnf"), root, str(tmp_path / "tokens.bin"), str(tmp_path / "seq.bin")],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert res.returncode == 0 and res.stdout.startswith("ok"), res.stdout[-3000:]
    return [int(x) for x in res.stdout.split()[1:]]


@pytest.mark.parametrize("index", [1, 2, 3, 5])
def test_lowering_parser_and_cores_under_sanitizers(exe, tmp_path, index):
    cfg = gen.build_config(index, n_tools=3) if index == 3 else gen.build_config(index, max_objects=40) if index == 5 else gen.build_config(index)
    ebnf, root = cfg.grammars[0]
    rng = random.Random(9000 + index)
    seg = gen.Segmenter(cfg.vocab)
    ids = []
    for _ in range(2):
        ids += seg.segment(cfg.sample_text(rng, 0), rng)[:60] + [-1]
    # a sampled vocabulary that still holds the tokens of the sequences
    used = sorted({i for i in ids if i >= 0})
    extra = rng.sample(range(1, cfg.vocab.size), 250)
    keep = [0] + used + [i for i in extra if i not in set(used)]
    remap = {old: new for new, old in enumerate(keep)}
    tokens = [cfg.vocab.tokens[i] for i in keep]
    seq = [remap[i] if i >= 0 else -1 for i in ids]
    a, b, c = run(exe, tmp_path, ebnf, root, tokens, seq)
    assert a > 1000 and c > 50


def test_tag_dispatch_and_recursion_under_sanitizers(exe, tmp_path):
    ebnf = ('root ::= TagDispatch(("<t>", body), ("<u>", num), stop_strs=("END",))\n'
            'body ::= list "</t>"\nlist ::= "[" (list ("," list)*)? "]" | [a-z]{1,3}\nnum ::= [0-9]{1,3} ";"\n')
    alphabet = b"<>tu/END1;abcz[],"
    rng = random.Random(12)
    tokens = [b""] + [bytes([c]) for c in sorted(set(alphabet))]
    tokens += sorted({bytes(rng.choice(alphabet) for _ in range(rng.randrange(2, 20))) for _ in range(200)} - set(tokens))
    single = {t: i for i, t in enumerate(tokens) if len(t) == 1}
    seq = [single[bytes([c])] for c in b"zz<t>[[a,bc],[]]</t>a<u>11;END"] + [-1]
    a, b, c = run(exe, tmp_path, ebnf, "root", tokens, seq)
    assert a > 1000 and c > 30
