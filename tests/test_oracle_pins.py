"""Pins for the CPU oracle: brute force on tiny grammars, closed forms, library routines.

Each test is chosen so that a plausible mistake in the oracle (a dropped completion, a wrong
nullable rule, a transposed bit, a bad UTF-8 boundary, a wrong merge in the minimiser) fails it.
None of the expected values comes from the GPU library.
"""
import random
import re

import numpy as np
import pytest

import oracle
from oracle import fsm as ofsm
from bruteforce import all_strings, languages, prefixes

# (name, EBNF text, the same grammar as plain data, alphabet, enumeration bound N)
TINY = [
    ("nest", 'root ::= "a" root "b" | "c"\n',
     {"root": ("alt", ("seq", ("lit", b"a"), ("ref", "root"), ("lit", b"b")), ("lit", b"c"))}, b"abc", 15),
    ("nullable_leftrec", 'root ::= a b\na ::= a "x" | ""\nb ::= "y"?\n',
     {"root": ("seq", ("ref", "a"), ("ref", "b")), "a": ("alt", ("seq", ("ref", "a"), ("lit", b"x")), ("lit", b"")),
      "b": ("opt", ("lit", b"y"))}, b"xy", 9),
    ("list", 'root ::= "[" (item ("," item)*)? "]"\nitem ::= "0" | "1" item?\n',
     {"root": ("seq", ("lit", b"["), ("opt", ("seq", ("ref", "item"), ("star", ("seq", ("lit", b","), ("ref", "item"))))),
               ("lit", b"]")),
      "item": ("alt", ("lit", b"0"), ("seq", ("lit", b"1"), ("opt", ("ref", "item"))))}, b"[],01", 9),
    ("repeat", 'root ::= x{2,4} "c"\nx ::= "a" | "ab"\n',
     {"root": ("seq", ("rep", ("ref", "x"), 2, 4), ("lit", b"c")), "x": ("alt", ("lit", b"a"), ("lit", b"ab"))}, b"abc", 10),
    ("ambiguous", 'root ::= s "."\ns ::= s s | "a" | ""\n',
     {"root": ("seq", ("ref", "s"), ("lit", b".")), "s": ("alt", ("seq", ("ref", "s"), ("ref", "s")), ("lit", b"a"), ("lit", b""))},
     b"a.", 9),
    ("mutual", 'root ::= "(" mid ")"\nmid ::= root mid | ""\n',
     {"root": ("seq", ("lit", b"("), ("ref", "mid"), ("lit", b")")), "mid": ("alt", ("seq", ("ref", "root"), ("ref", "mid")), ("lit", b""))},
     b"()", 12),
    ("classes_and_groups", 'root ::= ([ab] | "c" k)+ "d"{0,2}\nk ::= [a-c]{1,2}\n',
     {"root": ("seq", ("alt", ("set", b"ab"), ("seq", ("lit", b"c"), ("ref", "k"))),
               ("star", ("alt", ("set", b"ab"), ("seq", ("lit", b"c"), ("ref", "k")))), ("rep", ("lit", b"d"), 0, 2)),
      "k": ("rep", ("set", b"abc"), 1, 2)}, b"abcd", 8),
]


def _tiny_vocab(alphabet: bytes, max_len: int = 3):
    toks = [b""] + [s for s in all_strings(alphabet, max_len) if s]
    return toks, oracle.VocabArrays(toks, 0, [0])


@pytest.mark.parametrize("name,ebnf,rules,alphabet,N", TINY, ids=[t[0] for t in TINY])
def test_sentences_match_enumeration(name, ebnf, rules, alphabet, N):
    """accepts(s) for every string up to length 7 == membership in the enumerated language."""
    o = oracle.Oracle(ebnf)
    L = languages(rules, N)["root"]
    for s in all_strings(alphabet, 7 if len(alphabet) <= 3 else 6):
        want = s in L
        assert o.accepts(s) == want, s
        assert o.accepts(s, direct=True) == want, s


@pytest.mark.parametrize("name,ebnf,rules,alphabet,N", TINY, ids=[t[0] for t in TINY])
def test_masks_match_enumeration(name, ebnf, rules, alphabet, N):
    """mask(h)[t] == (h.t is a prefix of an enumerated sentence), EOS == (h is a sentence)."""
    o = oracle.Oracle(ebnf)
    L = languages(rules, N)["root"]
    P = prefixes(L)
    toks, va = _tiny_vocab(alphabet)
    # completions stay within N for these histories: every viable prefix of length <= 6 must be in P
    for h in all_strings(alphabet, 3):
        if h not in P:
            with pytest.raises(ValueError):
                o.mask(h, va)
            continue
        for direct in (False, True):
            m = o.mask(h, va, direct=direct)
            assert m[0] == (h in L), h
            for i, t in enumerate(toks):
                if i:
                    assert m[i] == ((h + t) in P), (h, t, direct)


def _access_words(d: ofsm.DFA):
    """Shortest symbol word reaching each DFA state; a rule edge is written as byte 0xF0 + rule index."""
    word = {d.start: b""}
    order = [d.start]
    for q in order:
        for mask, t in d.bedges[q]:
            if t not in word:
                word[t] = word[q] + bytes([(mask & -mask).bit_length() - 1])
                order.append(t)
        for r, t in d.redges[q].items():
            if t not in word:
                word[t] = word[q] + bytes([0xF0 + r])
                order.append(t)
    return word


def _placeholder(e, index):
    k = e[0]
    if k == "ref":
        return ("lit", bytes([0xF0 + index[e[1]]]))
    if k in ("seq", "alt"):
        return (k,) + tuple(_placeholder(c, index) for c in e[1:])
    if k in ("star", "opt"):
        return (k, _placeholder(e[1], index))
    if k == "rep":
        return ("rep", _placeholder(e[1], index), e[2], e[3])
    return e


def _suffix_languages(o, rules, N):
    """{(rule, state): enumerated Suf(rule, state)}: (access word)^-1 L_symbolic(rule) with every rule
    symbol replaced by that rule's enumerated sentences."""
    index = o.low.index
    L = languages(rules, N)
    out = {}
    for rule in o.low.reachable:
        sym_lang = languages({"r": _placeholder(rules[rule], index)}, N)["r"]
        for q, w in _access_words(o.low.dfa[rule]).items():
            suf = set()
            for s in sym_lang:
                if not s.startswith(w):
                    continue
                cur = {b""}
                for c in s[len(w):]:
                    nxt = L[o.order[c - 0xF0]] if c >= 0xF0 else {bytes([c])}
                    cur = {x + y for x in cur for y in nxt if len(x) + len(y) <= N}
                suf |= cur
            out[(rule, q)] = suf
    return out


def _classes_by_definition(suf, toks):
    pre = prefixes(suf)
    want = [oracle.REJECTED]
    for t in toks[1:]:
        if t in pre:
            want.append(oracle.ACCEPTED)
        elif any(t[:k] in suf for k in range(1, len(t))):
            want.append(oracle.UNCERTAIN)
        else:
            want.append(oracle.REJECTED)
    return want


@pytest.mark.parametrize("name,ebnf,rules,alphabet,N", TINY, ids=[t[0] for t in TINY])
def test_classes_match_enumeration(name, ebnf, rules, alphabet, N):
    """accepted / uncertain / rejected of every position == the definition evaluated on the
    enumerated suffix language."""
    o = oracle.Oracle(ebnf)
    sufs = _suffix_languages(o, rules, N)
    toks, va = _tiny_vocab(alphabet)
    n_checked = 0
    for pos in o.positions():
        got = o.classes(pos, va)
        assert list(got) == _classes_by_definition(sufs[pos], toks), pos
        n_checked += 1
    assert n_checked >= 2


@pytest.mark.parametrize("name,ebnf,rules,alphabet,N", TINY, ids=[t[0] for t in TINY])
def test_classes_with_one_level_of_context_match_enumeration(name, ebnf, rules, alphabet, N):
    """With a parent state x (where the referencing rule continues), the suffix language is the
    concatenation Suf(position) . Suf(x); classes follow the same definition on it."""
    o = oracle.Oracle(ebnf)
    sufs = _suffix_languages(o, rules, N)
    toks, va = _tiny_vocab(alphabet)
    n_checked = 0
    for parent_rule in o.low.reachable:
        d = o.low.dfa[parent_rule]
        for q in range(d.n):
            for r, x in d.redges[q].items():
                child = o.order[r]
                for pos in o.positions():
                    if pos[0] != child:
                        continue
                    cat = {a + b for a in sufs[pos] for b in sufs[(parent_rule, x)] if len(a) + len(b) <= N}
                    got = o.classes(pos, va, parent=(parent_rule, x))
                    assert list(got) == _classes_by_definition(cat, toks), (pos, parent_rule, x)
                    n_checked += 1
    assert n_checked >= 1


@pytest.mark.parametrize("name,ebnf,rules,alphabet,N", TINY, ids=[t[0] for t in TINY])
def test_follow_filtered_classes_match_enumeration(name, ebnf, rules, alphabet, N):
    """With the follow filter a token that leaves the outermost rule after t[0:i] stays uncertain only if
    t[i:] is a prefix of an enumerated follow string of that rule; follow strings are enumerated as the least
    fixed point of  follow(R) = U over sites  Suf(site) . follow(site's rule),  follow(root) containing ''."""
    o = oracle.Oracle(ebnf)
    sufs = _suffix_languages(o, rules, N)
    toks, va = _tiny_vocab(alphabet)
    follow = {r: set() for r in o.low.reachable}
    follow[o.root].add(b"")
    while True:
        grew = False
        for q_rule in o.low.reachable:
            d = o.low.dfa[q_rule]
            for q in range(d.n):
                for r, x in d.redges[q].items():
                    add = {a + b for a in sufs[(q_rule, x)] for b in follow[q_rule] if len(a) + len(b) <= N}
                    if not add <= follow[o.order[r]]:
                        follow[o.order[r]] |= add
                        grew = True
        if not grew:
            break

    def want(lang, outer):
        pre, fpre = prefixes(lang), prefixes(follow[outer])
        out = [oracle.REJECTED]
        for t in toks[1:]:
            if t in pre:
                out.append(oracle.ACCEPTED)
            elif any(t[:k] in lang and t[k:] in fpre for k in range(1, len(t))):
                out.append(oracle.UNCERTAIN)
            else:
                out.append(oracle.REJECTED)
        return out
    n_moved = 0
    for pos in o.positions():
        got = list(o.classes(pos, va, follow=True))
        assert got == want(sufs[pos], pos[0]), pos
        n_moved += sum(1 for a, b in zip(got, o.classes(pos, va)) if a != b)
    for parent_rule in o.low.reachable:
        d = o.low.dfa[parent_rule]
        for q in range(d.n):
            for r, x in d.redges[q].items():
                for pos in o.positions():
                    if pos[0] == o.order[r]:
                        cat = {a + b for a in sufs[pos] for b in sufs[(parent_rule, x)] if len(a) + len(b) <= N}
                        assert list(o.classes(pos, va, parent=(parent_rule, x), follow=True)) == want(cat, parent_rule), (pos, parent_rule, x)
    if name in ("list", "repeat"):
        assert n_moved > 0                     # the filter does reject something on these grammars


def _reach_languages(o, rules, N):
    """{(rule, state): the enumerated strings that take the rule's automaton from its start state to the state}, every
    rule symbol on the way replaced by that rule's enumerated sentences."""
    index = o.low.index
    L = languages(rules, N)
    out = {}
    for rule in o.low.reachable:
        d = o.low.dfa[rule]
        sym_lang = languages({"r": _placeholder(rules[rule], index)}, N)["r"]
        reach = {q: set() for q in range(d.n)}
        seen = set()
        for s in sym_lang:
            for k in range(len(s) + 1):
                w = s[:k]
                if w in seen:
                    continue
                seen.add(w)
                q = d.start
                cur = {b""}
                for c in w:
                    if c >= 0xF0:
                        q = d.redges[q][c - 0xF0]
                        nxt = L[o.order[c - 0xF0]]
                    else:
                        q = next(t for m, t in d.bedges[q] if (m >> c) & 1)
                        nxt = {bytes([c])}
                    cur = {x + y for x in cur for y in nxt if len(x) + len(y) <= N}
                reach[q] |= cur
        for q in range(d.n):
            out[(rule, q)] = reach[q]
    return out


@pytest.mark.parametrize("name,ebnf,rules,alphabet,N", TINY, ids=[t[0] for t in TINY])
def test_frontier_matches_enumeration(name, ebnf, rules, alphabet, N):
    """The scannable frontier after a history h, by its definition: position (R, q) belongs to it iff q has a byte edge
    and h = u.v where an instance of R can start after u (u is a left context of R: the empty string for the root rule,
    else a left context of a referencing rule followed by a string that takes that rule to the referencing state) and v
    takes R from its start state to q.  The grammars are reduced, so every such partial parse can be completed.  A
    spurious position, or a missing one, in Oracle.frontier fails this."""
    o = oracle.Oracle(ebnf)
    reach = _reach_languages(o, rules, N)
    H = 4 if len(alphabet) <= 3 else 3
    ctx = {r: set() for r in o.low.reachable}
    ctx[o.root].add(b"")
    while True:
        grew = False
        for q_rule in o.low.reachable:
            d = o.low.dfa[q_rule]
            for q in range(d.n):
                for r, x in d.redges[q].items():
                    add = {u + v for u in ctx[q_rule] for v in reach[(q_rule, q)] if len(u) + len(v) <= H}
                    if not add <= ctx[o.order[r]]:
                        ctx[o.order[r]] |= add
                        grew = True
        if not grew:
            break
    P = prefixes(languages(rules, N)["root"])
    n = 0
    for h in all_strings(alphabet, H):
        if h not in P:
            continue
        want = sorted((rule, q) for rule in o.low.reachable for q in range(o.low.dfa[rule].n)
                      if o.low.dfa[rule].bedges[q]
                      and any(h[:k] in ctx[rule] and h[k:] in reach[(rule, q)] for k in range(len(h) + 1)))
        assert o.frontier(h) == want, (h, o.frontier(h), want)
        n += 1
    assert n >= 5


def test_number_grammar_equals_python_regex():
    """A grammar without rule references is a regular expression: compare with `re`."""
    o = oracle.Oracle('root ::= "-"? ("0" | [1-9] [0-9]*) ("." [0-9]+)? ([eE] [+\\-]? [0-9]+)?\n')
    rx = re.compile(rb"-?(0|[1-9][0-9]*)(\.[0-9]+)?([eE][+-]?[0-9]+)?")
    alpha = b"-0.7eE+"
    sentences = set()
    for s in all_strings(alpha, 6):
        ok = rx.fullmatch(s) is not None
        assert o.accepts(s) == ok, s
        if ok:
            sentences.add(s)
    # viable prefixes: every prefix of length <= 3 that extends to a sentence of length <= 6
    P = prefixes(sentences)
    toks, va = _tiny_vocab(alpha, 2)
    for h in all_strings(alpha, 2):
        if h in P:
            m = o.mask(h, va)
            for i, t in enumerate(toks):
                if i:
                    assert m[i] == ((h + t) in P), (h, t)


@pytest.mark.parametrize("cls", ['[^"\\\\]', "[\\x80-\\U0010FFFF]", "[a-z\\u00e9-\\uffff]", "[^\\x00-\\U0001F600]",
                                 "[\\u07ff-\\u0800\\uffff-\\U00010000]"])
def test_utf8_class_lowering_is_exactly_the_encodings(cls):
    """The byte automaton of a character class accepts exactly {chr(c).encode()}: enumerate it."""
    order, rules = oracle.parse_ebnf(f"root ::= {cls}\n")
    _, neg, ranges = rules["root"]
    d = ofsm.class_dfa(neg, tuple(ranges))
    accepted = set()
    stack = [(d.start, b"")]
    while stack:
        q, s = stack.pop()
        if d.final[q]:
            accepted.add(s)
        assert len(s) <= 4
        for mask, t in d.bedges[q]:
            m = mask
            while m:
                b = (m & -m).bit_length() - 1
                m &= m - 1
                stack.append((t, s + bytes([b])))
    listed = set()
    for lo, hi in ranges:
        listed.update(range(lo, hi + 1))
    want = set()
    for cp in range(0x110000):
        if 0xD800 <= cp <= 0xDFFF:
            continue
        if (cp in listed) != neg:
            want.add(chr(cp).encode("utf-8"))
    assert accepted == want


def test_token_may_end_inside_a_code_point():
    o = oracle.Oracle('root ::= "\\u00e9" [^a]\n')
    toks = [b"", b"\xc3", b"\xa9", b"\xc3\xa9", b"\xc3\xa9\xe2", b"\xc3\xa9\xe2\x82", b"\xc3\xa9a", b"\xa9\xc3", b"\xc3\xa9\xed\xa0"]
    va = oracle.VocabArrays(toks, 0, [0])
    m = o.mask(b"", va)
    assert list(m) == [False, True, False, True, True, True, False, False, False]   # ED A0 starts a surrogate
    # after C3: A9 completes the e-acute; A9 C3 goes on into a two-byte scalar of [^a]
    assert list(o.mask(b"\xc3", va)) == [False, False, True, False, False, False, False, True, False]


def _naive_dispatch_ok(text: bytes, tags, stops):
    """Plain simulation of section 3.2 for sub-grammars that are prefix-free finite sets of literals.
    -> True if text is a complete sentence."""
    pos = 0
    seg_start = 0
    while True:
        hit = None
        for e in range(seg_start + 1, len(text) + 1):           # earliest completed pattern
            for k, (tag, _) in enumerate(tags):
                if e - len(tag) >= seg_start and text[e - len(tag):e] == tag:
                    hit = ("tag", k, e)
            for s in stops:
                if e - len(s) >= seg_start and text[e - len(s):e] == s:
                    hit = ("stop", 0, e)
            if hit:
                break
        if hit is None:
            return len(stops) == 0
        if hit[0] == "stop":
            return hit[2] == len(text)
        body = [lit for lit in tags[hit[1]][1] if text.startswith(lit, hit[2])]
        if not body:
            return False
        seg_start = hit[2] + len(body[0])


@pytest.mark.parametrize("stops", [(), (b"!!",)])
def test_tagdispatch_equals_naive_scan(stops):
    tags = [(b"<a>", [b"xy", b"z"]), (b"<bc>", [b"q"]), (b"<<", [b"a"])]
    stop_txt = ("" if not stops else ', stop_strs=("!!")')
    ebnf = ('root ::= TagDispatch(("<a>", g1), ("<bc>", g2), ("<<", g3)' + stop_txt + ')\n'
            'g1 ::= "xy" | "z"\ng2 ::= "q"\ng3 ::= "a"\n')
    o = oracle.Oracle(ebnf)
    rng = random.Random(7)
    alpha = b"<abc>xyzq!"
    n_yes = 0
    for trial in range(6000):
        if trial % 3 == 0:
            parts = []
            for _ in range(rng.randint(0, 3)):
                parts.append(bytes(rng.choice(b"abcxyzq>") for _ in range(rng.randint(0, 3))))
                tag, lits = rng.choice(tags)
                parts.append(tag + rng.choice(lits))
            parts.append(bytes(rng.choice(b"abcxyzq>") for _ in range(rng.randint(0, 3))))
            if stops and rng.random() < 0.7:
                parts.append(b"!!")
            text = b"".join(parts)
        else:
            text = bytes(rng.choice(alpha) for _ in range(rng.randint(0, 9)))
        want = _naive_dispatch_ok(text, tags, list(stops))
        n_yes += want
        assert o.accepts(text) == want, text
        assert o.accepts(text, direct=True) == want, text
    assert n_yes > 500


@pytest.mark.parametrize("n_tags,total_len,paper_states", [(5, 100, 60), (20, 400, 207), (50, 1000, 487), (100, 2000, 952)])
def test_tag_automaton_size_closed_form(n_tags, total_len, paper_states):
    """Section 4.1, Table 2: tags share the prefix `<function=`, the rest is random; the number of
    automaton states equals the number of distinct tag prefixes (trie nodes, root included), which
    for 20-byte tags is 1 + 10 + (about 10 per tag): 60 / 207 / 487 / 952 in the paper's draw."""
    rng = random.Random(n_tags)
    tags = set()
    while len(tags) < n_tags:
        tags.add(b"<function=" + bytes(rng.choice(b"abcdefghijklmnopqrstuvwxyz_") for _ in range(9)) + b">")
    tags = sorted(tags)
    assert sum(len(t) for t in tags) == total_len
    d = ofsm.tagdispatch_dfa([(t, 0) for t in tags], [])
    trie_nodes = len({t[:i] for t in tags for i in range(len(t) + 1)})
    dispatching_states = sum(1 for q in range(d.n) if d.final[q])
    assert dispatching_states + n_tags == trie_nodes
    assert 1 + 10 + 9 * n_tags - n_tags <= trie_nodes <= 1 + 10 + 10 * n_tags
    assert abs(trie_nodes - paper_states) <= 0.05 * paper_states


def _moore(d: ofsm.DFA):
    """Plain Moore refinement as a second opinion on the minimiser (number of classes)."""
    n = d.n
    block = [1 if d.final[q] else 0 for q in range(n)]
    while True:
        sig = {}
        new = []
        for q in range(n):
            row = [-1] * 256
            for mask, t in d.bedges[q]:
                for b in range(256):
                    if (mask >> b) & 1:
                        row[b] = block[t]
            key = (block[q], tuple(row), tuple(sorted((r, block[t]) for r, t in d.redges[q].items())))
            new.append(sig.setdefault(key, len(sig)))
        if len(sig) == len(set(block)):
            return len(sig)
        block = new


def test_minimiser_against_moore_on_random_automata():
    rng = random.Random(11)
    for trial in range(60):
        n = rng.randint(2, 14)
        d = ofsm.DFA()
        for _ in range(n):
            d.new(rng.random() < 0.3)
        d.final[rng.randrange(n)] = True
        for q in range(n):
            free = list(range(4))
            rng.shuffle(free)
            by_t = {}
            for b in free[:rng.randint(0, 4)]:
                t = rng.randrange(n)
                by_t[t] = by_t.get(t, 0) | (1 << (97 + b))
            d.bedges[q] = [(m, t) for t, m in by_t.items()]
            if rng.random() < 0.3:
                d.redges[q][rng.randrange(2)] = rng.randrange(n)
        try:
            m = ofsm.minimize(d)
        except ValueError:
            continue
        # Moore on the trimmed automaton = Moore on the minimiser's own output must be a fixed point,
        # and the output must have exactly as many states as Moore finds classes among useful states
        assert _moore(m) == m.n
        c = ofsm.canonical(m)
        assert c.n == m.n
        # same language on all words up to length 5 over bytes a-d and rule symbols 0/1 (as bytes 0,1)
        def run(dfa, word):
            q = dfa.start
            for s in word:
                nxt = None
                if s < 2:
                    nxt = dfa.redges[q].get(s)
                else:
                    for mask, t in dfa.bedges[q]:
                        if (mask >> s) & 1:
                            nxt = t
                if nxt is None:
                    return False
                q = nxt
            return dfa.final[q]
        for w in all_strings(bytes([0, 1, 97, 98, 99, 100]), 4):
            assert run(d, w) == run(c, w), w


def test_pack_bitmask_against_packbits():
    rng = np.random.default_rng(5)
    for V in (1, 31, 32, 33, 2048, 151936, 100001):
        m = rng.random(V) < 0.3
        got = oracle.pack_bitmask(m)
        pad = np.zeros(((V + 31) // 32) * 32, dtype=bool)
        pad[:V] = m
        want = np.packbits(pad, bitorder="little").view(np.uint32).view(np.int32)
        assert np.array_equal(got, want)
        assert got.dtype == np.int32


def test_apply_is_a_bitwise_select():
    """Masked entries become exactly -inf, the others keep their bit pattern (NaN payloads, -0.0,
    denormals, +-inf included)."""
    specials32 = np.array([0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00001, 0xFFC12345, 0x00000001,
                           0x807FFFFF, 0x3F800000, 0x7F7FFFFF], dtype=np.uint32)
    rng = np.random.default_rng(3)
    B, V = 3, 77
    lg = rng.integers(0, 2 ** 32, size=(B, V), dtype=np.uint64).astype(np.uint32)
    lg[0, :10] = specials32
    lg[1, 32:42] = specials32
    allow = rng.random((B, V)) < 0.5
    bm = np.stack([oracle.pack_bitmask(allow[b]) for b in range(B)])
    out = lg.copy()
    oracle.apply_f32(out, bm)
    assert np.array_equal(out, np.where(allow, lg, np.uint32(0xFF800000)))
    assert np.isneginf(out.view(np.float32)[~allow]).all()
    lg16 = rng.integers(0, 2 ** 16, size=(B, V), dtype=np.uint64).astype(np.uint16)
    lg16[0, :10] = (specials32 >> 16).astype(np.uint16)
    out16 = lg16.copy()
    oracle.apply_bf16(out16, bm)
    assert np.array_equal(out16, np.where(allow, lg16, np.uint16(0xFF80)))
    # a bf16 -inf widened to fp32 is -inf
    assert np.isneginf((out16[~allow].astype(np.uint32) << 16).view(np.float32)).all()


def test_ebnf_errors():
    for bad in ['root ::= "a', 'root ::= [a', 'root ::= (a', 'root ::= b\n', 'root ::= "a"{3,2}\n', 'root ::= "\\q"\n',
                'root ::= "a"\nroot ::= "b"\n', '::= "a"\n']:
        with pytest.raises(oracle.EBNFError):
            oracle.parse_ebnf(bad)
    with pytest.raises(ValueError):
        oracle.Oracle('root ::= "a" b\nb ::= "x" b\n')            # b derives nothing: not reduced
    with pytest.raises(ValueError):
        oracle.Oracle('root ::= TagDispatch(("<a>", g), ("x<a>y", g))\ng ::= "k"\n')   # tag inside a tag
