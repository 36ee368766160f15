// EBNF -> canonical minimal per-rule automata -> structural hashes.  Host code only.
#include "grammar.hpp"

#include <algorithm>
#include <queue>
#include <array>
#include <atomic>
#include <cstring>
#include <deque>
#include <functional>
#include <map>
#include <memory>
#include <mutex>
#include <set>
#include <sstream>
#include <unordered_map>

namespace xg2 {
namespace {

// ------------------------------------------------------------------------------------------------
// byte sets
struct ByteSet {
    uint64_t w[4] = {0, 0, 0, 0};
    void set(int b) { w[b >> 6] |= 1ull << (b & 63); }
    void set_range(int lo, int hi) { for (int b = lo; b <= hi; ++b) set(b); }
    bool test(int b) const { return (w[b >> 6] >> (b & 63)) & 1ull; }
};

// ------------------------------------------------------------------------------------------------
// syntax tree of the EBNF dialect
enum class NK { Lit, Cls, Ref, Seq, Alt, Rep, Tag };
struct Node {
    NK k = NK::Seq;
    std::vector<uint32_t> cps;                                  // Lit: code points
    bool neg = false;                                           // Cls
    std::vector<std::pair<uint32_t, uint32_t>> ranges;          // Cls: scalar ranges as written
    std::string name;                                           // Ref
    std::vector<Node> kids;                                     // Seq / Alt / Rep (one kid)
    int m = 0, n = -1;                                          // Rep: n < 0 = unbounded
    std::vector<std::pair<std::string, std::string>> tags;      // Tag: (tag bytes, rule name)
    std::vector<std::string> stops;                             // Tag: stop strings (bytes)
};

void append_utf8(std::string& out, uint32_t cp) {
    if (cp < 0x80) out.push_back((char)cp);
    else if (cp < 0x800) { out.push_back((char)(0xC0 | (cp >> 6))); out.push_back((char)(0x80 | (cp & 63))); }
    else if (cp < 0x10000) {
        out.push_back((char)(0xE0 | (cp >> 12))); out.push_back((char)(0x80 | ((cp >> 6) & 63)));
        out.push_back((char)(0x80 | (cp & 63)));
    } else {
        out.push_back((char)(0xF0 | (cp >> 18))); out.push_back((char)(0x80 | ((cp >> 12) & 63)));
        out.push_back((char)(0x80 | ((cp >> 6) & 63))); out.push_back((char)(0x80 | (cp & 63)));
    }
}

class Parser {
  public:
    explicit Parser(const std::string& s) : s_(s) {}

    void parse(std::vector<std::string>& order, std::map<std::string, Node>& rules) {
        while (peek() != 0) {
            std::string nm;
            if (!name(nm)) fail("rule name expected");
            expect("::=");
            skip();
            size_t save = i_;
            std::string head;
            Node body;
            if (name(head) && head == "TagDispatch" && peek() == '(') body = tagdispatch();
            else { i_ = save; body = alternation(); }
            if (peek() != 0 && !at_rule_head()) fail("unexpected text after rule body");
            if (rules.count(nm)) fail("rule " + nm + " defined twice");
            order.push_back(nm);
            rules.emplace(nm, std::move(body));
        }
    }

  private:
    const std::string& s_;
    size_t i_ = 0;

    [[noreturn]] void fail(const std::string& msg) const {
        size_t line = 1 + (size_t)std::count(s_.begin(), s_.begin() + (long)std::min(i_, s_.size()), '\n');
        throw ParseError("line " + std::to_string(line) + ": " + msg);
    }
    void skip() {
        while (i_ < s_.size()) {
            char c = s_[i_];
            if (c == ' ' || c == '\t' || c == '\r' || c == '\n') ++i_;
            else if (c == '#') { while (i_ < s_.size() && s_[i_] != '\n') ++i_; }
            else break;
        }
    }
    char peek() { skip(); return i_ < s_.size() ? s_[i_] : 0; }
    static bool name_start(char c) { return (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || c == '_'; }
    static bool name_cont(char c) { return name_start(c) || (c >= '0' && c <= '9') || c == '.' || c == '-'; }
    bool name(std::string& out) {
        skip();
        size_t j = i_;
        if (j < s_.size() && name_start(s_[j])) {
            ++j;
            while (j < s_.size() && name_cont(s_[j])) ++j;
            out = s_.substr(i_, j - i_);
            i_ = j;
            return true;
        }
        return false;
    }
    bool at_rule_head() {
        size_t save = i_;
        std::string nm;
        bool ok = false;
        if (name(nm)) { skip(); ok = s_.compare(i_, 3, "::=") == 0; }
        i_ = save;
        return ok;
    }
    void expect(const char* tok) {
        skip();
        size_t n = std::strlen(tok);
        if (s_.compare(i_, n, tok) != 0) fail(std::string("'") + tok + "' expected");
        i_ += n;
    }
    // one source character as a code point (the grammar text is UTF-8)
    uint32_t source_char() {
        unsigned char c = (unsigned char)s_[i_];
        int n = c < 0x80 ? 1 : (c >> 5) == 6 ? 2 : (c >> 4) == 14 ? 3 : (c >> 3) == 30 ? 4 : 0;
        if (n == 0 || i_ + (size_t)n > s_.size()) fail("grammar text is not valid UTF-8");
        uint32_t cp = n == 1 ? c : (c & (0xFF >> (n + 1)));
        for (int k = 1; k < n; ++k) {
            unsigned char d = (unsigned char)s_[i_ + (size_t)k];
            if ((d & 0xC0) != 0x80) fail("grammar text is not valid UTF-8");
            cp = (cp << 6) | (d & 63);
        }
        i_ += (size_t)n;
        return cp;
    }
    uint32_t escape(bool in_class) {
        if (i_ >= s_.size()) fail("dangling backslash");
        char c = s_[i_++];
        switch (c) {
            case '"': return 34; case '\\': return 92; case 'n': return 10; case 't': return 9;
            case 'r': return 13; case '/': return 47; case '\'': return 39;
            default: break;
        }
        if (in_class && (c == '-' || c == ']' || c == '[' || c == '^')) return (uint32_t)c;
        int width = c == 'x' ? 2 : c == 'u' ? 4 : c == 'U' ? 8 : 0;
        if (!width) fail(std::string("unknown escape \\") + c);
        if (i_ + (size_t)width > s_.size()) fail("bad hex escape");
        uint32_t cp = 0;
        for (int k = 0; k < width; ++k) {
            char h = s_[i_++];
            int v = h >= '0' && h <= '9' ? h - '0' : h >= 'a' && h <= 'f' ? h - 'a' + 10 : h >= 'A' && h <= 'F' ? h - 'A' + 10 : -1;
            if (v < 0) fail("bad hex escape");
            cp = cp * 16 + (uint32_t)v;
        }
        if (cp > 0x10FFFF || (cp >= 0xD800 && cp <= 0xDFFF)) fail("escape is not a Unicode scalar value");
        return cp;
    }
    std::vector<uint32_t> literal() {
        ++i_;                                                   // opening quote
        std::vector<uint32_t> out;
        for (;;) {
            if (i_ >= s_.size()) fail("unterminated literal");
            char c = s_[i_];
            if (c == '"') { ++i_; return out; }
            if (c == '\\') { ++i_; out.push_back(escape(false)); }
            else out.push_back(source_char());
        }
    }
    Node char_class() {
        ++i_;                                                   // '['
        Node n; n.k = NK::Cls;
        if (i_ < s_.size() && s_[i_] == '^') { n.neg = true; ++i_; }
        auto one = [&]() -> uint32_t {
            if (i_ >= s_.size()) fail("unterminated class");
            if (s_[i_] == '\\') { ++i_; return escape(true); }
            return source_char();
        };
        for (;;) {
            if (i_ >= s_.size()) fail("unterminated class");
            if (s_[i_] == ']') { ++i_; break; }
            uint32_t lo = one(), hi = lo;
            if (i_ + 1 < s_.size() && s_[i_] == '-' && s_[i_ + 1] != ']') {
                ++i_;
                hi = one();
                if (hi < lo) fail("reversed range in class");
            }
            n.ranges.emplace_back(lo, hi);
        }
        return n;
    }
    int number() {
        skip();
        size_t j = i_;
        long v = 0;
        while (j < s_.size() && s_[j] >= '0' && s_[j] <= '9') { v = v * 10 + (s_[j] - '0'); if (v > 1000000) fail("repetition bound too large"); ++j; }
        if (j == i_) fail("number expected");
        i_ = j;
        return (int)v;
    }
    Node atom() {
        char c = peek();
        if (c == '"') { Node n; n.k = NK::Lit; n.cps = literal(); return n; }
        if (c == '[') return char_class();
        if (c == '(') {
            ++i_;
            Node n = alternation();
            if (peek() != ')') fail("')' expected");
            ++i_;
            return n;
        }
        Node n; n.k = NK::Ref;
        if (!name(n.name)) fail(std::string("unexpected character '") + c + "'");
        return n;
    }
    static Node rep(Node x, int m, int n) {
        Node r; r.k = NK::Rep; r.m = m; r.n = n; r.kids.push_back(std::move(x));
        return r;
    }
    Node term() {
        Node a = atom();
        for (;;) {
            char c = peek();
            if (c == '*') { ++i_; a = rep(std::move(a), 0, -1); }
            else if (c == '+') { ++i_; a = rep(std::move(a), 1, -1); }
            else if (c == '?') { ++i_; a = rep(std::move(a), 0, 1); }
            else if (c == '{') {
                ++i_;
                int m = number(), n = m;
                if (peek() == ',') { ++i_; n = peek() == '}' ? -1 : number(); }
                if (peek() != '}') fail("'}' expected");
                ++i_;
                if (n >= 0 && n < m) fail("repetition bounds reversed");
                a = rep(std::move(a), m, n);
            } else return a;
        }
    }
    Node sequence() {
        Node s; s.k = NK::Seq;
        for (;;) {
            char c = peek();
            if (c == 0 || c == '|' || c == ')' || at_rule_head()) break;
            s.kids.push_back(term());
        }
        if (s.kids.size() == 1) { Node only = std::move(s.kids[0]); return only; }
        return s;
    }
    Node alternation() {
        Node a; a.k = NK::Alt;
        a.kids.push_back(sequence());
        while (peek() == '|') { ++i_; a.kids.push_back(sequence()); }
        if (a.kids.size() == 1) { Node only = std::move(a.kids[0]); return only; }
        return a;
    }
    static std::string to_bytes(const std::vector<uint32_t>& cps) {
        std::string out;
        for (uint32_t c : cps) append_utf8(out, c);
        return out;
    }
    Node tagdispatch() {
        Node t; t.k = NK::Tag;
        expect("(");
        for (;;) {
            char c = peek();
            if (c == '(') {
                ++i_;
                if (peek() != '"') fail("tag literal expected");
                std::string tag = to_bytes(literal());
                expect(",");
                std::string nm;
                if (!name(nm)) fail("rule name expected");
                expect(")");
                t.tags.emplace_back(tag, nm);
            } else if (s_.compare(i_, 9, "stop_strs") == 0) {
                i_ += 9;
                expect("="); expect("(");
                while (peek() == '"') { t.stops.push_back(to_bytes(literal())); if (peek() == ',') ++i_; }
                expect(")");
            } else fail("tag pair or stop_strs expected");
            if (peek() == ',') { ++i_; continue; }
            break;
        }
        expect(")");
        return t;
    }
};

// ------------------------------------------------------------------------------------------------
// character classes: scalar ranges -> sequences of byte ranges (UTF-8, shortest form, no surrogates)
using ScalarRanges = std::vector<std::pair<uint32_t, uint32_t>>;

ScalarRanges normalise_class(bool neg, ScalarRanges rs) {
    std::sort(rs.begin(), rs.end());
    ScalarRanges merged;
    for (auto& r : rs) {
        if (!merged.empty() && r.first <= merged.back().second + 1) merged.back().second = std::max(merged.back().second, r.second);
        else merged.push_back(r);
    }
    if (neg) {
        ScalarRanges out;
        uint32_t prev = 0;
        for (auto& r : merged) { if (r.first > prev) out.emplace_back(prev, r.first - 1); prev = r.second + 1; }
        if (prev <= 0x10FFFF) out.emplace_back(prev, 0x10FFFF);
        merged.swap(out);
    }
    ScalarRanges fin;
    for (auto r : merged) {
        r.second = std::min<uint32_t>(r.second, 0x10FFFF);
        if (r.first > r.second) continue;
        if (r.second < 0xD800 || r.first > 0xDFFF) { fin.push_back(r); continue; }
        if (r.first < 0xD800) fin.emplace_back(r.first, 0xD7FF);
        if (r.second > 0xDFFF) fin.emplace_back(0xE000, r.second);
    }
    return fin;
}

struct ByteSeq { int n; uint8_t lo[4], hi[4]; };

// [lo, hi] encodes to `len` bytes throughout; cut it until each piece is a product of byte ranges.
void split_same_length(uint32_t lo, uint32_t hi, int len, std::vector<ByteSeq>& out) {
    for (int i = 1; i < len; ++i) {
        uint32_t m = (1u << (6 * i)) - 1;
        if ((lo & ~m) != (hi & ~m)) {
            if ((lo & m) != 0) {
                split_same_length(lo, lo | m, len, out);
                split_same_length((lo | m) + 1, hi, len, out);
                return;
            }
            if ((hi & m) != m) {
                split_same_length(lo, (hi & ~m) - 1, len, out);
                split_same_length(hi & ~m, hi, len, out);
                return;
            }
        }
    }
    std::string a, b;
    append_utf8(a, lo);
    append_utf8(b, hi);
    ByteSeq s; s.n = len;
    for (int k = 0; k < len; ++k) { s.lo[k] = (uint8_t)a[(size_t)k]; s.hi[k] = (uint8_t)b[(size_t)k]; }
    out.push_back(s);
}

std::vector<ByteSeq> class_byte_sequences(bool neg, const ScalarRanges& written) {
    static const uint32_t bound[5] = {0, 0x7F, 0x7FF, 0xFFFF, 0x10FFFF};
    std::vector<ByteSeq> out;
    for (auto r : normalise_class(neg, written))
        for (int len = 1; len <= 4; ++len) {
            uint32_t lo = std::max(r.first, bound[len - 1] + (len > 1 ? 1u : 0u));
            uint32_t hi = std::min(r.second, bound[len]);
            if (lo <= hi) split_same_length(lo, hi, len, out);
        }
    return out;
}

// ------------------------------------------------------------------------------------------------
// Thompson construction over the alphabet {bytes} U {rule symbols}
struct NEdge { int kind; ByteSet set; int rule; int dst; };   // kind 0 epsilon, 1 bytes, 2 rule symbol
struct Nfa {
    std::vector<std::vector<NEdge>> e;
    int add() { e.emplace_back(); return (int)e.size() - 1; }
    void eps(int a, int b) { e[(size_t)a].push_back({0, ByteSet(), -1, b}); }
    void bytes(int a, const ByteSet& s, int b) { e[(size_t)a].push_back({1, s, -1, b}); }
    void rule(int a, int r, int b) { e[(size_t)a].push_back({2, ByteSet(), r, b}); }
};

void build_nfa(const Node& nd, Nfa& nfa, int s, int e, const std::map<std::string, int>& index) {
    switch (nd.k) {
        case NK::Lit: {
            std::string data;
            for (uint32_t c : nd.cps) append_utf8(data, c);
            int cur = s;
            for (unsigned char b : data) { int nx = nfa.add(); ByteSet bs; bs.set(b); nfa.bytes(cur, bs, nx); cur = nx; }
            nfa.eps(cur, e);
            break;
        }
        case NK::Cls: {
            for (const ByteSeq& q : class_byte_sequences(nd.neg, nd.ranges)) {
                int cur = s;
                for (int k = 0; k < q.n; ++k) {
                    int nx = k + 1 == q.n ? e : nfa.add();
                    ByteSet bs; bs.set_range(q.lo[k], q.hi[k]);
                    nfa.bytes(cur, bs, nx);
                    cur = nx;
                }
            }
            break;
        }
        case NK::Ref: {
            auto it = index.find(nd.name);
            if (it == index.end()) throw GrammarError("undefined rule " + nd.name);
            nfa.rule(s, it->second, e);
            break;
        }
        case NK::Seq: {
            int cur = s;
            for (const Node& c : nd.kids) { int a = nfa.add(), b = nfa.add(); build_nfa(c, nfa, a, b, index); nfa.eps(cur, a); cur = b; }
            nfa.eps(cur, e);
            break;
        }
        case NK::Alt:
            for (const Node& c : nd.kids) { int a = nfa.add(), b = nfa.add(); build_nfa(c, nfa, a, b, index); nfa.eps(s, a); nfa.eps(b, e); }
            break;
        case NK::Rep: {
            const Node& x = nd.kids[0];
            int cur = s;
            for (int k = 0; k < nd.m; ++k) { int a = nfa.add(), b = nfa.add(); build_nfa(x, nfa, a, b, index); nfa.eps(cur, a); cur = b; }
            if (nd.n < 0) {
                int a = nfa.add(), b = nfa.add();
                build_nfa(x, nfa, a, b, index);
                nfa.eps(cur, a); nfa.eps(b, cur); nfa.eps(cur, e);
            } else {
                nfa.eps(cur, e);
                for (int k = nd.m; k < nd.n; ++k) {
                    int a = nfa.add(), b = nfa.add();
                    build_nfa(x, nfa, a, b, index);
                    nfa.eps(cur, a); cur = b; nfa.eps(cur, e);
                }
            }
            break;
        }
        case NK::Tag: throw GrammarError("TagDispatch must be the whole body of a rule");
    }
}

// ------------------------------------------------------------------------------------------------
// deterministic automaton with dense rows over byte classes (one rule at a time, so the memory is transient).
// Bytes of one class behave alike in every state; classes are numbered in the order of their smallest byte, so
// visiting the classes in ascending order visits targets in the order of ascending bytes.
struct Dfa {
    int ncls = 1;
    std::array<uint8_t, 256> cls{};                           // byte -> class
    std::vector<int32_t> bt;                                  // [state * ncls + class] -> target or -1
    std::vector<std::vector<std::pair<int, int>>> rt;         // (rule decl index, target), sorted by rule
    std::vector<uint8_t> fin;
    int start = 0;
    int add(bool f) {
        bt.resize(bt.size() + (size_t)ncls, -1);
        rt.emplace_back(); fin.push_back(f ? 1 : 0);
        return (int)fin.size() - 1;
    }
    int n() const { return (int)fin.size(); }
    int32_t& at(int q, int c) { return bt[(size_t)q * (size_t)ncls + (size_t)c]; }
    int32_t at(int q, int c) const { return bt[(size_t)q * (size_t)ncls + (size_t)c]; }
    int32_t byte_target(int q, int b) const { return at(q, cls[(size_t)b]); }
    // classes from a list of byte sets: two bytes are alike if they are in the same sets
    void classes_from(const std::vector<ByteSet>& sets) {
        std::vector<std::vector<uint8_t>> sig(256);
        for (size_t k = 0; k < sets.size(); ++k)
            for (int b = 0; b < 256; ++b) if (sets[k].test(b)) { if (sig[(size_t)b].size() <= k / 8) sig[(size_t)b].resize(k / 8 + 1, 0); sig[(size_t)b][k / 8] |= (uint8_t)(1u << (k % 8)); }
        std::map<std::vector<uint8_t>, int> ids;
        ncls = 0;
        for (int b = 0; b < 256; ++b) {
            auto it = ids.find(sig[(size_t)b]);
            if (it == ids.end()) it = ids.emplace(sig[(size_t)b], ncls++).first;
            cls[(size_t)b] = (uint8_t)it->second;
        }
    }
};

Dfa subset_construction(const Nfa& nfa, int start, int end) {
    std::vector<int> stamp(nfa.e.size(), -1);
    int tick = 0;
    auto closure = [&](std::vector<int> seed) {
        ++tick;
        std::vector<int> out, stack;
        for (int q : seed) if (stamp[(size_t)q] != tick) { stamp[(size_t)q] = tick; out.push_back(q); stack.push_back(q); }
        while (!stack.empty()) {
            int q = stack.back(); stack.pop_back();
            for (const NEdge& ed : nfa.e[(size_t)q])
                if (ed.kind == 0 && stamp[(size_t)ed.dst] != tick) { stamp[(size_t)ed.dst] = tick; out.push_back(ed.dst); stack.push_back(ed.dst); }
        }
        std::sort(out.begin(), out.end());
        return out;
    };
    Dfa d;
    {   // byte classes of the whole automaton: the distinct byte sets on its edges
        std::vector<ByteSet> sets;
        std::set<std::array<uint64_t, 4>> seen;
        for (auto& es : nfa.e)
            for (const NEdge& ed : es)
                if (ed.kind == 1 && seen.insert({ed.set.w[0], ed.set.w[1], ed.set.w[2], ed.set.w[3]}).second) sets.push_back(ed.set);
        d.classes_from(sets);
    }
    std::vector<int> rep_byte((size_t)d.ncls, 0);
    for (int b = 255; b >= 0; --b) rep_byte[d.cls[(size_t)b]] = b;
    std::map<std::vector<int>, int> ids;
    std::vector<std::vector<int>> sets;
    auto intern = [&](std::vector<int> S) {
        auto it = ids.find(S);
        if (it != ids.end()) return it->second;
        int id = d.add(std::binary_search(S.begin(), S.end(), end));
        ids.emplace(S, id);
        sets.push_back(std::move(S));
        return id;
    };
    intern(closure({start}));
    for (size_t cur = 0; cur < sets.size(); ++cur) {
        std::vector<const NEdge*> bedges;
        std::map<int, std::vector<int>> by_rule;
        for (int q : sets[cur])
            for (const NEdge& ed : nfa.e[(size_t)q]) {
                if (ed.kind == 1) bedges.push_back(&ed);
                else if (ed.kind == 2) by_rule[ed.rule].push_back(ed.dst);
            }
        // classes with the same set of matching edges go to the same target
        std::vector<std::pair<std::vector<int>, int>> seen;        // matching edges -> target: few per state
        std::vector<int> hit;
        for (int c = 0; c < d.ncls; ++c) {
            hit.clear();
            for (size_t k = 0; k < bedges.size(); ++k) if (bedges[k]->set.test(rep_byte[(size_t)c])) hit.push_back((int)k);
            if (hit.empty()) continue;
            int t = -1;
            for (auto& sm : seen) if (sm.first == hit) { t = sm.second; break; }
            if (t < 0) {
                std::vector<int> seed;
                for (int k : hit) seed.push_back(bedges[(size_t)k]->dst);
                t = intern(closure(seed));
                seen.emplace_back(hit, t);
            }
            d.at((int)cur, c) = t;
        }
        for (auto& r : by_rule) { int t = intern(closure(r.second)); d.rt[cur].emplace_back(r.first, t); }
    }
    d.start = 0;
    return d;
}

// TagDispatch (section 3.2) as an Aho-Corasick automaton: goto trie over tags and stop strings,
// failure links, transitions completed so that every byte is free text; completing a tag leads to
// a state whose only edge is the tag's rule and returns to the trie root; completing a stop string
// leads to the single final exit state.  Without stop strings every dispatching state is final.
Dfa tagdispatch_automaton(const Node& nd, const std::map<std::string, int>& index) {
    std::vector<std::string> pats;
    for (auto& t : nd.tags) pats.push_back(t.first);
    for (auto& s : nd.stops) pats.push_back(s);
    if (nd.tags.empty()) throw GrammarError("TagDispatch needs at least one tag");
    for (size_t a = 0; a < pats.size(); ++a) {
        if (pats[a].empty()) throw GrammarError("empty tag or stop string");
        for (size_t b = 0; b < pats.size(); ++b)
            if (a != b && pats[b].find(pats[a]) != std::string::npos)
                throw GrammarError("a tag or stop string occurs inside another one");
    }
    struct TNode { std::map<unsigned char, int> kid; int pat = -1; int fail = 0; };
    std::vector<TNode> trie(1);
    for (size_t p = 0; p < pats.size(); ++p) {
        int cur = 0;
        for (unsigned char c : pats[p]) {
            auto it = trie[(size_t)cur].kid.find(c);
            if (it == trie[(size_t)cur].kid.end()) { trie.emplace_back(); int id = (int)trie.size() - 1; trie[(size_t)cur].kid[c] = id; cur = id; }
            else cur = it->second;
        }
        trie[(size_t)cur].pat = (int)p;
    }
    // dense goto over breadth-first order, failure transitions folded in
    std::vector<std::array<int, 256>> go(trie.size());
    std::deque<int> bfs;
    for (int c = 0; c < 256; ++c) {
        auto it = trie[0].kid.find((unsigned char)c);
        go[0][(size_t)c] = it == trie[0].kid.end() ? 0 : it->second;
        if (it != trie[0].kid.end()) { trie[(size_t)it->second].fail = 0; bfs.push_back(it->second); }
    }
    while (!bfs.empty()) {
        int u = bfs.front(); bfs.pop_front();
        for (int c = 0; c < 256; ++c) {
            auto it = trie[(size_t)u].kid.find((unsigned char)c);
            if (it == trie[(size_t)u].kid.end()) go[(size_t)u][(size_t)c] = go[(size_t)trie[(size_t)u].fail][(size_t)c];
            else {
                int v = it->second;
                trie[(size_t)v].fail = go[(size_t)trie[(size_t)u].fail][(size_t)c];
                go[(size_t)u][(size_t)c] = v;
                bfs.push_back(v);
            }
        }
    }
    Dfa d;
    {   // every byte of a tag or stop string is a class of its own, all other bytes are one class
        std::vector<ByteSet> sets;
        bool used[256] = {false};
        for (auto& pat : pats) for (unsigned char c : pat) if (!used[c]) { used[c] = true; ByteSet bs; bs.set(c); sets.push_back(bs); }
        d.classes_from(sets);
    }
    bool no_stops = nd.stops.empty();
    std::vector<int> state_of(trie.size(), -1);
    for (size_t u = 0; u < trie.size(); ++u) if (trie[u].pat < 0) state_of[u] = d.add(no_stops);
    std::vector<int> after_tag(nd.tags.size());
    for (size_t k = 0; k < nd.tags.size(); ++k) {
        auto it = index.find(nd.tags[k].second);
        if (it == index.end()) throw GrammarError("undefined rule " + nd.tags[k].second);
        after_tag[k] = d.add(false);
        d.rt[(size_t)after_tag[k]].emplace_back(it->second, state_of[0]);
    }
    int exit_state = no_stops ? -1 : d.add(true);
    for (size_t u = 0; u < trie.size(); ++u) {
        if (trie[u].pat >= 0) continue;
        for (int c = 0; c < 256; ++c) {
            int v = go[u][(size_t)c];
            int p = trie[(size_t)v].pat;
            d.at(state_of[u], d.cls[(size_t)c]) = p < 0 ? state_of[(size_t)v] : (size_t)p < nd.tags.size() ? after_tag[(size_t)p] : exit_state;
        }
    }
    d.start = state_of[0];
    return d;
}

// Trim (reachable and able to reach a final state), Hopcroft partition refinement with bytes that
// behave alike everywhere treated as one symbol, then canonical breadth-first renaming: out-edges
// visited by ascending byte, then by ascending declaration index of the referenced rule.
Dfa minimise_canonical(const Dfa& in, const std::string& rule_name) {
    int n0 = in.n();
    const int nc0 = in.ncls;
    std::vector<uint8_t> reach((size_t)n0, 0), live((size_t)n0, 0);
    std::vector<int> stack{in.start};
    reach[(size_t)in.start] = 1;
    std::vector<std::vector<int>> rev((size_t)n0);
    while (!stack.empty()) {
        int q = stack.back(); stack.pop_back();
        auto visit = [&](int t) { if (t >= 0 && !reach[(size_t)t]) { reach[(size_t)t] = 1; stack.push_back(t); } };
        for (int c = 0; c < nc0; ++c) visit(in.at(q, c));
        for (auto& r : in.rt[(size_t)q]) visit(r.second);
    }
    for (int q = 0; q < n0; ++q) {
        if (!reach[(size_t)q]) continue;
        int last = -1;
        for (int c = 0; c < nc0; ++c) { int t = in.at(q, c); if (t >= 0 && t != last) { rev[(size_t)t].push_back(q); last = t; } }
        for (auto& r : in.rt[(size_t)q]) rev[(size_t)r.second].push_back(q);
    }
    for (int q = 0; q < n0; ++q) if (reach[(size_t)q] && in.fin[(size_t)q]) { live[(size_t)q] = 1; stack.push_back(q); }
    while (!stack.empty()) {
        int q = stack.back(); stack.pop_back();
        for (int p : rev[(size_t)q]) if (!live[(size_t)p]) { live[(size_t)p] = 1; stack.push_back(p); }
    }
    if (!live[(size_t)in.start]) throw GrammarError("rule " + rule_name + " has an empty language");
    std::vector<int> keep_id((size_t)n0, -1), keep;
    for (int q = 0; q < n0; ++q) if (reach[(size_t)q] && live[(size_t)q]) { keep_id[(size_t)q] = (int)keep.size(); keep.push_back(q); }
    int n = (int)keep.size();

    // byte classes: two input classes merge if they lead to the same target in every kept state.  New classes are
    // numbered by first occurrence over ascending input classes, i.e. still by their smallest byte.
    std::vector<int> cclass((size_t)nc0, 0);                   // input class -> class so far
    int nclass = 1;
    {
        struct Split { int old_class, target, new_class; };
        std::vector<Split> splits;                                  // few per state: searched linearly
        for (int q : keep) {
            splits.clear();
            for (int c = 0; c < nc0; ++c) {
                int t = in.at(q, c);
                t = t >= 0 ? keep_id[(size_t)t] : -1;
                const int oc = cclass[(size_t)c];
                int nc = -1;
                for (const Split& sp : splits) if (sp.old_class == oc && sp.target == t) { nc = sp.new_class; break; }
                if (nc < 0) { nc = (int)splits.size(); splits.push_back({oc, t, nc}); }
                cclass[(size_t)c] = nc;
            }
            nclass = std::max(nclass, (int)splits.size());
        }
    }
    std::vector<int> class_rep((size_t)nclass, 0);              // an input class of each class
    for (int c = nc0 - 1; c >= 0; --c) class_rep[(size_t)cclass[(size_t)c]] = c;
    std::vector<int> rule_syms;
    for (int q : keep) for (auto& r : in.rt[(size_t)q]) if (keep_id[(size_t)r.second] >= 0) rule_syms.push_back(r.first);
    std::sort(rule_syms.begin(), rule_syms.end());
    rule_syms.erase(std::unique(rule_syms.begin(), rule_syms.end()), rule_syms.end());
    int nsym = nclass + (int)rule_syms.size();
    std::vector<int> delta((size_t)n * (size_t)nsym, -1);
    for (int i = 0; i < n; ++i) {
        int q = keep[(size_t)i];
        for (int c = 0; c < nclass; ++c) { int t = in.at(q, class_rep[(size_t)c]); delta[(size_t)i * nsym + c] = t >= 0 ? keep_id[(size_t)t] : -1; }
        for (auto& r : in.rt[(size_t)q]) {
            int t = keep_id[(size_t)r.second];
            if (t < 0) continue;
            int s = nclass + (int)(std::lower_bound(rule_syms.begin(), rule_syms.end(), r.first) - rule_syms.begin());
            delta[(size_t)i * nsym + s] = t;
        }
    }
    // inverse transitions: for target t, list of (symbol, source)
    std::vector<std::vector<std::pair<int, int>>> inv((size_t)n);
    for (int i = 0; i < n; ++i)
        for (int s = 0; s < nsym; ++s) { int t = delta[(size_t)i * nsym + s]; if (t >= 0) inv[(size_t)t].emplace_back(s, i); }

    std::vector<int> block_of((size_t)n);
    std::vector<std::vector<int>> blocks;
    {
        std::vector<int> f, nf;
        for (int i = 0; i < n; ++i) (in.fin[(size_t)keep[(size_t)i]] ? f : nf).push_back(i);
        if (!f.empty()) blocks.push_back(f);
        if (!nf.empty()) blocks.push_back(nf);
        for (size_t b = 0; b < blocks.size(); ++b) for (int i : blocks[b]) block_of[(size_t)i] = (int)b;
    }
    std::deque<int> work;
    std::vector<uint8_t> in_work(blocks.size(), 1);
    for (size_t b = 0; b < blocks.size(); ++b) work.push_back((int)b);
    std::vector<int> mark_count, touched;
    std::vector<uint8_t> marked((size_t)n, 0);
    std::vector<std::vector<int>> pre((size_t)nsym);
    while (!work.empty()) {
        int B = work.front(); work.pop_front();
        in_work[(size_t)B] = 0;
        std::vector<int> used_syms;
        for (int t : blocks[(size_t)B])
            for (auto& e : inv[(size_t)t]) { if (pre[(size_t)e.first].empty()) used_syms.push_back(e.first); pre[(size_t)e.first].push_back(e.second); }
        for (int s : used_syms) {
            std::vector<int>& X = pre[(size_t)s];
            mark_count.resize(blocks.size(), 0);                  // all zero here: the touched entries are cleared below
            touched.clear();
            for (int q : X) { if (!marked[(size_t)q]) { marked[(size_t)q] = 1; int b = block_of[(size_t)q]; if (mark_count[(size_t)b]++ == 0) touched.push_back(b); } }
            for (int Y : touched) {
                if (mark_count[(size_t)Y] == (int)blocks[(size_t)Y].size()) continue;
                std::vector<int> in_x, out_x;
                for (int q : blocks[(size_t)Y]) (marked[(size_t)q] ? in_x : out_x).push_back(q);
                bool new_is_in = in_x.size() <= out_x.size();
                std::vector<int>& small = new_is_in ? in_x : out_x;
                std::vector<int>& large = new_is_in ? out_x : in_x;
                int nb = (int)blocks.size();
                for (int q : small) block_of[(size_t)q] = nb;
                blocks[(size_t)Y] = large;
                blocks.push_back(small);
                in_work.push_back(1);
                work.push_back(nb);                              // Y keeps the larger half (and stays queued if it was)
            }
            for (int Y : touched) mark_count[(size_t)Y] = 0;
            for (int q : X) marked[(size_t)q] = 0;
            X.clear();
        }
    }
    // quotient automaton over the merged classes, renamed breadth-first on the way: out-edges by ascending class
    // (= ascending smallest byte), then by rule
    int nb = (int)blocks.size();
    const int start_block = block_of[(size_t)keep_id[(size_t)in.start]];
    auto class_target = [&](int b, int c) { int t = delta[(size_t)blocks[(size_t)b][0] * nsym + c]; return t >= 0 ? block_of[(size_t)t] : -1; };
    auto rule_target = [&](int b, size_t r) { int t = delta[(size_t)blocks[(size_t)b][0] * nsym + nclass + (int)r]; return t >= 0 ? block_of[(size_t)t] : -1; };
    std::vector<int> ident((size_t)nb, -1), order{start_block};
    ident[(size_t)start_block] = 0;
    for (size_t k = 0; k < order.size(); ++k) {
        int q = order[k];
        auto visit = [&](int t) { if (t >= 0 && ident[(size_t)t] < 0) { ident[(size_t)t] = (int)order.size(); order.push_back(t); } };
        for (int c = 0; c < nclass; ++c) visit(class_target(q, c));
        for (size_t r = 0; r < rule_syms.size(); ++r) visit(rule_target(q, r));
    }
    Dfa out;
    out.ncls = nclass;
    for (int b = 0; b < 256; ++b) out.cls[(size_t)b] = (uint8_t)cclass[(size_t)in.cls[(size_t)b]];
    for (int q : order) out.add(in.fin[(size_t)keep[(size_t)blocks[(size_t)q][0]]]);
    for (size_t k = 0; k < order.size(); ++k) {
        int q = order[k];
        for (int c = 0; c < nclass; ++c) { int t = class_target(q, c); out.at((int)k, c) = t >= 0 ? ident[(size_t)t] : -1; }
        for (size_t r = 0; r < rule_syms.size(); ++r) { int t = rule_target(q, r); if (t >= 0) out.rt[k].emplace_back(rule_syms[r], ident[(size_t)t]); }
    }
    out.start = 0;
    return out;
}

// ------------------------------------------------------------------------------------------------
// structural hashing (Algorithm 1, Algorithm 2)
constexpr uint64_t NODE_TAG = 0xA1, RANGE_TAG = 0xB2, REF_TAG = 0xC3;

void put_u64(std::string& s, uint64_t v) { for (int k = 0; k < 8; ++k) s.push_back((char)((v >> (8 * k)) & 0xFF)); }

// Algorithm 1 on one rule.  ref_hash[r] = hash of referenced rule r (kInCycleRef for the unresolved
// in-cycle reference).  Fills canon_id and redges_by_hash, returns the hash.
uint64_t hash_one_fsm(RuleFsm& f, const std::vector<uint64_t>& ref_hash) {
    int n = f.n_states();
    // phase 1: out-edges sorted (ranges by (min,max); references by hash), BFS canonical ids
    f.redges_by_hash.assign((size_t)n, {});
    for (int s = 0; s < n; ++s) {
        f.redges_by_hash[(size_t)s] = f.redges[(size_t)s];
        std::stable_sort(f.redges_by_hash[(size_t)s].begin(), f.redges_by_hash[(size_t)s].end(),
                         [&](const RefEdge& a, const RefEdge& b) { return ref_hash[(size_t)a.rule] < ref_hash[(size_t)b.rule]; });
    }
    f.canon_id.assign((size_t)n, -1);
    std::vector<int> order{0};
    f.canon_id[0] = 0;
    for (size_t k = 0; k < order.size(); ++k) {
        int s = order[k];
        auto visit = [&](int t) { if (f.canon_id[(size_t)t] < 0) { f.canon_id[(size_t)t] = (int)order.size(); order.push_back(t); } };
        for (auto& e : f.bedges[(size_t)s]) visit(e.tgt);       // already sorted by (lo, hi)
        for (auto& e : f.redges_by_hash[(size_t)s]) visit(e.tgt);
    }
    // phase 2
    uint64_t h = 0;
    for (int s : order) {
        h = hash_combine(hash_combine(h, NODE_TAG), f.is_final[(size_t)s]);
        for (auto& e : f.bedges[(size_t)s])
            h = hash_combine(hash_combine(hash_combine(hash_combine(h, RANGE_TAG), e.lo), e.hi), (uint64_t)f.canon_id[(size_t)e.tgt]);
        for (auto& e : f.redges_by_hash[(size_t)s])
            h = hash_combine(hash_combine(hash_combine(h, REF_TAG), ref_hash[(size_t)e.rule]), (uint64_t)f.canon_id[(size_t)e.tgt]);
    }
    return h;
}

std::atomic<uint64_t> g_unshareable_salt{1};

void hash_rules(Grammar& g) {
    int R = (int)g.rules.size();
    // reference graph and its strongly connected components (Tarjan; components come out callee-first)
    std::vector<std::vector<int>> refs((size_t)R);
    for (int r = 0; r < R; ++r) {
        std::set<int> s;
        for (auto& es : g.rules[(size_t)r].redges) for (auto& e : es) s.insert(e.rule);
        refs[(size_t)r].assign(s.begin(), s.end());
    }
    std::vector<int> idx((size_t)R, -1), low((size_t)R, 0), comp((size_t)R, -1), st;
    std::vector<uint8_t> on((size_t)R, 0);
    std::vector<std::vector<int>> comps;
    int counter = 0;
    std::function<void(int)> dfs = [&](int v) {
        idx[(size_t)v] = low[(size_t)v] = counter++;
        st.push_back(v); on[(size_t)v] = 1;
        for (int w : refs[(size_t)v]) {
            if (idx[(size_t)w] < 0) { dfs(w); low[(size_t)v] = std::min(low[(size_t)v], low[(size_t)w]); }
            else if (on[(size_t)w]) low[(size_t)v] = std::min(low[(size_t)v], idx[(size_t)w]);
        }
        if (low[(size_t)v] == idx[(size_t)v]) {
            comps.emplace_back();
            for (;;) { int w = st.back(); st.pop_back(); on[(size_t)w] = 0; comp[(size_t)w] = (int)comps.size() - 1; comps.back().push_back(w); if (w == v) break; }
        }
    };
    for (int r = 0; r < R; ++r) if (idx[(size_t)r] < 0) dfs(r);

    std::vector<uint64_t> hash((size_t)R, 0);
    for (auto& members : comps) {
        int c = comp[(size_t)members[0]];
        bool self_loop = false;
        for (int w : refs[(size_t)members[0]]) if (w == members[0]) self_loop = true;
        if (members.size() == 1 && !self_loop) {                 // acyclic part: bottom-up, Algorithm 1
            RuleFsm& f = g.rules[(size_t)members[0]];
            f.hash = hash[(size_t)members[0]] = hash_one_fsm(f, hash);
            g.hash_order.push_back(members);
            continue;
        }
        // is it a simple cycle?  every member references exactly one member, and those links form one ring
        std::vector<int> ring;
        bool simple = true;
        std::map<int, int> next;
        for (int v : members) {
            int cnt = 0, nx = -1;
            for (int w : refs[(size_t)v]) if (comp[(size_t)w] == c) { ++cnt; nx = w; }
            if (cnt != 1) simple = false;
            next[v] = nx;
        }
        if (simple) {
            int v = *std::min_element(members.begin(), members.end());
            for (size_t k = 0; k < members.size(); ++k) { ring.push_back(v); v = next[v]; }
            std::set<int> seen(ring.begin(), ring.end());
            if (seen.size() != members.size() || v != ring[0]) simple = false;
        }
        // local hashes with the shared placeholder on the unresolved in-cycle references
        std::vector<uint64_t> with_ph = hash;
        for (int v : members) with_ph[(size_t)v] = kInCycleRef;
        std::map<int, uint64_t> local;
        for (int v : members) local[v] = hash_one_fsm(g.rules[(size_t)v], with_ph);
        g.hash_order.push_back(simple ? ring : members);
        if (simple) {                                             // Algorithm 2
            size_t L = ring.size();
            for (size_t i = 0; i < L; ++i) {
                uint64_t H = 0;
                RuleFsm& f = g.rules[(size_t)ring[i]];
                for (size_t j = 0; j < L; ++j) { int v = ring[(i + j) % L]; H = hash_combine(H, local[v]); f.ring.push_back(v); }
                f.hash = hash[(size_t)ring[i]] = H;
            }
        } else {                                                  // not a simple cycle: never shared
            for (int v : members) {
                RuleFsm& f = g.rules[(size_t)v];
                f.shareable = false;
                f.hash = hash[(size_t)v] = hash_combine(local[v], 0xDEAD0000ull + g_unshareable_salt.fetch_add(1));
            }
        }
    }
}

}  // namespace

uint64_t hash_combine(uint64_t h, uint64_t v) {
    // order-sensitive: H(H(h, a), b) != H(H(h, b), a)
    uint64_t x = h ^ (v + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2));
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

std::string serialise_rule(const Grammar& g, int32_t rule, const std::vector<uint64_t>& ref_id) {
    const RuleFsm& f = g.rules[(size_t)rule];
    int n = f.n_states();
    std::vector<int> by_canon((size_t)n);
    for (int s = 0; s < n; ++s) by_canon[(size_t)f.canon_id[(size_t)s]] = s;
    std::string text;
    for (int s : by_canon) {
        text.push_back('N'); text.push_back((char)f.is_final[(size_t)s]);
        for (auto& e : f.bedges[(size_t)s]) {
            text.push_back('R'); text.push_back((char)e.lo); text.push_back((char)e.hi); put_u64(text, (uint64_t)f.canon_id[(size_t)e.tgt]);
        }
        for (auto& e : f.redges_by_hash[(size_t)s]) {
            text.push_back('F'); put_u64(text, ref_id[(size_t)e.rule]); put_u64(text, (uint64_t)f.canon_id[(size_t)e.tgt]);
        }
    }
    return text;
}

// ---- process-wide memo of lowered rule bodies ------------------------------------------------------------
std::mutex g_body_memo_mu;
std::unordered_map<std::string, std::shared_ptr<Dfa>> g_body_memo;

void collect_refs(const Node& nd, const std::map<std::string, int>& index, std::vector<int>& out, bool& ok) {
    auto add = [&](const std::string& name) { auto it = index.find(name); if (it == index.end()) ok = false; else out.push_back(it->second); };
    if (nd.k == NK::Ref) add(nd.name);
    for (auto& t : nd.tags) add(t.second);
    for (const Node& k : nd.kids) collect_refs(k, index, out, ok);
}

void body_key(const Node& nd, const std::map<std::string, int>& index, const std::vector<int>& ref_decl, std::string& out) {
    auto put = [&](uint64_t v) { for (int k = 0; k < 8; ++k) out.push_back((char)((v >> (8 * k)) & 0xFF)); };
    auto rank = [&](const std::string& name) { return (uint64_t)(std::lower_bound(ref_decl.begin(), ref_decl.end(), index.at(name)) - ref_decl.begin()); };
    out.push_back((char)('A' + (int)nd.k));
    switch (nd.k) {
        case NK::Lit: put(nd.cps.size()); for (uint32_t c : nd.cps) put(c); break;
        case NK::Cls: put(nd.neg); put(nd.ranges.size()); for (auto& r : nd.ranges) { put(r.first); put(r.second); } break;
        case NK::Ref: put(rank(nd.name)); break;
        case NK::Rep: put((uint64_t)(int64_t)nd.m); put((uint64_t)(int64_t)nd.n); break;
        case NK::Tag:
            put(nd.tags.size());
            for (auto& t : nd.tags) { put(t.first.size()); out += t.first; put(rank(t.second)); }
            put(nd.stops.size());
            for (auto& st : nd.stops) { put(st.size()); out += st; }
            break;
        default: break;
    }
    put(nd.kids.size());
    for (const Node& k : nd.kids) body_key(k, index, ref_decl, out);
}

Grammar lower_grammar(const std::string& ebnf, const std::string& root_rule) {
    std::vector<std::string> order;
    std::map<std::string, Node> rules;
    Parser(ebnf).parse(order, rules);
    std::map<std::string, int> index;
    for (size_t i = 0; i < order.size(); ++i) index[order[i]] = (int)i;
    if (!index.count(root_rule)) throw GrammarError("unknown root rule " + root_rule);

    // lower the rules reachable from the root
    std::map<int, Dfa> dfas;
    std::vector<int> todo{index[root_rule]};
    while (!todo.empty()) {
        int r = todo.back(); todo.pop_back();
        if (dfas.count(r)) continue;
        const Node& body = rules.at(order[(size_t)r]);
        // Rule bodies recur across grammars (the same tool schema in many requests): the minimal automaton of a body is
        // kept process-wide under its structure, references written as their rank among the body's references by
        // declaration index (which is all the canonical numbering depends on).
        std::vector<int> ref_decl;                                  // declaration indices referenced, ascending
        bool refs_ok = true;
        collect_refs(body, index, ref_decl, refs_ok);
        std::sort(ref_decl.begin(), ref_decl.end());
        ref_decl.erase(std::unique(ref_decl.begin(), ref_decl.end()), ref_decl.end());
        std::string key;
        if (refs_ok) body_key(body, index, ref_decl, key);
        Dfa d;
        bool from_memo = false;
        if (refs_ok) {
            std::lock_guard<std::mutex> lk(g_body_memo_mu);
            auto it = g_body_memo.find(key);
            if (it != g_body_memo.end()) { d = *it->second; from_memo = true; }
        }
        if (from_memo) {
            for (auto& es : d.rt) for (auto& e : es) e.first = ref_decl[(size_t)e.first];   // rank -> declaration index here
        } else {
            Dfa raw;
            if (body.k == NK::Tag) raw = tagdispatch_automaton(body, index);
            else {
                Nfa nfa;
                int s = nfa.add(), e = nfa.add();
                build_nfa(body, nfa, s, e, index);
                raw = subset_construction(nfa, s, e);
            }
            d = minimise_canonical(raw, order[(size_t)r]);
            if (refs_ok) {
                auto keep = std::make_shared<Dfa>(d);
                for (auto& es : keep->rt)
                    for (auto& e : es) e.first = (int)(std::lower_bound(ref_decl.begin(), ref_decl.end(), e.first) - ref_decl.begin());
                std::lock_guard<std::mutex> lk(g_body_memo_mu);
                if (g_body_memo.size() > 200000) g_body_memo.clear();   // a bound on memory, not a policy
                g_body_memo.emplace(std::move(key), std::move(keep));
            }
        }
        for (auto& es : d.rt) for (auto& e : es) todo.push_back(e.first);
        dfas.emplace(r, std::move(d));
    }
    Grammar g;
    std::map<int, int> remap;                                    // declaration index -> index in g.rules
    for (auto& kv : dfas) { remap[kv.first] = (int)remap.size(); }
    for (auto& kv : dfas) {
        const Dfa& d = kv.second;
        RuleFsm f;
        f.name = order[(size_t)kv.first];
        f.decl_index = kv.first;
        int n = d.n();
        f.is_final.assign(d.fin.begin(), d.fin.end());
        f.bedges.resize((size_t)n);
        f.redges.resize((size_t)n);
        // maximal runs of consecutive bytes of one class: the same for every state of the automaton
        std::vector<std::array<int, 3>> class_runs;                 // {lo, hi, class}
        for (int b = 0; b < 256;) {
            int e = b;
            while (e + 1 < 256 && d.cls[(size_t)(e + 1)] == d.cls[(size_t)b]) ++e;
            class_runs.push_back({b, e, (int)d.cls[(size_t)b]});
            b = e + 1;
        }
        for (int q = 0; q < n; ++q) {
            int lo = -1, hi = -1, tgt = -1;                          // run of bytes with one target being grown
            for (const auto& cr : class_runs) {
                const int t = d.at(q, cr[2]);
                if (t == tgt && lo >= 0 && cr[0] == hi + 1) { hi = cr[1]; continue; }
                if (lo >= 0 && tgt >= 0) f.bedges[(size_t)q].push_back({(uint8_t)lo, (uint8_t)hi, tgt});
                lo = cr[0]; hi = cr[1]; tgt = t;
            }
            if (lo >= 0 && tgt >= 0) f.bedges[(size_t)q].push_back({(uint8_t)lo, (uint8_t)hi, tgt});
            for (auto& r : d.rt[(size_t)q]) f.redges[(size_t)q].push_back({remap.at(r.first), r.second});
        }
        g.rules.push_back(std::move(f));
    }
    g.root = remap.at(index[root_rule]);
    int R = (int)g.rules.size();
    // nullable rules (least fixed point) and productivity (every reachable rule must derive a string)
    auto fixed_point = [&](bool want_nullable) {
        std::vector<uint8_t> ok((size_t)R, 0);
        for (bool changed = true; changed;) {
            changed = false;
            for (int r = 0; r < R; ++r) {
                if (ok[(size_t)r]) continue;
                const RuleFsm& f = g.rules[(size_t)r];
                std::vector<uint8_t> seen((size_t)f.n_states(), 0);
                std::vector<int> stack{0};
                seen[0] = 1;
                bool hit = false;
                while (!stack.empty() && !hit) {
                    int q = stack.back(); stack.pop_back();
                    if (f.is_final[(size_t)q]) { hit = true; break; }
                    auto visit = [&](int t) { if (!seen[(size_t)t]) { seen[(size_t)t] = 1; stack.push_back(t); } };
                    if (!want_nullable) for (auto& e : f.bedges[(size_t)q]) visit(e.tgt);
                    for (auto& e : f.redges[(size_t)q]) if (ok[(size_t)e.rule]) visit(e.tgt);
                }
                if (hit) { ok[(size_t)r] = 1; changed = true; }
            }
        }
        return ok;
    };
    std::vector<uint8_t> nullable = fixed_point(true), productive = fixed_point(false);
    for (int r = 0; r < R; ++r) {
        g.rules[(size_t)r].nullable = nullable[(size_t)r];
        if (!productive[(size_t)r]) throw GrammarError("rule " + g.rules[(size_t)r].name + " derives no string (grammar is not reduced)");
    }
    // shortest sentence of every rule: relax until stable (byte edge = 1, rule edge = the rule's own minimum)
    {
        const int32_t INF = 1 << 28;
        std::vector<int32_t> ml((size_t)R, INF);
        for (bool changed = true; changed;) {
            changed = false;
            for (int r = 0; r < R; ++r) {
                const RuleFsm& f = g.rules[(size_t)r];
                std::vector<int32_t> dist((size_t)f.n_states(), INF);
                dist[0] = 0;
                for (bool moved = true; moved;) {                   // Bellman-Ford over the (small) automaton
                    moved = false;
                    for (int q = 0; q < f.n_states(); ++q) {
                        if (dist[(size_t)q] >= INF) continue;
                        for (auto& e : f.bedges[(size_t)q]) if (dist[(size_t)q] + 1 < dist[(size_t)e.tgt]) { dist[(size_t)e.tgt] = dist[(size_t)q] + 1; moved = true; }
                        for (auto& e : f.redges[(size_t)q]) {
                            int32_t c = ml[(size_t)e.rule];
                            if (c < INF && dist[(size_t)q] + c < dist[(size_t)e.tgt]) { dist[(size_t)e.tgt] = dist[(size_t)q] + c; moved = true; }
                        }
                    }
                }
                int32_t best = INF;
                for (int q = 0; q < f.n_states(); ++q) if (f.is_final[(size_t)q]) best = std::min(best, dist[(size_t)q]);
                if (best < ml[(size_t)r]) { ml[(size_t)r] = best; changed = true; }
            }
        }
        for (int r = 0; r < R; ++r) g.rules[(size_t)r].min_len = ml[(size_t)r];
    }
    g.state_base.resize((size_t)R);
    g.n_states = 0;
    for (int r = 0; r < R; ++r) { g.state_base[(size_t)r] = g.n_states; g.n_states += g.rules[(size_t)r].n_states(); }
    g.sid_to_pos.assign((size_t)g.n_states, -1);
    for (int r = 0; r < R; ++r)
        for (int q = 0; q < g.rules[(size_t)r].n_states(); ++q)
            if (!g.rules[(size_t)r].bedges[(size_t)q].empty()) {
                g.sid_to_pos[(size_t)g.sid(r, q)] = (int)g.positions.size();
                g.positions.push_back({r, q, g.sid(r, q)});
            }
    hash_rules(g);
    return g;
}

std::vector<std::vector<int32_t>> bounded_classes(const Grammar& g, int32_t budget, const std::vector<uint64_t>& ref_identity) {
    std::vector<std::vector<int32_t>> rep(g.rules.size());
    for (size_t r = 0; r < g.rules.size(); ++r) rep[r] = bounded_classes_rule(g, (int32_t)r, budget, ref_identity);
    return rep;
}

std::vector<int32_t> bounded_classes_rule(const Grammar& g, int32_t rule, int32_t budget, const std::vector<uint64_t>& ref_identity,
                                          NearClasses* near) {
    std::vector<int32_t> rep_r;
    {
        const size_t r = (size_t)rule;
        const RuleFsm& f = g.rules[r];
        const int n = f.n_states();
        // level[d][x] = class of x with d bytes left; level 0 tells nothing apart.  Signatures of one level lie back to
        // back in one buffer; states are grouped through a hash table whose hits are confirmed by comparing the
        // signatures themselves, and classes are numbered in the order of their first state.
        std::vector<std::vector<int32_t>> level(1, std::vector<int32_t>((size_t)n, 0));
        bool any_nullable_edge = false;
        for (int x = 0; x < n && !any_nullable_edge; ++x)
            for (auto& e : f.redges[(size_t)x]) if (g.rules[(size_t)e.rule].nullable) { any_nullable_edge = true; break; }
        std::vector<int64_t> base, full;
        std::vector<size_t> base_off((size_t)n + 1), full_off((size_t)n + 1);
        std::vector<std::pair<int64_t, int64_t>> refs;
        std::vector<int32_t> slot_state;                            // open addressing: slot -> first state of the class, or -1
        auto group = [&](const std::vector<int64_t>& buf, const std::vector<size_t>& off, std::vector<int32_t>& out) -> size_t {
            size_t cap = 16;
            while (cap < (size_t)n * 2) cap <<= 1;
            slot_state.assign(cap, -1);
            size_t n_classes = 0;
            for (int x = 0; x < n; ++x) {
                const int64_t* sx = buf.data() + off[(size_t)x];
                const size_t lx = off[(size_t)x + 1] - off[(size_t)x];
                uint64_t h = 0x9E3779B97F4A7C15ull ^ lx;
                for (size_t k = 0; k < lx; ++k) { h ^= (uint64_t)sx[k]; h *= 0xFF51AFD7ED558CCDull; h ^= h >> 32; }
                for (size_t at = (size_t)h & (cap - 1);; at = (at + 1) & (cap - 1)) {
                    const int32_t y = slot_state[at];
                    if (y < 0) { slot_state[at] = x; out[(size_t)x] = (int32_t)n_classes++; break; }
                    const size_t ly = off[(size_t)y + 1] - off[(size_t)y];
                    if (ly == lx && std::equal(sx, sx + lx, buf.data() + off[(size_t)y])) { out[(size_t)x] = out[(size_t)y]; break; }
                }
            }
            return n_classes;
        };
        // Levels only refine.  Level d is a function of level d - 1 and of the levels d - m for the shortest sentences m
        // of the referenced rules, so once the partition has not changed over max m (at least one) levels in a row it
        // never changes again.
        int32_t settle = 1;
        for (int x = 0; x < n; ++x)
            for (auto& e : f.redges[(size_t)x]) {
                const RuleFsm& c = g.rules[(size_t)e.rule];
                if (!c.nullable && c.min_len <= budget) settle = std::max(settle, c.min_len);
            }
        size_t last_count = 1;
        int32_t unchanged = 0;
        for (int32_t d = 1; d <= budget; ++d) {
            if (unchanged >= settle) { level.push_back(level.back()); continue; }
            const std::vector<int32_t>& prev = level.back();
            // part of the signature that does not depend on the level being computed
            base.clear();
            for (int x = 0; x < n; ++x) {
                base_off[(size_t)x] = base.size();
                base.push_back(prev[(size_t)x]);
                base.push_back(f.is_final[(size_t)x]);
                // maximal runs of consecutive bytes that lead to the same class (edges are sorted and disjoint)
                {
                    int run_lo = -1, run_hi = -1; int32_t run_cls = -1;
                    for (auto& e : f.bedges[(size_t)x]) {
                        const int32_t c = prev[(size_t)e.tgt];
                        if (run_lo >= 0 && (int)e.lo == run_hi + 1 && c == run_cls) { run_hi = e.hi; continue; }
                        if (run_lo >= 0) { base.push_back(run_lo); base.push_back(run_hi); base.push_back(run_cls); }
                        run_lo = e.lo; run_hi = e.hi; run_cls = c;
                    }
                    if (run_lo >= 0) { base.push_back(run_lo); base.push_back(run_hi); base.push_back(run_cls); }
                }
                base.push_back(-7);
                refs.clear();
                for (auto& e : f.redges[(size_t)x]) {
                    const RuleFsm& c = g.rules[(size_t)e.rule];
                    if (c.nullable) continue;
                    int32_t left = d - c.min_len;
                    refs.emplace_back((int64_t)ref_identity[(size_t)e.rule], left >= 0 ? level[(size_t)left][(size_t)e.tgt] : -1);
                }
                if (refs.size() > 1) std::sort(refs.begin(), refs.end());
                for (auto& p : refs) { base.push_back(p.first); base.push_back(p.second); }
            }
            base_off[(size_t)n] = base.size();
            std::vector<int32_t> cur((size_t)n, 0);
            size_t count = 0;
            if (!any_nullable_edge) {
                count = group(base, base_off, cur);
            } else {
                // coarsest partition stable under "a nullable rule edge leads to the same class of this level"; it refines
                // the previous level, so the iteration may start there
                cur = prev;
                std::vector<int32_t> nxt((size_t)n);
                for (size_t n_classes = 0;;) {
                    full.clear();
                    for (int x = 0; x < n; ++x) {
                        full_off[(size_t)x] = full.size();
                        full.insert(full.end(), base.begin() + (long)base_off[(size_t)x], base.begin() + (long)base_off[(size_t)x + 1]);
                        full.push_back(-9);
                        refs.clear();
                        for (auto& e : f.redges[(size_t)x])
                            if (g.rules[(size_t)e.rule].nullable) refs.emplace_back((int64_t)ref_identity[(size_t)e.rule], cur[(size_t)e.tgt]);
                        if (refs.size() > 1) std::sort(refs.begin(), refs.end());
                        for (auto& p : refs) { full.push_back(p.first); full.push_back(p.second); }
                    }
                    full_off[(size_t)n] = full.size();
                    const size_t got = group(full, full_off, nxt);
                    cur.swap(nxt);
                    count = got;
                    if (got == n_classes) break;
                    n_classes = got;
                }
            }
            unchanged = count == last_count ? unchanged + 1 : 0;
            last_count = count;
            level.push_back(cur);
        }
        const std::vector<int32_t>& fin = level.back();
        std::vector<int32_t> best((size_t)n, -1);                // class (numbered below n) -> member with the smallest canonical id
        for (int x = 0; x < n; ++x) {
            int32_t& b = best[(size_t)fin[(size_t)x]];
            if (b < 0 || f.canon_id[(size_t)x] < f.canon_id[(size_t)b]) b = x;
        }
        rep_r.resize((size_t)n);
        for (int x = 0; x < n; ++x) rep_r[(size_t)x] = best[(size_t)fin[(size_t)x]];
        if (near) {
            // classes in the order of falling size (the class a long repetition collapses into comes first); each looks
            // for the deepest level at which it still coincides with a class that is built in full
            near->base.assign((size_t)n, -1);
            near->depth.assign((size_t)n, 0);
            std::vector<int32_t> weight((size_t)n, 0);                                    // by class number (< n)
            for (int x = 0; x < n; ++x) ++weight[(size_t)fin[(size_t)x]];
            std::vector<std::array<int32_t, 3>> keyed;                                   // {-size, canonical id, state}
            for (int c = 0; c < n; ++c) if (best[(size_t)c] >= 0) keyed.push_back({-weight[(size_t)c], f.canon_id[(size_t)best[(size_t)c]], best[(size_t)c]});
            std::sort(keyed.begin(), keyed.end());
            std::vector<int32_t> reps;
            for (auto& k : keyed) reps.push_back(k[2]);
            const int32_t top = std::min<int32_t>(budget - 1, kMaxNearDepth);
            // per level: class -> a class built in full (-1: none yet)
            std::vector<std::vector<int32_t>> full((size_t)std::max(top + 1, 1));
            for (int32_t e = kMinNearDepth; e <= top; ++e) full[(size_t)e].assign((size_t)n, -1);
            for (int32_t x : reps) {
                if (f.bedges[(size_t)x].empty()) continue;                               // no plane
                int32_t d = top;
                for (; d >= kMinNearDepth; --d) {
                    const int32_t y = full[(size_t)d][(size_t)level[(size_t)d][(size_t)x]];
                    if (y >= 0) { near->base[(size_t)x] = y; near->depth[(size_t)x] = d; break; }
                }
                if (d < kMinNearDepth)
                    for (int32_t e = kMinNearDepth; e <= top; ++e) {
                        int32_t& y = full[(size_t)e][(size_t)level[(size_t)e][(size_t)x]];
                        if (y < 0) y = x;
                    }
            }
        }
    }
    return rep_r;
}

FollowInfo follow_signatures(const Grammar& g, int32_t budget, const std::vector<std::vector<int32_t>>* rep,
                             const std::vector<uint64_t>* ref_identity, const FollowInterner* intern, const FollowMemo* memo_of) {
    const int R = (int)g.rules.size();
    // A node of the unfolding is described by a list of words (constants, byte ranges, the values of its children).
    // Without an interner its value is the hash of the list; with one it is the interner's number for exactly this
    // list, so that equal values mean equal structures as long as the children's values do.
    auto value_of = [&](std::vector<uint64_t>& desc) -> uint64_t {
        if (intern) return (*intern)(desc);
        uint64_t h = desc.empty() ? 0 : desc[0];
        for (size_t k = 1; k < desc.size(); ++k) h = hash_combine(h, desc[k]);
        return h;
    };
    auto rule_identity = [&](int rule) -> uint64_t { return ref_identity ? (*ref_identity)[(size_t)rule] : g.rules[(size_t)rule].hash; };
    const int32_t INF = 1 << 28;
    // shortest completion of every state, in bytes
    std::vector<std::vector<int32_t>> min_suf((size_t)R);
    for (int r = 0; r < R; ++r) {
        const RuleFsm& f = g.rules[(size_t)r];
        std::vector<int32_t>& d = min_suf[(size_t)r];
        d.assign((size_t)f.n_states(), INF);
        // shortest paths to a final state over the reversed edges (a byte costs 1, a rule its shortest sentence)
        const int n = f.n_states();
        std::vector<std::vector<std::pair<int32_t, int32_t>>> back((size_t)n);      // target -> (source, cost)
        for (int q = 0; q < n; ++q) {
            for (auto& e : f.bedges[(size_t)q]) back[(size_t)e.tgt].emplace_back(q, 1);
            for (auto& e : f.redges[(size_t)q]) back[(size_t)e.tgt].emplace_back(q, g.rules[(size_t)e.rule].min_len);
        }
        std::priority_queue<std::pair<int32_t, int32_t>, std::vector<std::pair<int32_t, int32_t>>, std::greater<>> heap;
        for (int q = 0; q < n; ++q) if (f.is_final[(size_t)q]) { d[(size_t)q] = 0; heap.emplace(0, q); }
        while (!heap.empty()) {
            const auto [dist, q] = heap.top();
            heap.pop();
            if (dist > d[(size_t)q]) continue;
            for (auto& [src, cost] : back[(size_t)q])
                if (dist + cost < d[(size_t)src]) { d[(size_t)src] = dist + cost; heap.emplace(dist + cost, src); }
        }
    }
    // unfold(d, rule, state): structural hash of the state's behaviour on at most d bytes (0 for d = 0).  Computed on
    // demand: only the states in which referencing rules continue, and what is within d bytes of them, are ever asked
    // for.  States on a cycle of nullable rule edges get a fresh salt.
    std::vector<uint8_t> cyclic((size_t)g.n_states, 1);
    for (int r = 0; r < R; ++r) {
        const RuleFsm& f = g.rules[(size_t)r];
        const int n = f.n_states();
        std::vector<int> indeg((size_t)n, 0), order;
        std::vector<std::vector<int>> preds((size_t)n);
        for (int x = 0; x < n; ++x)
            for (auto& e : f.redges[(size_t)x]) if (g.rules[(size_t)e.rule].nullable) { ++indeg[(size_t)x]; preds[(size_t)e.tgt].push_back(x); }
        for (int x = 0; x < n; ++x) if (indeg[(size_t)x] == 0) order.push_back(x);
        for (size_t k = 0; k < order.size(); ++k) for (int p : preds[(size_t)order[k]]) if (--indeg[(size_t)p] == 0) order.push_back(p);
        for (int x : order) cyclic[(size_t)g.sid(r, x)] = 0;
    }
    std::vector<std::vector<uint64_t>> unfold_memo((size_t)budget + 1);
    std::vector<std::vector<uint8_t>> unfold_have((size_t)budget + 1);
    std::function<uint64_t(int32_t, int, int)> unfold = [&](int32_t d, int r, int x) -> uint64_t {
        if (d <= 0) return 0;
        if (unfold_memo[(size_t)d].empty()) { unfold_memo[(size_t)d].assign((size_t)g.n_states, 0); unfold_have[(size_t)d].assign((size_t)g.n_states, 0); }
        const size_t sid = (size_t)g.sid(r, x);
        if (unfold_have[(size_t)d][sid]) return unfold_memo[(size_t)d][sid];
        const RuleFsm& f = g.rules[(size_t)r];
        // the unfolding of a state depends on its rule and the rules that one references, not on the grammar around it:
        // an identical rule met before (in this grammar or an earlier one of the pool) has it ready
        uint64_t* kept = memo_of ? (*memo_of)(r, x, d) : nullptr;
        if (kept && *kept) {
            unfold_memo[(size_t)d][sid] = *kept;
            unfold_have[(size_t)d][sid] = 1;
            return *kept;
        }
        uint64_t h;
        std::vector<uint64_t> desc;
        if (cyclic[sid]) {
            desc = {0xC1C1ull, g_unshareable_salt.fetch_add(1)};
            h = value_of(desc);
        } else {
            desc = {0x51ull, (uint64_t)f.is_final[(size_t)x]};
            {   // maximal runs of consecutive bytes with the same unfolding (edges are sorted and disjoint)
                int run_lo = -1, run_hi = -1; uint64_t run_h = 0;
                for (auto& e : f.bedges[(size_t)x]) {
                    const uint64_t u = unfold(d - 1, r, e.tgt);
                    if (run_lo >= 0 && (int)e.lo == run_hi + 1 && u == run_h) { run_hi = e.hi; continue; }
                    if (run_lo >= 0) { desc.push_back((uint64_t)run_lo); desc.push_back((uint64_t)run_hi); desc.push_back(run_h); }
                    run_lo = e.lo; run_hi = e.hi; run_h = u;
                }
                if (run_lo >= 0) { desc.push_back((uint64_t)run_lo); desc.push_back((uint64_t)run_hi); desc.push_back(run_h); }
            }
            if (!f.redges[(size_t)x].empty()) {
                std::vector<std::pair<uint64_t, uint64_t>> refs;
                for (auto& e : f.redges[(size_t)x]) {
                    const RuleFsm& c = g.rules[(size_t)e.rule];
                    int32_t left = c.nullable ? d : d - c.min_len;
                    refs.emplace_back(rule_identity(e.rule), left >= 0 ? unfold(left, r, e.tgt) : 0x7777ull);
                }
                std::sort(refs.begin(), refs.end());
                for (auto& p : refs) { desc.push_back(0xEFull << 56); desc.push_back(p.first); desc.push_back(p.second); }
            }
            h = value_of(desc);
        }
        unfold_memo[(size_t)d][sid] = h;
        unfold_have[(size_t)d][sid] = 1;
        if (kept) *kept = h;
        return h;
    };
    // reference sites of every rule
    struct Site { int q, x; };
    std::vector<std::vector<Site>> sites((size_t)R);
    for (int q = 0; q < R; ++q)
        for (int s = 0; s < g.rules[(size_t)q].n_states(); ++s)
            for (auto& e : g.rules[(size_t)q].redges[(size_t)s]) sites[(size_t)e.rule].push_back({q, rep ? (*rep)[(size_t)q][(size_t)e.tgt] : e.tgt});
    for (auto& v : sites) {                                         // one site per state (class) a referencing rule continues in
        std::sort(v.begin(), v.end(), [](const Site& a, const Site& b) { return a.q != b.q ? a.q < b.q : a.x < b.x; });
        v.erase(std::unique(v.begin(), v.end(), [](const Site& a, const Site& b) { return a.q == b.q && a.x == b.x; }), v.end());
    }
    std::vector<uint64_t> memo((size_t)R * ((size_t)budget + 1), 0);
    std::vector<uint8_t> memo_state((size_t)R * ((size_t)budget + 1), 0);      // 0 unknown, 1 being computed, 2 known
    std::function<uint64_t(int, int)> sig = [&](int rule, int d) -> uint64_t {
        const size_t key = (size_t)rule * ((size_t)budget + 1) + (size_t)d;
        if (memo_state[key] == 2) return memo[key];
        if (memo_state[key] == 1) {                                         // cycle through rule ends
            std::vector<uint64_t> salt{0xCCCCull, g_unshareable_salt.fetch_add(1)};
            return value_of(salt);
        }
        memo_state[key] = 1;
        std::vector<uint64_t> parts;
        if (rule == g.root) parts.push_back(0xE0Full);                      // the input may end here
        for (const Site& st : sites[(size_t)rule]) {
            uint64_t h = unfold(d, st.q, st.x);
            int32_t left = d - min_suf[(size_t)st.q][(size_t)st.x];
            if (left > 0 || (left == 0 && d > 0 && min_suf[(size_t)st.q][(size_t)st.x] == 0)) {
                std::vector<uint64_t> pair{0x5173ull, h, sig(st.q, left)};
                h = value_of(pair);
            }
            parts.push_back(h);
        }
        std::sort(parts.begin(), parts.end());
        parts.erase(std::unique(parts.begin(), parts.end()), parts.end());
        std::vector<uint64_t> desc{0xF011ull};
        desc.insert(desc.end(), parts.begin(), parts.end());
        uint64_t h = value_of(desc);
        memo_state[key] = 2;
        memo[key] = h;
        return h;
    };
    FollowInfo out;
    out.sig.assign((size_t)R, std::vector<uint64_t>((size_t)budget + 1, 0));
    for (int r = 0; r < R; ++r)
        for (int32_t d = 0; d <= budget; ++d) out.sig[(size_t)r][(size_t)d] = sig(r, d);
    out.min_suf = std::move(min_suf);
    return out;
}

std::string describe_grammar(const Grammar& g) {
    std::ostringstream o;
    o << "{\"root\":\"" << g.rules[(size_t)g.root].name << "\",\"rules\":[";
    for (size_t r = 0; r < g.rules.size(); ++r) {
        const RuleFsm& f = g.rules[r];
        if (r) o << ",";
        o << "{\"name\":\"" << f.name << "\",\"decl_index\":" << f.decl_index << ",\"nullable\":" << (f.nullable ? "true" : "false")
          << ",\"shareable\":" << (f.shareable ? "true" : "false") << ",\"hash\":\"" << std::hex << f.hash << std::dec << "\",\"states\":[";
        for (int q = 0; q < f.n_states(); ++q) {
            if (q) o << ",";
            o << "{\"final\":" << (f.is_final[(size_t)q] ? "true" : "false") << ",\"canon\":" << f.canon_id[(size_t)q] << ",\"bytes\":[";
            for (size_t k = 0; k < f.bedges[(size_t)q].size(); ++k) {
                auto& e = f.bedges[(size_t)q][k];
                if (k) o << ",";
                o << "[" << (int)e.lo << "," << (int)e.hi << "," << e.tgt << "]";
            }
            o << "],\"refs\":[";
            for (size_t k = 0; k < f.redges[(size_t)q].size(); ++k) {
                auto& e = f.redges[(size_t)q][k];
                if (k) o << ",";
                o << "[\"" << g.rules[(size_t)e.rule].name << "\"," << e.tgt << "]";
            }
            o << "]}";
        }
        o << "]}";
    }
    o << "],\"positions\":[";
    for (size_t p = 0; p < g.positions.size(); ++p) {
        if (p) o << ",";
        o << "[\"" << g.rules[(size_t)g.positions[p].rule].name << "\"," << g.positions[p].state << "]";
    }
    o << "]}";
    return o.str();
}

}  // namespace xg2
