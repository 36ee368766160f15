// Test helper (CPU only): steps the recogniser core that the kernels run per lane, compiled for the host,
// against the host Earley parser of the library, for every plane context of a grammar and a list of tokens.
// Built by tests/test_host_logic.py with g++; it is not part of the library.
#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

#include "../../paper_2601_04426_amd/csrc/earley_core.hpp"
#include "../../paper_2601_04426_amd/csrc/grammar.hpp"
#include "../../paper_2601_04426_amd/csrc/tables.hpp"

#ifndef HC_K
#define HC_K 6      // capacities of the LDS path of the build kernel (its long lists; the short ones fall back to these at half width)
#define HC_WM 10
#endif
using namespace xg2;
using namespace xg2::core;

namespace {

template <int K_, int WM_, int MAXLEN_>
struct HostStore {
    static constexpr int K = K_, WM = WM_, MAXLEN = MAXLEN_;
    std::vector<uint32_t> a, b, w, ws;
    uint32_t* cur; uint32_t* nxt;
    HostStore() : a(K_), b(K_), w(2 * WM_), ws(MAXLEN_ + 1) { cur = a.data(); nxt = b.data(); }
    uint32_t get_cur(int k) const { return cur[k]; }
    void set_cur(int k, uint32_t v) { cur[k] = v; }
    uint32_t get_nxt(int k) const { return nxt[k]; }
    void set_nxt(int k, uint32_t v) { nxt[k] = v; }
    uint32_t wait_rule(int k) const { return w[2 * (size_t)k]; }
    uint32_t wait_tgt(int k) const { return w[2 * (size_t)k + 1]; }
    void set_wait(int k, uint32_t r, uint32_t t) { w[2 * (size_t)k] = r; w[2 * (size_t)k + 1] = t; }
    void swap() { std::swap(cur, nxt); }
    bool charge(int) { return true; }
    void reset() {}
    void set_wstart(int j, uint32_t v) { ws.at((size_t)j) = v; }
    uint32_t get_wstart(int j) const { return ws.at((size_t)j); }
};

struct Ctx {
    std::vector<uint32_t> items, wait, wait_off;
    uint32_t H = 0;
};

Ctx ctx_of(const EarleyChart& chart, bool renumber) {
    Ctx c;
    if (renumber) {
        ScanContext sc;
        if (!chart.context(sc)) throw std::runtime_error("context too deep");
        c.items = sc.items; c.wait = sc.wait; c.wait_off = sc.wait_off; c.H = sc.H;
        return c;
    }
    // the way the build plans a plane: every set of the chart, in order
    const auto& sets = chart.sets();
    auto loc = [](int32_t o) { return o < 0 ? kRootOrigin : (uint32_t)o; };
    for (const ChartItem& it : sets.back().scan) c.items.push_back(pack_item(chart.tables()->ref(it.sid), loc(it.origin)));
    for (const ChartSet& cs : sets) {
        c.wait_off.push_back((uint32_t)(c.wait.size() / 2));
        for (const ChartItem& it : cs.wait) chart.push_triples(it, loc(it.origin), c.wait);
    }
    c.wait_off.push_back((uint32_t)(c.wait.size() / 2));
    c.H = (uint32_t)sets.size();
    return c;
}

// what the host parser says about token t from the chart's current state: bit 0 alive, bit 1 early
int host_result(EarleyChart chart, const uint8_t* t, size_t n) {
    int res = 0;
    for (size_t i = 0; i < n; ++i) {
        if (!chart.advance(t + i, 1)) return res;
        if (chart.last().root_done && i + 1 < n) res |= RES_EARLY;
    }
    return res | RES_ALIVE;
}

template <class S>
int core_result(const FlatTables& ft, const DevTables& T, const Ctx& c, const uint8_t* t, size_t n) {
    DevCtx C;
    C.items = c.items.data(); C.n_items = (uint32_t)c.items.size();
    C.wait = reinterpret_cast<const uint2*>(c.wait.data()); C.wait_off = c.wait_off.data(); C.H = c.H;
    S st;
    MemBytes tok{t};
    return scan_token<S, false, MemBytes>(T, ft.byte_class_words.data(), C, tok, (int)n, st);
}

}  // namespace

// Returns the number of (context, token) pairs checked, or -(1 + index of the first mismatch) with a
// description in msg.  Contexts: every position alone; every position inside every state that references
// its rule; and the states along `sentence` (renumbered contexts, as fill builds them).
extern "C" long long xg2hc_check(const char* ebnf, size_t len, const char* root, const uint8_t* bytes, const uint64_t* offs, int n_tok,
                                 const uint8_t* sentence, size_t sentence_len, int max_contexts, char* msg, size_t msg_cap,
                                 long long* n_small_overflow) {
    try {
        Grammar g = lower_grammar(std::string(ebnf, len), root);
        FlatTables ft = flatten(g);
        DevTables T{};
        T.state = reinterpret_cast<const uint4*>(ft.dev_state.data());
        T.exp_list = ft.exp_list.data();
        T.trans = ft.trans.data();
        T.byte_class_words = ft.byte_class_words.data();
        T.n_classes = ft.n_classes;
        T.sink = ft.sink;
        long long checked = 0, small_over = 0, n_walked = 0;
        int n_ctx = 0;
        auto run = [&](const EarleyChart& chart, bool renumber, const std::string& what) -> bool {
            Ctx c = ctx_of(chart, renumber);
            for (int k = 0; k < n_tok; ++k) {
                const uint8_t* t = bytes + offs[k];
                size_t n = (size_t)(offs[k + 1] - offs[k]);
                if (n == 0) continue;
                int want = host_result(chart, t, n);
                int got = n <= 16 ? core_result<HostStore<HC_K, HC_WM, 16>>(ft, T, c, t, n) : RES_OVERFLOW;
                if (got & RES_OVERFLOW) { ++small_over; got = core_result<HostStore<256, 1024, 1024>>(ft, T, c, t, n); }
                ++checked;
                if (got != want) {
                    snprintf(msg, msg_cap, "%s token %d: host parser %d, recogniser core %d", what.c_str(), k, want, got);
                    return false;
                }
                // the branch-free automaton walk of the build's first phase, where the start set is one plain automaton state
                if (c.items.size() == 1 && (c.items[0] & (F_BYTE | F_REF)) == F_BYTE && n <= 16) {
                    uint4 tv = make_uint4(0, 0, 0, 0);
                    std::memcpy(&tv, t, n);
                    const bool root = (c.items[0] >> REF_BITS) == ROOT_ORIGIN;
                    const uint8_t* cls = reinterpret_cast<const uint8_t*>(ft.byte_class_words.data());
                    const WalkResult r = root ? walk_tokens<true>(T.trans, T.n_classes, T.sink, cls, c.items[0] & REF_MASK, tv, (int)n)
                                              : walk_tokens<false>(T.trans, T.n_classes, T.sink, cls, c.items[0] & REF_MASK, tv, (int)n);
                    const bool defer = (r.seen & (root ? F_REF : (F_REF | F_FINAL))) != 0;
                    if (!defer) {
                        const bool alive = r.state != T.sink;
                        const bool dead_early = root && !alive && (r.seen_before_last & F_FINAL);
                        const int walked = alive ? RES_ALIVE : dead_early ? RES_EARLY : 0;
                        const int expect = (want & RES_ALIVE) ? RES_ALIVE : (want & RES_EARLY);
                        ++n_walked;
                        if (walked != expect) {
                            snprintf(msg, msg_cap, "%s token %d: host parser %d, automaton walk %d", what.c_str(), k, want, walked);
                            return false;
                        }
                    }
                }
            }
            return true;
        };
        EarleyChart chart(&ft);
        for (const Position& ps : g.positions) {
            if (n_ctx++ >= max_contexts) break;
            chart.start((uint32_t)ps.sid);
            if (!run(chart, false, "position " + std::to_string(ps.sid))) return -checked - 1;
            for (size_t w = 0; w < ft.state_info.size(); ++w) {
                const StateInfo& wi = ft.state_info[w];
                bool refs = false;
                for (uint32_t e = 0; e < (wi.counts >> 16); ++e) refs |= ft.ref_edges[wi.ref_off + e].rule == (uint32_t)ps.rule;
                if (!refs) continue;
                if (n_ctx++ >= max_contexts) break;
                chart.start_pair((uint32_t)ps.sid, (uint32_t)w);
                if (!run(chart, false, "position " + std::to_string(ps.sid) + " inside state " + std::to_string(w))) return -checked - 1;
            }
        }
        chart.start(ft.root_start);
        for (size_t i = 0; i <= sentence_len; ++i) {
            if (!run(chart, true, "after " + std::to_string(i) + " sentence bytes")) return -checked - 1;
            if (i < sentence_len && !chart.advance(sentence + i, 1)) { snprintf(msg, msg_cap, "sentence rejected at byte %zu", i); return -checked - 1; }
        }
        if (n_small_overflow) *n_small_overflow = small_over;
        if (n_walked == 0 && checked > 1000) { snprintf(msg, msg_cap, "no context exercised the automaton walk"); return -1; }
        return checked;
    } catch (const std::exception& e) {
        snprintf(msg, msg_cap, "exception: %s", e.what());
        return -1;
    }
}

// States the library treats as equivalent on short tokens: for every state x that the bounded-class analysis gives a
// base b and a depth d (no string of at most d bytes tells x from b), the host parser must give every token of at
// most d bytes the same result from x as from b, alone and inside every state that references the rule.  Returns the
// number of (state, context, token) comparisons, or -(1 + that number) at the first difference; *n_near = states
// that have a base.  Rules are given distinct identities, as for a grammar compiled without a pool.
extern "C" long long xg2hc_check_near(const char* ebnf, size_t len, const char* root, const uint8_t* bytes, const uint64_t* offs, int n_tok,
                                      char* msg, size_t msg_cap, long long* n_near, long long* max_depth) {
    try {
        Grammar g = lower_grammar(std::string(ebnf, len), root);
        FlatTables ft = flatten(g);
        int32_t budget = 1;
        for (int k = 0; k < n_tok; ++k) budget = std::max<int32_t>(budget, (int32_t)(offs[k + 1] - offs[k]));
        std::vector<uint64_t> ids(g.rules.size());
        for (size_t r = 0; r < ids.size(); ++r) ids[r] = r + 1;
        long long checked = 0, near_states = 0, deepest = 0;
        EarleyChart cx(&ft), cb(&ft);
        for (size_t r = 0; r < g.rules.size(); ++r) {
            NearClasses nc;
            std::vector<int32_t> rep = bounded_classes_rule(g, (int32_t)r, budget, ids, &nc);
            std::vector<int64_t> waiters{-1};
            for (size_t w = 0; w < ft.state_info.size(); ++w) {
                const StateInfo& wi = ft.state_info[w];
                for (uint32_t e = 0; e < (wi.counts >> 16); ++e)
                    if (ft.ref_edges[wi.ref_off + e].rule == (uint32_t)r) { waiters.push_back((int64_t)w); break; }
            }
            for (int x = 0; x < g.rules[r].n_states(); ++x) {
                const int32_t b = nc.base[(size_t)x], d = nc.depth[(size_t)x];
                if (b < 0) continue;
                ++near_states;
                deepest = std::max<long long>(deepest, d);
                if (nc.base[(size_t)b] >= 0) { snprintf(msg, msg_cap, "rule %zu: base %d of state %d has a base itself", r, b, x); return -checked - 1; }
                for (int64_t w : waiters) {
                    if (w < 0) { cx.start((uint32_t)g.sid((int32_t)r, x)); cb.start((uint32_t)g.sid((int32_t)r, b)); }
                    else { cx.start_pair((uint32_t)g.sid((int32_t)r, x), (uint32_t)w); cb.start_pair((uint32_t)g.sid((int32_t)r, b), (uint32_t)w); }
                    for (int k = 0; k < n_tok; ++k) {
                        const size_t n = (size_t)(offs[k + 1] - offs[k]);
                        if (n == 0 || n > (size_t)d) continue;
                        ++checked;
                        const int rx = host_result(cx, bytes + offs[k], n), rb = host_result(cb, bytes + offs[k], n);
                        if (rx != rb) {
                            snprintf(msg, msg_cap, "rule %zu state %d (base %d, depth %d) waiter %lld token %d: %d vs %d", r, x, b, d, (long long)w, k, rx, rb);
                            return -checked - 1;
                        }
                    }
                }
            }
        }
        if (n_near) *n_near = near_states;
        if (max_depth) *max_depth = deepest;
        return checked;
    } catch (const std::exception& e) {
        snprintf(msg, msg_cap, "exception: %s", e.what());
        return -1;
    }
}
