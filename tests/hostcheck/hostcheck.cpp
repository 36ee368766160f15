// Test helper (CPU only): steps the recogniser core that the kernels run per lane, compiled for the host,
// against the host Earley parser of the library, for every plane context of a grammar and a list of tokens.
// Built by tests/test_host_logic.py with g++; it is not part of the library.
#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

#include <algorithm>
#include <map>

#include "../../paper_2601_04426_amd/csrc/accept_core.hpp"
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


// The device matcher's "accept a token" step (accept_core.hpp), compiled for the host, against the host Earley parser:
// along every token sequence given (ids into the token list, -1 ends a sequence) the context it writes must equal
// EarleyChart::context() after the same tokens (same sets in the same order; items and wait entries as sets), the
// root-can-end flag must agree, rejected tokens must be rejected and leave the state alone, and the frontier planes must
// be the ones the host's rule gives (plane tables here hold made-up row numbers, one per (state) and (state, site)).
// Extra tokens tried at every step (try_ids) exercise rejection.  Returns steps checked or -1 with a message.
namespace {
struct HostX {
    std::vector<uint8_t> map; std::vector<uint64_t> front;
    HostX(size_t n_map, size_t n_front) : map(n_map), front(n_front) {}
    uint32_t map_cap() const { return (uint32_t)map.size(); }
    uint32_t front_cap() const { return (uint32_t)front.size(); }
    uint32_t map_get(uint32_t i) const { return map.at(i); }
    void map_set(uint32_t i, uint32_t v) { map.at(i) = (uint8_t)v; }
    uint64_t front_get(uint32_t k) const { return front.at(k); }
    void front_set(uint32_t k, uint64_t v) { front.at(k) = v; }
};
}  // namespace

extern "C" long long xg2hc_check_accept(const char* ebnf, size_t len, const char* root, const uint8_t* bytes, const uint64_t* offs, int n_tok,
                                        const int32_t* seq, int n_seq, const int32_t* try_ids, int n_try, int small_lists, char* msg, size_t msg_cap) {
    try {
        Grammar g = lower_grammar(std::string(ebnf, len), root);
        FlatTables ft = flatten(g);
        CacheDev Cd{};
        Cd.T.state = reinterpret_cast<const uint4*>(ft.dev_state.data());
        Cd.T.exp_list = ft.exp_list.data();
        Cd.T.trans = ft.trans.data();
        Cd.T.byte_class_words = ft.byte_class_words.data();
        Cd.T.n_classes = ft.n_classes;
        Cd.T.sink = ft.sink;
        Cd.context_depth = 2;
        // made-up plane rows: plain plane of state s = (s + 1) << 4; plane of (s, site state x) numbered as listed
        const size_t n_states = ft.state_info.size();
        std::vector<uint64_t> plain(n_states);
        for (size_t sid = 0; sid < n_states; ++sid) plain[sid] = (uint64_t)(sid + 1) << 4;
        std::vector<uint32_t> pair_off(n_states + 1, 0), pair_key;
        std::vector<uint64_t> pair_row;
        std::map<std::pair<uint32_t, uint32_t>, uint64_t> pair_of;
        for (size_t sid = 0; sid < n_states; ++sid) {
            const uint32_t rule = ft.state_info[sid].rule_final & 0x7FFFFFFFu;
            for (const RefEdgeP& e : ft.ref_edges)
                if (e.rule == rule && !pair_of.count({(uint32_t)sid, e.tgt})) {
                    const uint64_t row = ((uint64_t)(n_states + pair_of.size() + 1)) << 4;
                    pair_of[{(uint32_t)sid, e.tgt}] = row;
                }
        }
        for (auto& kv : pair_of) {                                  // sorted by state, then by site: the order the look-up expects
            pair_key.push_back(kv.first.second); pair_row.push_back(kv.second);
            ++pair_off[(size_t)kv.first.first + 1];
        }
        for (size_t sid = 0; sid < n_states; ++sid) pair_off[sid + 1] += pair_off[sid];
        if (pair_key.empty()) { pair_key.push_back(0); pair_row.push_back(0); }
        Cd.plain_row = plain.data(); Cd.pair_off = pair_off.data(); Cd.pair_key = pair_key.data(); Cd.pair_row = pair_row.data();
        const uint32_t KI = 64, KH = 240, KW = 512, KF = 16;
        struct State { std::vector<uint32_t> items, wait_off; std::vector<uint2> wait; uint32_t H = 0; bool root_done = false; std::vector<uint64_t> front; };
        auto host_state = [&](const EarleyChart& chart) {
            State s;
            // sets still reachable from the items that can scan (and the current set), through the origins of waiting items
            const auto& sets = chart.sets();
            const int32_t J = (int32_t)sets.size() - 1;
            std::vector<uint8_t> need(sets.size(), 0);
            need[(size_t)J] = 1;
            for (const ChartItem& it : sets[(size_t)J].scan)
                if ((ft.state_info[it.sid].counts & 0xFFFF) && it.origin >= 0) need[(size_t)it.origin] = 1;
            for (int32_t k = J; k >= 0; --k)
                if (need[(size_t)k]) for (const ChartItem& w : sets[(size_t)k].wait) if (w.origin >= 0) need[(size_t)w.origin] = 1;
            std::vector<uint32_t> local(sets.size(), 0);
            for (size_t k = 0; k < sets.size(); ++k) if (need[k]) local[k] = s.H++;
            auto loc = [&](int32_t o) { return o < 0 ? kRootOrigin : local[(size_t)o]; };
            for (const ChartItem& it : sets[(size_t)J].scan)
                if (ft.state_info[it.sid].counts & 0xFFFF) s.items.push_back(pack_item(ft.ref(it.sid), loc(it.origin)));
            std::vector<uint32_t> flat;
            for (size_t k = 0; k < sets.size(); ++k) {
                if (!need[k]) continue;
                s.wait_off.push_back((uint32_t)s.wait.size());
                flat.clear();
                for (const ChartItem& w : sets[k].wait) chart.push_triples(w, loc(w.origin), flat);
                for (size_t q = 0; q + 1 < flat.size(); q += 2) s.wait.push_back(make_uint2(flat[q], flat[q + 1]));
            }
            s.wait_off.push_back((uint32_t)s.wait.size());
            s.root_done = chart.last().root_done;
            // the host's rule for the frontier planes
            for (const ChartItem& it : chart.last().scan) {
                const StateInfo& si = ft.state_info[it.sid];
                if (!(si.counts & 0xFFFF)) continue;
                auto add = [&](uint64_t row) {
                    for (uint64_t& have : s.front) if ((have & ~(uint64_t)1) == (row & ~(uint64_t)1)) { have &= row | ~(uint64_t)1; return; }
                    s.front.push_back(row);
                };
                if (it.origin < 0) { add(plain[it.sid] | 1u); continue; }
                const uint32_t rule = si.rule_final & 0x7FFFFFFFu;
                for (const ChartItem& w : chart.sets()[(size_t)it.origin].wait) {
                    const StateInfo& wi = ft.state_info[w.sid];
                    for (uint32_t k = 0; k < (wi.counts >> 16); ++k) {
                        const RefEdgeP& e = ft.ref_edges[wi.ref_off + k];
                        if (e.rule == rule) add(pair_of.at({it.sid, e.tgt}));
                    }
                }
            }
            return s;
        };
        auto same = [&](const State& a, const State& b, std::string& why) {
            if (a.H != b.H) { why = "number of sets " + std::to_string(a.H) + " vs " + std::to_string(b.H); return false; }
            if (a.root_done != b.root_done) { why = "root-can-end flag"; return false; }
            std::vector<uint32_t> ia = a.items, ib = b.items;
            std::sort(ia.begin(), ia.end()); std::sort(ib.begin(), ib.end());
            if (ia != ib) { why = "items"; return false; }
            for (uint32_t s = 0; s < a.H; ++s) {
                std::vector<std::pair<uint32_t, uint32_t>> wa, wb;
                for (uint32_t k = a.wait_off[s]; k < a.wait_off[s + 1]; ++k) wa.emplace_back(a.wait[k].x, a.wait[k].y);
                for (uint32_t k = b.wait_off[s]; k < b.wait_off[s + 1]; ++k) wb.emplace_back(b.wait[k].x, b.wait[k].y);
                std::sort(wa.begin(), wa.end()); wa.erase(std::unique(wa.begin(), wa.end()), wa.end());
                std::sort(wb.begin(), wb.end()); wb.erase(std::unique(wb.begin(), wb.end()), wb.end());
                if (wa != wb) { why = "wait entries of set " + std::to_string(s); return false; }
            }
            std::vector<uint64_t> fa = a.front, fb = b.front;
            std::sort(fa.begin(), fa.end()); std::sort(fb.begin(), fb.end());
            if (fa != fb) { why = "frontier planes"; return false; }
            return true;
        };
        // one accept step on the device-side state `cur`: 0 accepted (next filled), 1 rejected, else error
        auto step = [&](const State& cur, const uint8_t* t, int n, State& next) -> int {
            MatcherIn in{cur.items.data(), (uint32_t)cur.items.size(), cur.wait.data(), cur.wait_off.data(), cur.H};
            next.items.assign(KI, 0); next.wait.assign(KW, make_uint2(0, 0)); next.wait_off.assign(KH + 1, 0); next.front.assign(KF, 0);
            MatcherOut out{next.items.data(), next.wait.data(), next.wait_off.data(), next.front.data(), KI, KH, KW, KF, 0, 0, 0, 0};
            int acc;
            if (small_lists) {
                HostStore<8, 12, 16> st;
                HostX x(256, 16);
                acc = accept_token(Cd, ft.byte_class_words.data(), in, t, n, st, x, out);
                if (acc != ACC_RETRY) goto done;
            }
            {
                HostStore<256, 1024, 1024> st;
                HostX x(KH + 1025, KF);
                acc = accept_token(Cd, ft.byte_class_words.data(), in, t, n, st, x, out);
            }
        done:
            if (acc == ACC_REJECTED) return 1;
            if (acc != ACC_OK) return 2 + acc;
            next.items.resize(out.n_items); next.H = out.H; next.wait_off.resize(out.H + 1); next.wait.resize(next.wait_off[out.H]);
            next.front.resize(out.n_front); next.root_done = out.root_done != 0;
            return 0;
        };
        long long checked = 0;
        EarleyChart chart(&ft);
        chart.start(ft.root_start);
        State cur = host_state(chart);
        for (int q = 0; q < n_seq; ++q) {
            if (seq[q] < 0) { chart.start(ft.root_start); cur = host_state(chart); continue; }
            // tokens that may or may not be allowed here
            for (int k = 0; k <= n_try; ++k) {
                const int id = k < n_try ? try_ids[k] : seq[q];
                const uint8_t* t = bytes + offs[id];
                const int n = (int)(offs[id + 1] - offs[id]);
                if (n == 0) continue;
                EarleyChart probe = chart;
                const bool host_ok = probe.advance(t, (size_t)n);
                State next;
                const int rc = step(cur, t, n, next);
                ++checked;
                if (rc > 1) { snprintf(msg, msg_cap, "step %d token %d: accept failed with code %d", q, id, rc - 2); return -1; }
                if ((rc == 0) != host_ok) { snprintf(msg, msg_cap, "step %d token %d: host parser %s, device matcher %s", q, id, host_ok ? "accepts" : "rejects", rc == 0 ? "accepts" : "rejects"); return -1; }
                if (host_ok) {
                    std::string why;
                    if (!same(next, host_state(probe), why)) { snprintf(msg, msg_cap, "step %d token %d: %s differ", q, id, why.c_str()); return -1; }
                }
                if (k == n_try) {
                    if (!host_ok) { snprintf(msg, msg_cap, "step %d: the sequence's own token %d is rejected", q, id); return -1; }
                    chart = probe; cur = next;
                }
            }
        }
        return checked;
    } catch (const std::exception& e) {
        snprintf(msg, msg_cap, "exception: %s", e.what());
        return -1;
    }
}
