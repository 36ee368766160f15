#include "tables.hpp"

#include <algorithm>
#include <map>
#include <stdexcept>

namespace xg2 {

FlatTables flatten(const Grammar& g) {
    FlatTables t;
    t.state_info.resize((size_t)g.n_states);
    t.rule_info.resize(g.rules.size());
    for (size_t r = 0; r < g.rules.size(); ++r) {
        const RuleFsm& f = g.rules[r];
        t.rule_info[r] = {(uint32_t)g.sid((int32_t)r, 0), f.nullable ? 1u : 0u};
        for (int q = 0; q < f.n_states(); ++q) {
            StateInfo si;
            si.byte_off = (uint32_t)t.byte_edges.size();
            si.ref_off = (uint32_t)t.ref_edges.size();
            for (auto& e : f.bedges[(size_t)q]) t.byte_edges.push_back({(uint32_t)e.lo | ((uint32_t)e.hi << 8), (uint32_t)g.sid((int32_t)r, e.tgt)});
            for (auto& e : f.redges[(size_t)q]) t.ref_edges.push_back({(uint32_t)e.rule, (uint32_t)g.sid((int32_t)r, e.tgt)});
            si.counts = (uint32_t)f.bedges[(size_t)q].size() | ((uint32_t)f.redges[(size_t)q].size() << 16);
            si.rule_final = (uint32_t)r | (f.is_final[(size_t)q] ? 0x80000000u : 0u);
            t.state_info[(size_t)g.sid((int32_t)r, q)] = si;
        }
    }
    t.root_start = (uint32_t)g.sid(g.root, 0);
    // expansions: closure of prediction and of advancing over empty-deriving rules, per state with rule edges
    t.dev_state.resize(t.state_info.size());
    {
        std::vector<std::pair<uint32_t, uint32_t>> queue;            // (state, 1 = origin is the set being built)
        std::vector<uint32_t> items, triples;
        for (size_t sid = 0; sid < t.state_info.size(); ++sid) {
            const StateInfo& s0 = t.state_info[sid];
            DevState ds{s0.rule_final & 0x7FFFFFFFu, (uint32_t)t.exp_list.size(), 0, 0};
            if (s0.counts >> 16) {
                queue.assign(1, {(uint32_t)sid, 0u});
                items.clear(); triples.clear();
                auto enqueue = [&](uint32_t u, uint32_t cur) {
                    for (auto& q : queue) if (q.first == u && q.second == cur) return;
                    queue.emplace_back(u, cur);
                };
                for (size_t qi = 0; qi < queue.size(); ++qi) {
                    const uint32_t u = queue[qi].first, cur = queue[qi].second;
                    const StateInfo& su = t.state_info[u];
                    const uint32_t nb = su.counts & 0xFFFF, nr = su.counts >> 16;
                    const bool listed = nb > 0 || (su.rule_final >> 31) || nr == 0;   // scannable or completing
                    if (qi > 0 && listed) items.push_back(t.ref(u) | (cur ? kExpCurrent : 0u));
                    for (uint32_t k = 0; k < nr; ++k) {
                        const RefEdgeP& e = t.ref_edges[su.ref_off + k];
                        triples.push_back(e.rule);
                        triples.push_back(t.ref(e.tgt) | (cur ? kExpCurrent : 0u));
                        enqueue(t.rule_info[e.rule].start, 1u);
                        if (t.rule_info[e.rule].nullable) enqueue(e.tgt, cur);
                    }
                }
                ds.n_items = (uint32_t)items.size();
                ds.n_triples = (uint32_t)(triples.size() / 2);
                t.exp_list.insert(t.exp_list.end(), items.begin(), items.end());
                t.exp_list.insert(t.exp_list.end(), triples.begin(), triples.end());
            }
            t.dev_state[sid] = ds;
        }
    }
    // byte classes: refine by (class so far, target) state after state.  Every edge is a byte range, so bytes between
    // two consecutive range boundaries always behave alike: the refinement runs over those intervals, not over bytes.
    const size_t n = t.state_info.size();
    std::vector<uint8_t> is_bound(257, 0);
    is_bound[0] = 1;
    for (const ByteEdge& e : t.byte_edges) { is_bound[e.lohi & 0xFF] = 1; is_bound[((e.lohi >> 8) & 0xFF) + 1] = 1; }
    std::vector<uint32_t> iv_lo;                                    // first byte of every interval, ascending
    std::vector<uint32_t> iv_of(256);
    for (uint32_t b = 0; b < 256; ++b) {
        if (is_bound[b]) iv_lo.push_back(b);
        iv_of[b] = (uint32_t)iv_lo.size() - 1;
    }
    const size_t m = iv_lo.size();
    std::vector<uint32_t> cls(m, 0);
    std::vector<int64_t> row(m);
    struct Split { uint32_t old_class; int64_t target; uint32_t new_class; };
    std::vector<Split> splits;
    for (size_t sid = 0; sid < n; ++sid) {
        const StateInfo& si = t.state_info[sid];
        if (!(si.counts & 0xFFFF)) continue;
        std::fill(row.begin(), row.end(), -1);
        for (uint32_t k = 0; k < (si.counts & 0xFFFF); ++k) {
            const ByteEdge& e = t.byte_edges[si.byte_off + k];
            for (uint32_t j = iv_of[e.lohi & 0xFF]; j <= iv_of[(e.lohi >> 8) & 0xFF]; ++j) row[j] = e.tgt;
        }
        splits.clear();                                             // few per state: searched linearly
        for (size_t j = 0; j < m; ++j) {
            const uint32_t oc = cls[j];
            const int64_t tg = row[j];
            int nc = -1;
            for (const Split& sp : splits) if (sp.old_class == oc && sp.target == tg) { nc = (int)sp.new_class; break; }
            if (nc < 0) { nc = (int)splits.size(); splits.push_back({oc, tg, (uint32_t)nc}); }
            cls[j] = (uint32_t)nc;
        }
    }
    t.n_classes = *std::max_element(cls.begin(), cls.end()) + 1;
    if (t.n_classes > 256) throw std::logic_error("more byte classes than bytes");
    t.byte_class_words.assign(64, 0);
    for (int b = 0; b < 256; ++b) t.byte_class_words[(size_t)b >> 2] |= cls[iv_of[(size_t)b]] << ((b & 3) * 8);
    // one row more than there are states: the sink, which every missing edge leads to and which leads to itself, so
    // that an automaton walk needs no "is there an edge" branch (a dead run just stays in the sink)
    t.sink = (uint32_t)n;
    t.trans.assign((n + 1) * t.n_classes, t.sink);
    for (size_t sid = 0; sid < n; ++sid) {
        const StateInfo& si = t.state_info[sid];
        for (uint32_t k = 0; k < (si.counts & 0xFFFF); ++k) {
            const ByteEdge& e = t.byte_edges[si.byte_off + k];
            const uint32_t ref = t.ref(e.tgt);
            for (uint32_t j = iv_of[e.lohi & 0xFF]; j <= iv_of[(e.lohi >> 8) & 0xFF]; ++j) t.trans[sid * t.n_classes + cls[j]] = ref;
        }
    }
    return t;
}

namespace {
inline bool has(const std::vector<ChartItem>& v, ChartItem it) {
    for (auto& x : v) if (x.sid == it.sid && x.origin == it.origin) return true;
    return false;
}
}  // namespace

// Predictor and completer until nothing new.  A predicted rule that can derive the empty string
// also advances the predicting item at once, so completions with origin == index need no lookup.
void EarleyChart::close(ChartSet& set, int32_t index, std::vector<ChartItem>& pending) {
    while (!pending.empty()) {
        ChartItem it = pending.back();
        pending.pop_back();
        const StateInfo& si = t_->state_info[it.sid];
        uint32_t nb = si.counts & 0xFFFF, nr = si.counts >> 16;
        bool in_scan = nb > 0 || nr == 0, in_wait = nr > 0;
        if (in_scan) { if (has(set.scan, it)) continue; set.scan.push_back(it); }
        if (in_wait) { if (has(set.wait, it)) continue; set.wait.push_back(it); }
        for (uint32_t k = 0; k < nr; ++k) {
            const RefEdgeP& e = t_->ref_edges[si.ref_off + k];
            pending.push_back({t_->rule_info[e.rule].start, index});
            if (t_->rule_info[e.rule].nullable) pending.push_back({e.tgt, it.origin});
        }
        if (si.rule_final & 0x80000000u) {
            uint32_t rule = si.rule_final & 0x7FFFFFFFu;
            if (it.origin < 0) set.root_done = true;
            else if (it.origin != index)
                for (const ChartItem& w : chart_[(size_t)it.origin].wait) {
                    const StateInfo& wi = t_->state_info[w.sid];
                    for (uint32_t k = 0; k < (wi.counts >> 16); ++k) {
                        const RefEdgeP& e = t_->ref_edges[wi.ref_off + k];
                        if (e.rule == rule) pending.push_back({e.tgt, w.origin});
                    }
                }
        }
    }
}

void EarleyChart::start(uint32_t sid) {
    chart_.clear();
    chart_.emplace_back();
    std::vector<ChartItem> pending{{sid, -1}};
    close(chart_[0], 0, pending);
}

void EarleyChart::start_pair(uint32_t sid, uint32_t waiter_sid) {
    chart_.clear();
    chart_.emplace_back();
    chart_[0].wait.push_back({waiter_sid, -1});
    chart_.emplace_back();
    std::vector<ChartItem> pending{{sid, 0}};
    close(chart_[1], 1, pending);
}

bool EarleyChart::advance(const uint8_t* bytes, size_t n) {
    size_t keep = chart_.size();
    std::vector<ChartItem> pending;
    for (size_t i = 0; i < n; ++i) {
        uint8_t b = bytes[i];
        pending.clear();
        for (const ChartItem& it : chart_.back().scan) {
            const StateInfo& si = t_->state_info[it.sid];
            for (uint32_t k = 0; k < (si.counts & 0xFFFF); ++k) {
                const ByteEdge& e = t_->byte_edges[si.byte_off + k];
                if (b >= (e.lohi & 0xFF) && b <= ((e.lohi >> 8) & 0xFF)) { pending.push_back({e.tgt, it.origin}); break; }
            }
        }
        chart_.emplace_back();
        close(chart_.back(), (int32_t)chart_.size() - 1, pending);
        if (chart_.back().scan.empty() && chart_.back().wait.empty()) { chart_.resize(keep); return false; }
    }
    return true;
}

bool EarleyChart::context(ScanContext& out) const {
    out.items.clear(); out.wait.clear(); out.wait_off.clear();
    int32_t J = (int32_t)chart_.size() - 1;
    // sets reachable through origins, starting from the current set
    std::vector<int32_t> needed{J}, stack{J};
    std::map<int32_t, uint32_t> local;
    auto reach = [&](int32_t o) {
        if (o >= 0 && !std::binary_search(needed.begin(), needed.end(), o)) {
            needed.insert(std::upper_bound(needed.begin(), needed.end(), o), o);
            stack.push_back(o);
        }
    };
    for (const ChartItem& it : chart_[(size_t)J].scan) reach(it.origin);
    while (!stack.empty()) {
        int32_t s = stack.back(); stack.pop_back();
        for (const ChartItem& w : chart_[(size_t)s].wait) reach(w.origin);
    }
    if (needed.size() > kMaxLocalSets - 64) return false;
    for (size_t k = 0; k < needed.size(); ++k) local[needed[k]] = (uint32_t)k;
    out.H = (uint32_t)needed.size();
    auto loc = [&](int32_t o) { return o < 0 ? kRootOrigin : local.at(o); };
    for (const ChartItem& it : chart_[(size_t)J].scan) out.items.push_back(pack_item(t_->ref(it.sid), loc(it.origin)));
    for (size_t k = 0; k < needed.size(); ++k) {
        out.wait_off.push_back((uint32_t)(out.wait.size() / 2));
        for (const ChartItem& w : chart_[(size_t)needed[k]].wait) push_triples(w, loc(w.origin), out.wait);
    }
    out.wait_off.push_back((uint32_t)(out.wait.size() / 2));
    return true;
}

void EarleyChart::push_triples(const ChartItem& w, uint32_t local_origin, std::vector<uint32_t>& out) const {
    const StateInfo& wi = t_->state_info[w.sid];
    for (uint32_t k = 0; k < (wi.counts >> 16); ++k) {
        const RefEdgeP& e = t_->ref_edges[wi.ref_off + k];
        out.push_back(e.rule);
        out.push_back(pack_item(t_->ref(e.tgt), local_origin));
    }
}

}  // namespace xg2
