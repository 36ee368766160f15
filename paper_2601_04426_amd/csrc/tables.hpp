// Packed grammar tables shared by the host matcher and the device kernels (same words on both
// sides), and the host Earley parser that follows a sequence (XGrammar-2 section 3.4 and the
// appendix "Earley's Parsing Algorithm": predict / scan / complete over the per-rule automata).
#pragma once
#include <cstdint>
#include <memory>
#include <vector>

#include "grammar.hpp"

namespace xg2 {

// A state reference in 21 bits: global state id (18 bits) | has-byte-edge << 18 | has-rule-edge << 19 |
// final << 20, so that a kernel knows what to do with a state without loading anything.
// An Earley item in 32 bits: state reference | origin << 21.  The origin is the index of the item set in
// which the rule instance started, or kRootOrigin for the instance nobody is waiting for.
constexpr uint32_t kSidBits = 18;
constexpr uint32_t kSidMask = (1u << kSidBits) - 1;
constexpr uint32_t kRefBits = 21;
constexpr uint32_t kHasByte = 1u << 18, kHasRef = 1u << 19, kFinal = 1u << 20;
constexpr uint32_t kRootOrigin = (1u << (32 - kRefBits)) - 1;     // 2047
constexpr uint32_t kMaxLocalSets = kRootOrigin - 1;
inline uint32_t pack_item(uint32_t state_ref, uint32_t origin) { return state_ref | (origin << kRefBits); }

struct StateInfo { uint32_t byte_off, ref_off, counts /* n_byte | n_ref << 16 */, rule_final /* rule | final << 31 */; };
struct ByteEdge { uint32_t lohi /* lo | hi << 8 */, tgt; };
struct RefEdgeP { uint32_t rule, tgt; };
struct RuleInfo { uint32_t start, nullable; };
struct DevState { uint32_t rule, exp_off, n_items, n_triples; };
constexpr uint32_t kExpCurrent = 1u << kRefBits;

struct FlatTables {
    std::vector<StateInfo> state_info;
    std::vector<ByteEdge> byte_edges;
    std::vector<RefEdgeP> ref_edges;
    std::vector<RuleInfo> rule_info;
    uint32_t root_start = 0;
    // device-side forms: every stored state is a state reference (id | flags).
    // dev_state[sid] = {rule, offset into exp_list, n_items, n_triples}.  The expansion of a state with rule
    // edges lists everything that entering it adds to an Earley set besides the item itself, predictions and
    // advances over rules that derive the empty string followed to the end: first n_items item words
    // (state reference | kExpCurrent if the origin is the set being built, else the origin of the entering
    // item), then n_triples pairs {rule, state reference [| kExpCurrent]}: "when `rule`, started in this
    // set, completes, continue in that state".
    std::vector<DevState> dev_state;
    std::vector<uint32_t> exp_list;
    // dense byte transitions: bytes that lead to the same state from every state form one class;
    // trans[sid * n_classes + class] = state reference of the target, or `sink` where the state has no edge for the
    // byte; sink = number of states, a row of its own whose entries are all `sink` (no flags)
    std::vector<uint32_t> byte_class_words;      // 64 words: class of byte b = byte (b & 3) of word b >> 2
    uint32_t n_classes = 0;
    uint32_t sink = 0;
    std::vector<uint32_t> trans;
    uint32_t ref(uint32_t sid) const {
        const StateInfo& si = state_info[sid];
        return sid | ((si.counts & 0xFFFF) ? kHasByte : 0u) | ((si.counts >> 16) ? kHasRef : 0u) | ((si.rule_final >> 31) ? kFinal : 0u);
    }
};

FlatTables flatten(const Grammar& g);

// One closed Earley item set of the host parser.  `scan` holds the items whose state has a byte
// edge or no edge at all, `wait` those whose state has a rule edge (an item can be in both).
// Origins are chart indices; -1 marks the root instance.
struct ChartItem { uint32_t sid; int32_t origin; };            // origin -1 = root instance
struct ChartSet {
    std::vector<ChartItem> scan, wait;
    bool root_done = false;
};

// The context a kernel needs to continue parsing from a closed set: that set's scan items plus, for every
// set reachable through origins, what its waiting items wait for, with set indices renumbered 0..H-1 (the
// current set is H-1).  A waiting item with rule edge (rule -> target) gives the triple
// {rule, state reference of the target | local origin << 21}, two words.
struct ScanContext {
    std::vector<uint32_t> items;       // packed (state reference, local origin)
    std::vector<uint32_t> wait;        // triples, two words each, grouped by local set
    std::vector<uint32_t> wait_off;    // [H+1], in triples
    uint32_t H = 0;
};

class EarleyChart {
  public:
    explicit EarleyChart(const FlatTables* t) : t_(t) {}
    void start(uint32_t sid);                        // chart = closure{(sid, root instance)}
    // Two sets: set 0 holds only the waiting item (waiter_sid, root instance), set 1 is the closure of
    // (sid, origin 0): the rule instance of `sid` one level inside the rule of `waiter_sid`.
    void start_pair(uint32_t sid, uint32_t waiter_sid);
    const std::vector<ChartSet>& sets() const { return chart_; }
    const FlatTables* tables() const { return t_; }
    bool advance(const uint8_t* bytes, size_t n);    // all or nothing: false leaves the chart unchanged
    const ChartSet& last() const { return chart_.back(); }
    size_t length() const { return chart_.size(); }
    // false if more than kMaxLocalSets sets are reachable
    bool context(ScanContext& out) const;
    // appends the triples of waiting item `w` (origin already renumbered) to `out`
    void push_triples(const ChartItem& w, uint32_t local_origin, std::vector<uint32_t>& out) const;

  private:
    const FlatTables* t_;
    std::vector<ChartSet> chart_;
    void close(ChartSet& set, int32_t index, std::vector<ChartItem>& pending);
};

}  // namespace xg2
