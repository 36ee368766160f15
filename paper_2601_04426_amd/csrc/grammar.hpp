// Host-side grammar lowering: EBNF text -> one canonical minimal byte-level automaton per rule
// (XGrammar-2 section 3.3: "structures are represented as multiple FSMs", edges are character
// ranges or references to other FSMs), plus the structural hashes of Algorithm 1 / Algorithm 2.
#pragma once
#include <cstdint>
#include <functional>
#include <stdexcept>
#include <string>
#include <vector>

namespace xg2 {

struct ParseError : std::runtime_error { using std::runtime_error::runtime_error; };
struct GrammarError : std::runtime_error { using std::runtime_error::runtime_error; };

struct ByteRange { uint8_t lo, hi; int32_t tgt; };   // bytes lo..hi -> rule-local state tgt
struct RefEdge { int32_t rule; int32_t tgt; };       // reference to Grammar::rules[rule] -> state tgt

struct RuleFsm {
    std::string name;
    int32_t decl_index = 0;                           // position of the rule in the EBNF text
    std::vector<uint8_t> is_final;                    // [n_states]
    std::vector<std::vector<ByteRange>> bedges;       // sorted by lo; maximal runs per target
    std::vector<std::vector<RefEdge>> redges;         // sorted by referenced rule's decl_index
    bool nullable = false;
    int32_t min_len = 0;                              // length of the rule's shortest sentence, in bytes
    // structural hash (Algorithm 1, refined by Algorithm 2 inside simple reference cycles)
    uint64_t hash = 0;
    bool shareable = true;                            // false: member of a non-simple cycle, never reused
    std::vector<int32_t> canon_id;                    // Algorithm 1 phase 1: state -> canonical id
    std::vector<std::vector<RefEdge>> redges_by_hash; // out-references in the order Algorithm 1 sorted them
    std::vector<int32_t> ring;                        // simple cycle through this rule, starting at it (else empty)
    int32_t n_states() const { return (int32_t)is_final.size(); }
};

struct Position { int32_t rule, state, sid; };

struct Grammar {
    std::vector<RuleFsm> rules;                       // rules reachable from the root, in declaration order
    int32_t root = 0;
    std::vector<int32_t> state_base;                  // global state id = state_base[rule] + state
    int32_t n_states = 0;
    std::vector<Position> positions;                  // states with at least one byte edge
    std::vector<int32_t> sid_to_pos;                  // [n_states] -> index into positions or -1
    std::vector<std::vector<int32_t>> hash_order;     // reference-graph components, referenced rules first
    int32_t sid(int32_t rule, int32_t state) const { return state_base[rule] + state; }
};

// Throws ParseError (syntax) or GrammarError (undefined rule, empty language, unproductive rule,
// ill-formed TagDispatch).
Grammar lower_grammar(const std::string& ebnf, const std::string& root_rule);

std::string describe_grammar(const Grammar& g);       // JSON

uint64_t hash_combine(uint64_t h, uint64_t v);        // the order-sensitive hash of Algorithms 1 and 2

// States of one rule that no string of at most `budget` bytes can tell apart (bounded bisimulation):
// returns, per rule and state, the member of the state's class with the smallest canonical id.
// Rule edges are compared by ref_identity[rule] (rules known to be identical may share an identity).
// This is what makes planes independent of the bounds of a long repetition (section 3.6 observes
// that the states inside a repetition differ minimally): tokens are at most `budget` bytes long, so
// equivalent states have equal planes.
std::vector<std::vector<int32_t>> bounded_classes(const Grammar& g, int32_t budget, const std::vector<uint64_t>& ref_identity);
// One rule of the above.  The result depends only on the rule's structure and on the identities (and through them the
// shortest sentence and nullability) of the rules it references.
// near (optional): for the representative x of a class, near->base[x] is the representative of another class of the
// same rule that no string of at most near->depth[x] bytes tells apart from x (-1: none worth using), so the plane of
// x equals the plane of base[x] on every token of at most depth[x] bytes and only the longer tokens need checking.
// Bases are never derived themselves.
struct NearClasses { std::vector<int32_t> base, depth; };
constexpr int32_t kMinNearDepth = 3;       // shorter agreements save too few tokens to be worth a second pass
constexpr int32_t kMaxNearDepth = 32;
std::vector<int32_t> bounded_classes_rule(const Grammar& g, int32_t rule, int32_t budget, const std::vector<uint64_t>& ref_identity,
                                          NearClasses* near = nullptr);

// Per rule and per depth d <= budget, a 64-bit signature of everything that can follow an instance of the rule within
// d bytes in this grammar: the set of states referencing rules continue in (as structural hashes of their
// unfolding to the bytes that are left), recursively through rules that can end within the budget, and
// whether the input may end (root rule).  Two rules with equal signatures reject the same uncertain
// tokens by context expansion (section 2.2), so filtered planes can be shared across grammars
// (section 3.3: reuse needs matching lookahead).  Rules on a reference cycle through rule ends, or behind
// a cycle of nullable rule edges, get a process-unique signature (never shared, always sound).
struct FollowInfo {
    std::vector<std::vector<uint64_t>> sig;        // [rule][d], d = 0..budget: what can follow the rule within d bytes
    std::vector<std::vector<int32_t>> min_suf;     // [rule][state]: bytes of the shortest completion of the rule from the state
};
// rep (optional): per rule and state, a state that no string of at most `budget` bytes tells apart from it; sites are then
// taken at these representatives, which leaves the follow language as it is and the work independent of repetition bounds.
// ref_identity (optional): per rule, a number that identical rules share and different ones do not (the pool's entry);
// without it the rule's structural hash stands in.  intern (optional): gives every distinct description (a list of words)
// a number of its own, the same for the same list as long as the interner lives; the signatures are then such numbers
// and comparing them is exact, not merely probable.
using FollowInterner = std::function<uint64_t(const std::vector<uint64_t>&)>;
// memo_of (optional, with an interner): where the value of (rule, state, depth) is kept across calls, or null for rules
// that are not shared; a slot holding 0 is empty.
using FollowMemo = std::function<uint64_t*(int rule, int state, int depth)>;
FollowInfo follow_signatures(const Grammar& g, int32_t budget, const std::vector<std::vector<int32_t>>* rep = nullptr,
                             const std::vector<uint64_t>* ref_identity = nullptr, const FollowInterner* intern = nullptr,
                             const FollowMemo* memo_of = nullptr);

// Exact serialisation of one rule in Algorithm 1's canonical order; a reference to rule r is
// written as ref_id[r].  Two rules with equal text and equal meaning of the ids are isomorphic.
std::string serialise_rule(const Grammar& g, int32_t rule, const std::vector<uint64_t>& ref_id);
constexpr uint64_t kInCycleRef = 0x5EEDF00DCAFEBEEFull;   // the shared placeholder X of Algorithm 2

}  // namespace xg2
