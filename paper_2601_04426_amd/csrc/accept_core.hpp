// Accepting a token on the device (XGrammar-2 section 3.4: the parser traces the output; appendix on Earley parsing):
// the recogniser of earley_core.hpp runs the token's bytes from the matcher's context, and what it leaves in its lists
// becomes the matcher's next context: the scannable items of the new current set, the wait entries of every older set
// that is still reachable through origins (renumbered 0 .. H - 1 in their old order, the current set last), and the
// planes of the new scannable frontier.  Written once for device and host (a CPU test steps it against the host parser).
#pragma once
#include "earley_core.hpp"

namespace xg2 {
namespace core {

struct MatcherIn {                   // the context to continue from
    const uint32_t* items; uint32_t n_items; const uint2* wait; const uint32_t* wait_off; uint32_t H;
};
struct MatcherOut {                  // where the next context goes, and how much room there is
    uint32_t* items; uint2* wait; uint32_t* wait_off; uint64_t* front;
    uint32_t KI, KH, KW, KF;
    uint32_t n_items, H, n_front, root_done;     // results
};
constexpr int ACC_OK = 0, ACC_REJECTED = 1, ACC_RETRY = 2 /* the recogniser's lists were too short */, ACC_OVERFLOW = 3 /* the slot is */,
              ACC_NO_PLANE = 4;

// X: per-lane scratch: a byte per item set (renumbering) and a few 64-bit words (frontier planes before they are stored).
//   uint32_t map_get(uint32_t i), void map_set(uint32_t i, uint32_t v); uint64_t front_get(uint32_t k), void front_set(uint32_t k, uint64_t v);
//   uint32_t map_cap() sets, uint32_t front_cap() planes.
template <class S, class X>
__device__ int accept_token(const CacheDev& Cd, const uint32_t* cls_words, const MatcherIn& in, const uint8_t* bytes, int n, S& st, X& x, MatcherOut& out) {
    const DevTables& T = Cd.T;
    DevCtx C;
    C.items = in.items; C.n_items = in.n_items; C.wait = in.wait; C.wait_off = in.wait_off; C.H = in.H;
    ScanOut so;
    MemBytes tok{bytes};
    const int res = scan_token<S, false, MemBytes, ScanOut>(T, cls_words, C, tok, n, st, &so);
    if (res & RES_OVERFLOW) return ACC_RETRY;
    if (!(res & RES_ALIVE)) return ACC_REJECTED;
    const uint32_t H = in.H, n_sets = H + (uint32_t)n;           // old numbering: sets 0 .. n_sets - 1, the last one is the new current set
    if (n_sets > x.map_cap()) return ACC_RETRY;
    const int nc = so.single ? 1 : so.nc;
    auto item_at = [&](int k) { return so.single ? so.one : st.get_cur(k); };
    // the wait entries of old-numbered set s: in the context, or made during this token
    auto wait_range = [&](uint32_t s, uint32_t& lo, uint32_t& hi) {
        if (s < H) { lo = in.wait_off[s]; hi = in.wait_off[s + 1]; }
        else { const uint32_t j = s - H; lo = st.get_wstart((int)j); hi = j + 1 < (uint32_t)n ? st.get_wstart((int)j + 1) : (uint32_t)so.nw; }
    };
    auto wait_at = [&](uint32_t s, uint32_t k, uint32_t& rule, uint32_t& tgt) {
        if (s < H) { const uint2 w = in.wait[k]; rule = w.x; tgt = w.y; }
        else { rule = st.wait_rule((int)k); tgt = st.wait_tgt((int)k); }
    };
    // 1. the sets still reachable: the current one, the origins of its items, and on from there through the wait entries
    //    (an entry's origin is never above its own set, so one pass downwards settles it)
    for (uint32_t s = 0; s < n_sets; ++s) x.map_set(s, 0u);
    x.map_set(n_sets - 1, 1u);
    for (int k = 0; k < nc; ++k) {
        const uint32_t it = item_at(k);
        if ((it & F_BYTE) && (it >> REF_BITS) != ROOT_ORIGIN) x.map_set(it >> REF_BITS, 1u);
    }
    for (uint32_t s = n_sets; s-- > 0;) {
        if (!x.map_get(s)) continue;
        uint32_t lo, hi;
        wait_range(s, lo, hi);
        for (uint32_t k = lo; k < hi; ++k) {
            uint32_t rule, tgt;
            wait_at(s, k, rule, tgt);
            if ((tgt >> REF_BITS) != ROOT_ORIGIN) x.map_set(tgt >> REF_BITS, 1u);
        }
    }
    // 2. new numbers (stored + 1; 0 = dropped), and the wait entries of the kept sets
    uint32_t newH = 0, nw_out = 0;
    for (uint32_t s = 0; s < n_sets; ++s) {
        if (!x.map_get(s)) continue;
        if (newH >= out.KH) return ACC_OVERFLOW;
        x.map_set(s, newH + 1);                                  // origins point downwards: every origin of this set has its number already
        out.wait_off[newH] = nw_out;
        ++newH;
        uint32_t lo, hi;
        wait_range(s, lo, hi);
        for (uint32_t k = lo; k < hi; ++k) {
            uint32_t rule, tgt;
            wait_at(s, k, rule, tgt);
            const uint32_t o = tgt >> REF_BITS;
            if (nw_out >= out.KW) return ACC_OVERFLOW;
            out.wait[nw_out++] = make_uint2(rule, (tgt & REF_MASK) | ((o == ROOT_ORIGIN ? ROOT_ORIGIN : x.map_get(o) - 1) << REF_BITS));
        }
    }
    out.wait_off[newH] = nw_out;
    // 3. the items that can scan, and 4. the planes of that frontier
    uint32_t ni = 0, nf = 0;
    for (int k = 0; k < nc; ++k) {
        const uint32_t it = item_at(k);
        if (!(it & F_BYTE)) continue;                            // final-only items have done their work in the closure
        const uint32_t o = it >> REF_BITS, sid = it & SID_MASK;
        if (ni >= out.KI) return ACC_OVERFLOW;
        out.items[ni++] = (it & REF_MASK) | ((o == ROOT_ORIGIN ? ROOT_ORIGIN : x.map_get(o) - 1) << REF_BITS);
        auto add_plane = [&](uint64_t row) -> bool {
            for (uint32_t f = 0; f < nf; ++f) {
                const uint64_t have = x.front_get(f);
                if ((have & ~(uint64_t)1) == (row & ~(uint64_t)1)) { x.front_set(f, have & (row | ~(uint64_t)1)); return true; }
            }
            if (nf >= x.front_cap() || nf >= out.KF) return false;
            x.front_set(nf++, row);
            return true;
        };
        if (o == ROOT_ORIGIN || Cd.context_depth == 1) {
            // the root instance: leaving the rule leaves the grammar, so its uncertain tokens are never allowed
            const uint64_t row = tab(Cd.plain_row + sid);
            if (!row) return ACC_NO_PLANE;
            if (!add_plane(o == ROOT_ORIGIN ? (row | 1u) : row)) return ACC_OVERFLOW;
            continue;
        }
        const uint32_t rule = tab(&T.state[sid].x);
        uint32_t lo, hi;
        wait_range(o, lo, hi);
        bool any = false;
        for (uint32_t k = lo; k < hi; ++k) {
            uint32_t wr, wt;
            wait_at(o, k, wr, wt);
            if (wr != rule) continue;
            const uint32_t key = wt & SID_MASK;
            // the state's planes are sorted by site (a state inside a long repetition is referenced from thousands of states)
            const uint32_t end_j = tab(Cd.pair_off + sid + 1);
            uint32_t lo_j = tab(Cd.pair_off + sid), hi_j = end_j;
            while (lo_j < hi_j) {
                const uint32_t mid = (lo_j + hi_j) >> 1;
                if (tab(Cd.pair_key + mid) < key) lo_j = mid + 1; else hi_j = mid;
            }
            if (lo_j >= end_j || tab(Cd.pair_key + lo_j) != key) return ACC_NO_PLANE;
            const uint64_t row = tab(Cd.pair_row + lo_j);
            if (!row) return ACC_NO_PLANE;
            if (!add_plane(row)) return ACC_OVERFLOW;
            any = true;
        }
        if (!any) return ACC_NO_PLANE;
    }
    for (uint32_t f = 0; f < nf; ++f) out.front[f] = x.front_get(f);
    out.n_items = ni; out.H = newH; out.n_front = nf; out.root_done = so.root_done ? 1u : 0u;
    return ACC_OK;
}

}  // namespace core
}  // namespace xg2
