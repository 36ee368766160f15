// The rule-scoped Earley recogniser the kernels run per lane (XGrammar-2 section 3.4 and the appendix on
// Earley parsing: scanner, predictor, completer over the per-rule automata), written once so that the same
// source also compiles for the host, where a test steps it against the host parser.  It only reads the
// packed tables and the caller's per-lane item store; it allocates nothing and every loop is bounded by a
// list capacity or by the token length.
#pragma once
#include "device.hpp"

namespace xg2 {
namespace core {

#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ uint32_t funnel_shift(uint32_t hi, uint32_t lo, uint32_t s) { return __builtin_amdgcn_alignbit(hi, lo, s); }
__device__ __forceinline__ bool wave_any(bool x) { return __any(x); }
#else
__device__ __forceinline__ uint32_t funnel_shift(uint32_t hi, uint32_t lo, uint32_t s) { return (uint32_t)(((((unsigned long long)hi) << 32) | lo) >> s); }
__device__ __forceinline__ bool wave_any(bool x) { return x; }      // the host build steps one lane at a time
#endif

// A state reference is 21 bits: state id (18) | has byte edge | has rule edge | final; an item is a state
// reference with the origin (item-set index, 2047 = root instance) in the upper 11 bits.
constexpr uint32_t SID_MASK = (1u << 18) - 1;
constexpr uint32_t F_BYTE = 1u << 18, F_REF = 1u << 19, F_FINAL = 1u << 20;
constexpr uint32_t REF_BITS = 21;
constexpr uint32_t ROOT_ORIGIN = (1u << (32 - REF_BITS)) - 1;
constexpr uint32_t NO_TARGET = 0xFFFFFFFFu;          // "none" marker in registers; the tables mark a missing edge by DevTables::sink

constexpr int RES_ALIVE = 1, RES_EARLY = 2, RES_OVERFLOW = 4, RES_LEFT_EARLY = 8 /* set by callers: left the outermost rule early, then died */;

struct DevCtx {                      // closed item set to continue from, plus what older sets wait for
    const uint32_t* items; uint32_t n_items;
    const uint2* wait; const uint32_t* wait_off; uint32_t H;    // pairs {rule, target | origin << 21} per set
};

// ---- token bytes, consumed front to back: in registers (at most 16) or in device memory ----------------
struct RegBytes {
    uint4 v;                                                    // a 128-bit shift register: no indexed access, no spill
    __device__ uint32_t peek() const { return v.x & 0xFF; }     // the byte next() would return
    __device__ uint32_t next() {
        const uint32_t b = v.x & 0xFF;
        v.x = funnel_shift(v.y, v.x, 8);
        v.y = funnel_shift(v.z, v.y, 8);
        v.z = funnel_shift(v.w, v.z, 8);
        v.w >>= 8;
        return b;
    }
};
struct MemBytes {
    const uint8_t* p;
    __device__ uint32_t peek() const { return *p; }
    __device__ uint32_t next() { return *p++; }
};

// Entering state `ref` with origin `origin` while set `set_idx` is under construction.  The item itself goes
// to `nxt` if its state can scan or complete (or has no edge at all); if it is there already nothing more
// happens.  A state with rule edges brings its expansion: every item that prediction, and advancing over
// rules that derive the empty string, add (already followed to the end on the host, so nothing added here
// needs expanding again) and one wait entry {rule, target | origin} per rule edge involved.  The flags
// travel with the state reference; memory is read only for expansions.
constexpr uint32_t REF_MASK = (1u << REF_BITS) - 1;

// A load from the grammar tables.  They always live in device memory; a kernel that got their addresses from memory
// itself (a batch of rows with a cache each) cannot know that, and would pay for generic-address loads.
template <class P>
__device__ __forceinline__ P tab(const P* p) {
#if defined(__HIP_DEVICE_COMPILE__)
    return *(const __attribute__((address_space(1))) P*)p;
#else
    return *p;
#endif
}
constexpr uint32_t EXP_CURRENT = 1u << REF_BITS;

// A list that is full, or a search bound that is used up, sets `full` and drops the entry; the caller looks at the flag
// once per byte (one way out of the step instead of one per call keeps the divergent control flow small).
template <class S>
__device__ __forceinline__ bool add_nxt(S& st, uint32_t item, int& nn, bool& full) {
    if (!st.charge(nn)) { full = true; return false; }           // large lists: a bound on the searching of one token
    bool found = false;                                          // no way out of the loop: one compare more costs less than the exit
    for (int k = 0; k < nn; ++k) found |= st.get_nxt(k) == item;
    if (found) return false;
    if (nn == st.K) { full = true; return false; }
    st.set_nxt(nn++, item);
    return true;                                                 // new in the list
}

template <class S>
__device__ __forceinline__ void add_wait(S& st, uint32_t rule, uint32_t tgt, int& nw, int wbeg, bool& full) {
    if (!st.charge(nw - wbeg)) { full = true; return; }
    bool found = false;
    for (int k = wbeg; k < nw; ++k) found |= (st.wait_tgt(k) == tgt) & (st.wait_rule(k) == rule);
    if (found) return;
    if (nw == st.WM) { full = true; return; }
    st.set_wait(nw++, rule, tgt);
}

// One byte of lookahead keeps the lists short: an item whose state has byte edges only and is not final can do nothing
// but scan, so if it has no edge for the byte that comes next it is left out (`la` = class of that byte, or NO_TARGET
// after the token's last byte, where every item counts because only "is the set empty" is asked).
__device__ __forceinline__ bool inert(const DevTables& T, uint32_t ref, uint32_t la) {
    return la != NO_TARGET && (ref & (F_BYTE | F_REF | F_FINAL)) == F_BYTE && tab(T.trans + (ref & SID_MASK) * T.n_classes + la) == T.sink;
}

template <class S>
__device__ __forceinline__ void enter(const DevTables& T, S& st, uint32_t ref, uint32_t origin, uint32_t set_idx, uint32_t la, int& nn, int& nw, int wbeg, bool& full) {
    if ((ref & (F_BYTE | F_FINAL)) || !(ref & F_REF)) {
        if (inert(T, ref, la)) return;
        if (!add_nxt(st, ref | (origin << REF_BITS), nn, full)) return;      // there already (or no room): nothing more to add
    }
    if (ref & F_REF) {
        const uint4 d = tab(T.state + (ref & SID_MASK));
        const uint32_t* e = T.exp_list + d.y;
        for (uint32_t k = 0; k < d.z; ++k) {
            const uint32_t w = tab(e + k);
            if (inert(T, w, la)) continue;
            add_nxt(st, (w & REF_MASK) | (((w & EXP_CURRENT) ? set_idx : origin) << REF_BITS), nn, full);
        }
        e += d.z;
        for (uint32_t k = 0; k < d.w; ++k) {
            const uint32_t w = tab(e + 2 * k + 1);
            add_wait(st, tab(e + 2 * k), (w & REF_MASK) | (((w & EXP_CURRENT) ? set_idx : origin) << REF_BITS), nw, wbeg, full);
        }
    }
}

// Earley recognition of the n bytes at tok, continuing from context C.  New item sets are numbered
// C.H, C.H + 1, ...  Returns RES_ALIVE if the set after the last byte is non-empty, RES_EARLY if the
// root instance could end after some proper non-empty prefix, RES_OVERFLOW if a list filled up.
// With FOLLOW, the end of the root instance is not the end of the parse: every state in which a rule
// referencing the ended rule continues (anywhere in the grammar) goes on as a new root instance, i.e.
// the rest of the token is matched against everything that can follow in some context.
// cls_words: the byte -> class table (64 words), in LDS or device memory.
//
// While the item set is a single item whose state has byte edges only (not final, no rule edge) the
// recogniser is a plain automaton walk: the item stays in a register and a byte costs one table load.
// The lists in `st` are used from the first state that predicts or completes, and left again when the
// set shrinks back to one such item (older wait entries stay where they are).
// What is left in the lists after the last byte, for a caller that goes on from there (a matcher accepting a token):
// the items of the last set are `one` if `single`, else cur[0 .. nc); the wait entries made during the token are
// wait[0 .. nw), those of new set j at [wstart(j), wstart(j + 1)) with wstart(n) = nw (with this output every new set's
// start is recorded, also the sets the automaton walk makes); root_done: the root instance can end after the last byte.
struct NoScanOut { static constexpr bool on = false; int nc; uint32_t one; bool single; int nw; bool root_done; };
struct ScanOut { static constexpr bool on = true; int nc = 0; uint32_t one = 0; bool single = false; int nw = 0; bool root_done = false; };

template <class S, bool FOLLOW = false, class BYTES = RegBytes, class OUT = NoScanOut>
__device__ int scan_token(const DevTables& T, const uint32_t* cls_words, const DevCtx& C, BYTES tok, int n, S& st, OUT* out = nullptr) {
    if (n > S::MAXLEN || (int)C.n_items > st.K) return RES_OVERFLOW;
    if (C.H + (uint32_t)n > ROOT_ORIGIN) return RES_OVERFLOW;       // the new sets C.H .. C.H + n - 1 must stay below the root mark
    int nc = (int)C.n_items;
    uint32_t one = nc == 1 ? C.items[0] : 0u;
    bool single = nc == 1 && (one & (F_BYTE | F_REF | F_FINAL)) == F_BYTE;
    if (!single) for (int k = 0; k < nc; ++k) st.set_cur(k, C.items[k]);
    int nw = 0;
    int res = 0;
    int i = 0;
    bool last_root = false;                                      // (OUT only) the root instance could end after the latest byte
    if (OUT::on) st.set_wstart(0, 0u);
    for (;;) {
        // ---- automaton walk: one item, in a register; a byte costs one table load ----------------
        uint32_t pending = NO_TARGET;
        while (single && i < n) {
            const uint32_t b = tok.next();
            const uint32_t cls = (cls_words[b >> 2] >> ((b & 3) * 8)) & 0xFF;
            const uint32_t tgt = tab(T.trans + (one & SID_MASK) * T.n_classes + cls);
            if (tgt == T.sink) return res;                       // dead
            if (tgt & (F_REF | F_FINAL)) { pending = tgt; single = false; break; }   // this state predicts or completes
            one = tgt | (one & ~REF_MASK);
            ++i;
            if (OUT::on) { last_root = false; if (i < n) st.set_wstart(i, (uint32_t)nw); }
        }
        if (i >= n) break;
        // ---- one general step for byte i ---------------------------------------------------------
        st.set_wstart(i, (uint32_t)nw);
        int nn = 0;
        const int wbeg = nw;
        const uint32_t set_idx = C.H + (uint32_t)i;
        bool full = false;
        uint32_t la = NO_TARGET;                                 // class of byte i + 1, if there is one
        {
            // scanner: one table word per scannable item (the automaton walk has looked its one word up already)
            const bool walked = pending != NO_TARGET;
            uint32_t cls = 0;
            if (!walked) {
                const uint32_t b = tok.next();
                cls = (cls_words[b >> 2] >> ((b & 3) * 8)) & 0xFF;
            }
            if (i + 1 < n) {                                     // (the automaton walk has consumed byte i already)
                const uint32_t b = tok.peek();
                la = (cls_words[b >> 2] >> ((b & 3) * 8)) & 0xFF;
            }
            const int n_scan = walked ? 1 : nc;
            for (int k = 0; k < n_scan; ++k) {
                uint32_t tgt = pending, origin = one >> REF_BITS;
                if (!walked) {
                    const uint32_t it = st.get_cur(k);
                    if (!(it & F_BYTE)) continue;
                    tgt = tab(T.trans + (it & SID_MASK) * T.n_classes + cls);
                    origin = it >> REF_BITS;
                }
                if (tgt != T.sink) enter(T, st, tgt, origin, set_idx, la, nn, nw, wbeg, full);
            }
        }
        // completer over the growing item list (prediction happened on entering).  What a completed item brings in
        // comes from one of three lists: the wait entries of its origin set made during this token, those of the
        // context, or (follow mode, end of the root instance) the states in which referencing rules continue.
        bool root_now = false;
        for (int pn = 0; pn < nn; ++pn) {
            const uint32_t it = st.get_nxt(pn);
            const uint32_t origin = it >> REF_BITS;
            if (!(it & F_FINAL) || origin == set_idx) continue;  // rules that derive the empty string were advanced over on entering
            const bool root_end = origin == ROOT_ORIGIN;
            if (root_end) {
                root_now = true;
                if (!FOLLOW) continue;
            }
            const uint32_t rule = tab(&T.state[it & SID_MASK].x);
            const bool local = !root_end && origin >= C.H;
            int lo, hi;
            if (root_end) { lo = (int)tab(T.site_off + rule); hi = (int)tab(T.site_off + rule + 1); }
            else if (local) { lo = (int)st.get_wstart((int)(origin - C.H)); hi = (int)st.get_wstart((int)(origin - C.H) + 1); }
            else { lo = (int)C.wait_off[origin]; hi = (int)C.wait_off[origin + 1]; }
            for (int k = lo; k < hi; ++k) {
                uint32_t wr, wt;
                if (root_end) { wr = rule; wt = tab(T.site_tgt + k) | (ROOT_ORIGIN << REF_BITS); }
                else if (local) { wr = st.wait_rule(k); wt = st.wait_tgt(k); }
                else { const uint2 w = C.wait[k]; wr = w.x; wt = w.y; }
                if (wr == rule) enter(T, st, wt & REF_MASK, wt >> REF_BITS, set_idx, la, nn, nw, wbeg, full);
            }
        }
        if (full) return RES_OVERFLOW;
        if (nn == 0 && nw == wbeg) return res;               // dead: nothing survives this byte
        if (root_now && i + 1 < n) res |= RES_EARLY;
        if (OUT::on) last_root = root_now;
        st.swap();
        nc = nn;
        ++i;
        if (i < n) st.set_wstart(i, (uint32_t)nw);             // sets made by the automaton walk add no wait entries
        if (nc == 1) {                                           // back to the register walk?
            one = st.get_cur(0);
            single = (one & (F_BYTE | F_REF | F_FINAL)) == F_BYTE;
        }
    }
    if (OUT::on) { out->nc = nc; out->one = one; out->single = single; out->nw = nw; out->root_done = last_root; }
    return res | RES_ALIVE;
}


// Phase 1 for a start set that is one item with byte edges only: the plain automaton walk of a wave's 64 tokens,
// without a branch inside.  A missing edge leads to the sink row of the table, which leads to itself, so a dead token
// simply stays there; a lane past the end of its token keeps its state.  What the walk met on the way is gathered in
// `seen` (the OR of the state references after each byte) and, for a plane whose start item is its outermost instance
// (ROOT: final states do not stop the walk, they only matter if the token dies later), in `seen_before_last` (the
// same without the last byte's target).
struct WalkResult { uint32_t state, seen, seen_before_last; };
template <bool ROOT>
__device__ __forceinline__ WalkResult walk_tokens(const uint32_t* __restrict__ trans, uint32_t n_classes, uint32_t sink, const uint8_t* cls_bytes,
                                                  uint32_t start, const uint4 tv, int n) {
    WalkResult r{n > 0 ? start : sink, 0u, 0u};
    const uint32_t words[4] = {tv.x, tv.y, tv.z, tv.w};
#pragma unroll
    for (int wi = 0; wi < 4; ++wi) {                                // unrolled: byte j of word wi is one bit-field extract
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = wi * 4 + j;
            const uint32_t b = (words[wi] >> (8 * j)) & 0xFF;
            const uint32_t t = trans[(r.state & SID_MASK) * n_classes + cls_bytes[b]];
            const bool live = i < n;
            if (ROOT) r.seen_before_last = live ? r.seen : r.seen_before_last;
            r.state = live ? t : r.state;
            r.seen |= r.state;                                      // idempotent once the token has ended
        }
        if (!wave_any(r.state != sink && (wi + 1) * 4 < n)) break;
    }
    return r;
}

}  // namespace core
}  // namespace xg2
