// gfx950 (CDNA4, wave64) kernels of the token-mask cache path:
//   k_build        classes of (position, token) pairs by a rule-scoped Earley recogniser, one lane per
//                  token, item sets in LDS                              (XGrammar-2 section 3.4)
//   k_build_slow   the same recogniser with larger item sets (LDS, then device memory), for lanes that overflowed
//   k_copy_masked  short tokens of a plane taken from the plane of a state they cannot tell apart (section 3.6)
//   k_copy_first_byte  tokens of a plane taken from the plane of a state that moves alike on their first byte
//   k_upload       per-call plan and tables from pinned host memory
//   k_stage        the same for a build, together with the clearing of fresh rows and the chunk records
//   k_plane_summary  per built plane: bit counts, and the short list of its uncertain tokens that the fill reads
//   k_finish_planes  the copy kernels and the summary in one pass, when no derived plane leans on another derived one
//   k_fill         union of cached planes over the scannable frontier and, beside it, the re-check of the uncertain
//                  tokens against the full Earley context              (section 3.4, runtime part)
//   k_recheck_slow the re-check with larger item sets, for the tokens that overflowed the short ones
//   k_apply_*      logits of disallowed tokens := -infinity, in place    (section 2.1)
// No MFMA: nothing here is a contraction.  All device writes are vector stores or LDS/L2 atomics.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "device.hpp"
#include "earley_core.hpp"
#include "accept_core.hpp"

namespace xg2 {
namespace {

using namespace core;

// ---- per-lane item storage -------------------------------------------------------------------------
// LDS: word (slot, column) lives at slot * COLS + column (a lane's column is its place among the lanes at work), so a
// wave touching one slot per lane hits every bank once per 32 lanes whatever the slots are.
template <int K_, int WM_, int COLS_ = 64>
struct LdsStore {
    static constexpr int K = K_, WM = WM_, MAXLEN = 16, COLS = COLS_, SLOTS = 2 * K_ + 2 * WM_;
    uint32_t* cur; uint32_t* nxt; uint32_t* wait;  // this lane's column of the two item lists and the wait list (two words an entry)
    unsigned long long ws_lo = 0, ws_hi = 0;        // wait-list length at the start of each new set, 8 bits each
    __device__ void init(uint32_t* base) { cur = base; nxt = base + K * COLS; wait = base + 2 * K * COLS; }
    __device__ uint32_t get_cur(int k) const { return cur[k * COLS]; }
    __device__ void set_cur(int k, uint32_t v) { cur[k * COLS] = v; }
    __device__ uint32_t get_nxt(int k) const { return nxt[k * COLS]; }
    __device__ void set_nxt(int k, uint32_t v) { nxt[k * COLS] = v; }
    __device__ uint32_t wait_rule(int k) const { return wait[k * 2 * COLS]; }
    __device__ uint32_t wait_tgt(int k) const { return wait[k * 2 * COLS + COLS]; }
    __device__ void set_wait(int k, uint32_t rule, uint32_t tgt) { wait[k * 2 * COLS] = rule; wait[k * 2 * COLS + COLS] = tgt; }
    __device__ void swap() { uint32_t* t = cur; cur = nxt; nxt = t; }
    __device__ bool charge(int) { return true; }   // short lists: nothing to bound
    __device__ void reset() { ws_lo = 0; ws_hi = 0; }
    __device__ void set_wstart(int j, uint32_t v) {
        const int sh = 8 * (j & 7);
        unsigned long long& w = j < 8 ? ws_lo : ws_hi;
        w = (w & ~(0xFFull << sh)) | ((unsigned long long)v << sh);
    }
    __device__ uint32_t get_wstart(int j) const {
        return (uint32_t)((j < 8 ? ws_lo >> (8 * j) : ws_hi >> (8 * (j - 8))) & 0xFF);
    }
};

// The same layout with more room and the set starts in LDS too: the first resort of the large-capacity kernels
// (one wave per workgroup, 37 KB), before the lists in device memory.
template <int K_, int WM_, int MAXLEN_>
struct LdsStoreWide {
    static constexpr int K = K_, WM = WM_, MAXLEN = MAXLEN_, SLOTS = 2 * K_ + 2 * WM_ + MAXLEN_ + 1;
    uint32_t* cur; uint32_t* nxt; uint32_t* wait; uint32_t* ws;
    __device__ void init(uint32_t* base) { cur = base; nxt = base + K * 64; wait = base + 2 * K * 64; ws = base + (2 * K + 2 * WM) * 64; }
    __device__ uint32_t get_cur(int k) const { return cur[k * 64]; }
    __device__ void set_cur(int k, uint32_t v) { cur[k * 64] = v; }
    __device__ uint32_t get_nxt(int k) const { return nxt[k * 64]; }
    __device__ void set_nxt(int k, uint32_t v) { nxt[k * 64] = v; }
    __device__ uint32_t wait_rule(int k) const { return wait[k * 128]; }
    __device__ uint32_t wait_tgt(int k) const { return wait[k * 128 + 64]; }
    __device__ void set_wait(int k, uint32_t rule, uint32_t tgt) { wait[k * 128] = rule; wait[k * 128 + 64] = tgt; }
    __device__ void swap() { uint32_t* t = cur; cur = nxt; nxt = t; }
    __device__ bool charge(int) { return true; }
    __device__ void reset() {}
    __device__ void set_wstart(int j, uint32_t v) { ws[j * 64] = v; }
    __device__ uint32_t get_wstart(int j) const { return ws[j * 64]; }
};
using MidStore = LdsStoreWide<16, 32, 48>;

// Device memory: word (slot, lane) lives at slot * n_lanes + lane (coalesced across lanes).
struct GlobalStore {
    static constexpr int MAXLEN = kSlowMaxLen;
    int K = kSlowK, WM = kSlowWM;                   // capacities in use (the memory is laid out for kSlowK, kSlowWM)
    uint32_t* cur; uint32_t* nxt; uint32_t* wait; uint32_t* ws; size_t stride;
    uint32_t budget = kSlowSearchBudget;           // list entries one token may still compare against: a bound on its run time
    __device__ bool charge(int n) { if ((uint32_t)n > budget) { budget = 0; return false; } budget -= (uint32_t)n; return true; }
    __device__ void init(uint32_t* base, size_t n_lanes, uint32_t k_cap = kSlowK, uint32_t wm_cap = kSlowWM) {
        K = (int)min(k_cap, kSlowK); WM = (int)min(wm_cap, kSlowWM);
        stride = n_lanes; cur = base; nxt = base + (size_t)kSlowK * stride; wait = base + (size_t)2 * kSlowK * stride;
        ws = base + (size_t)(2 * kSlowK + 2 * kSlowWM) * stride;
    }
    __device__ uint32_t get_cur(int k) const { return cur[(size_t)k * stride]; }
    __device__ void set_cur(int k, uint32_t v) { cur[(size_t)k * stride] = v; }
    __device__ uint32_t get_nxt(int k) const { return nxt[(size_t)k * stride]; }
    __device__ void set_nxt(int k, uint32_t v) { nxt[(size_t)k * stride] = v; }
    __device__ uint32_t wait_rule(int k) const { return wait[(size_t)(2 * k) * stride]; }
    __device__ uint32_t wait_tgt(int k) const { return wait[(size_t)(2 * k + 1) * stride]; }
    __device__ void set_wait(int k, uint32_t rule, uint32_t tgt) { wait[(size_t)(2 * k) * stride] = rule; wait[(size_t)(2 * k + 1) * stride] = tgt; }
    __device__ void swap() { uint32_t* t = cur; cur = nxt; nxt = t; }
    __device__ void reset() { budget = kSlowSearchBudget; }
    __device__ void set_wstart(int j, uint32_t v) { ws[(size_t)j * stride] = v; }
    __device__ uint32_t get_wstart(int j) const { return ws[(size_t)j * stride]; }
};

#ifndef XG2_BUILD_ATTR
#define XG2_BUILD_ATTR
#endif
// Item-list capacities of the LDS path with all 64 lanes at work: the host picks one of two sizes per launch (see
// launch_build); the LDS of a workgroup is sized to match.
#ifndef XG2_BUILD_K_SMALL
#define XG2_BUILD_K_SMALL 3
#define XG2_BUILD_WM_SMALL 4
#endif
#ifndef XG2_BUILD_LEVELS
#define XG2_BUILD_LEVELS 3
#endif
constexpr int BUILD_LEVELS = XG2_BUILD_LEVELS;        // 64, 32, 16, ... lanes at work with 1, 2, 4, ... times the capacity
constexpr int BUILD_K_SMALL = XG2_BUILD_K_SMALL, BUILD_WM_SMALL = XG2_BUILD_WM_SMALL, BUILD_K_LARGE = 6, BUILD_WM_LARGE = 10;

// The build kernel's item lists: the LDS layout above with capacities chosen at run time.  The lists are kept short
// because their size bounds how many workgroups a compute unit holds, and the kernel lives on hiding the latency of
// dependent table loads behind other wavefronts.  A token that outgrows them is run again with only the lower 32 lanes
// at work, each with two lanes' worth of the same memory (word (slot, lane) at slot * 32 + lane): twice the capacity,
// no more LDS; one that outgrows those too, once more with 16 lanes and four times the capacity (BUILD_LEVELS).
struct BuildStore {
    static constexpr int MAXLEN = 16;
    int K, WM, sh;                                  // capacities; log2 of the distance between a lane's consecutive slots
    uint32_t* cur; uint32_t* nxt; uint32_t* wait;
    unsigned long long ws_lo = 0, ws_hi = 0;        // wait-list length at the start of each new set, 8 bits each
    // lds: the workgroup's (2 k + 2 wm) * 64 words for lists of k items and wm wait entries a lane; level l: lanes
    // 0 .. (64 >> l) - 1 only, 2^l times the capacity
    __device__ void init(uint32_t* lds, uint32_t lane, int k, int wm, int level) {
        K = k << level; WM = wm << level; sh = 6 - level;
        cur = lds + lane; nxt = lds + k * 64 + lane; wait = lds + 2 * k * 64 + lane;
    }
    __device__ uint32_t get_cur(int k) const { return cur[k << sh]; }
    __device__ void set_cur(int k, uint32_t v) { cur[k << sh] = v; }
    __device__ uint32_t get_nxt(int k) const { return nxt[k << sh]; }
    __device__ void set_nxt(int k, uint32_t v) { nxt[k << sh] = v; }
    __device__ uint32_t wait_rule(int k) const { return wait[(2 * k) << sh]; }
    __device__ uint32_t wait_tgt(int k) const { return wait[(2 * k + 1) << sh]; }
    __device__ void set_wait(int k, uint32_t rule, uint32_t tgt) { wait[(2 * k) << sh] = rule; wait[(2 * k + 1) << sh] = tgt; }
    __device__ void swap() { uint32_t* t = cur; cur = nxt; nxt = t; }
    __device__ bool charge(int) { return true; }
    __device__ void reset() { ws_lo = 0; ws_hi = 0; }
    __device__ void set_wstart(int j, uint32_t v) {
        const int s8 = 8 * (j & 7);
        unsigned long long& w = j < 8 ? ws_lo : ws_hi;
        w = (w & ~(0xFFull << s8)) | ((unsigned long long)v << s8);
    }
    __device__ uint32_t get_wstart(int j) const {
        return (uint32_t)((j < 8 ? ws_lo >> (8 * j) : ws_hi >> (8 * (j - 8))) & 0xFF);
    }
};

__device__ __forceinline__ void push_overflow(const SlowScratch& S, uint32_t a, uint32_t b) {
    uint32_t idx = atomicAdd(S.count, 1u);
    if (idx < S.list_cap) { S.list[2 * idx] = a; S.list[2 * idx + 1] = b; }
    else atomicOr(S.count + 1, 1u);
}

__device__ __forceinline__ DevCtx position_ctx(const BuildPlan& P, uint32_t p) {
    const uint4 d = P.plane_ctx[p];
    DevCtx C;
    C.items = P.ctx_items + d.x;
    C.n_items = d.y;
    C.wait = P.ctx_wait;
    C.wait_off = P.ctx_wait_off + d.z;
    C.H = d.w;
    return C;
}

__device__ __forceinline__ void store_class(uint32_t* row, uint32_t W, uint32_t id, int res) {
    if (res & RES_ALIVE) atomicOr(row + (id >> 5), 1u << (id & 31));
    else if (res & RES_EARLY) atomicOr(row + W + (id >> 5), 1u << (id & 31));
}
__device__ __forceinline__ void store_class(const BuildPlan& P, uint32_t p, uint32_t W, uint32_t id, int res) {
    store_class(P.plane_ptr[p], W, id, res);
}
// The third row of a plane: the tokens that left the outermost rule early and then died, whatever the follow filter
// makes of them (with the filter off this is the uncertain row again).  It is what a plane of the same structure under
// another follow language is derived from (section 3.3: partial cache hit).
__device__ __forceinline__ void store_left_early(uint32_t* row, uint32_t W, uint32_t id) {
    atomicOr(row + 2 * W + (id >> 5), 1u << (id & 31));
}

// A persistent grid of single-wave workgroups: workgroup g handles chunks g, g + grid, g + 2 grid, ...
// (sorted ranks of one plane each; the host puts the long ones first), each in phases, so that the long
// divergent steps of the recogniser run on full waves instead of on the few lanes that need them.
// Phase 1 (when the plane's start set is a single item without rule edges, or one or two such items whose
// ends lead back into the outermost instance): every lane walks its token through the automaton, one table
// load per byte and thread.  A token that dies is rejected, one that reaches its end is accepted; one that
// reaches a state which predicts, or which completes a rule instance in a way the walk does not follow, goes
// on the deferred list.  One that dies after the outermost instance could have ended is what the plain run
// would call "left early": it goes straight to the follow-language run (or is stored as uncertain when that
// run is switched off).  Phase 2: the deferred tokens (for the other planes: all tokens of the chunk), 64 at
// a time, through the Earley recogniser.  Tokens that leave the outermost rule early and then die need the
// second, follow-language run; they are collected across chunks as (plane, rank) pairs and run 64 at a time too.
__device__ __forceinline__ void follow_batch(const DevTables& T, const DevVocab& Vd, const BuildPlan& P, const SlowScratch& S,
                                          const uint32_t* cls_words, uint32_t* lds, uint32_t* f_plane, uint32_t* f_rank,
                                          uint32_t first, uint32_t count, uint32_t lane) {
    // level 0: the batch, one token a lane; further levels: the tokens that outgrew the lists of the level before, half as
    // many at a time with twice the room (their entries have moved to the front of the batch's part of the queue, which
    // has been read)
    uint32_t cnt = count;
    for (int level = 0; level < BUILD_LEVELS && cnt; ++level) {
        const uint32_t lanes = 64u >> level;
        const bool last = level == BUILD_LEVELS - 1;
        uint32_t n_next = 0;
        for (uint32_t off = 0; off < cnt; off += lanes) {
            BuildStore st;
            st.init(lds, lane, (int)P.list_k, (int)P.list_wm, level);
            bool over = false;
            uint32_t p = 0, rank = 0;
            if (lane < lanes && off + lane < cnt) {
                p = f_plane[first + off + lane]; rank = f_rank[first + off + lane];
                const DevCtx C = position_ctx(P, p);
                const int n = (int)(Vd.off[rank + 1] - Vd.off[rank]);
                RegBytes tok;
                tok.v = Vd.tok16[rank];
                const int res = scan_token<BuildStore, true>(T, cls_words, C, tok, n, st);
                over = res & RES_OVERFLOW;
                if (over && last) push_overflow(S, p, rank);        // the large-capacity kernel takes it
                else if (res & RES_ALIVE) store_class(P, p, Vd.W, Vd.perm[rank], RES_EARLY);   // some context can take the rest: uncertain
            }
            if (!last) {
                const unsigned long long mo = __ballot(over);
                if (mo) {
                    __syncthreads();
                    if (over) {
                        const uint32_t at = first + n_next + (uint32_t)__popcll(mo & ((1ull << lane) - 1));
                        f_plane[at] = p; f_rank[at] = rank;
                    }
                    __syncthreads();
                    n_next += (uint32_t)__popcll(mo);
                }
            }
        }
        cnt = n_next;
    }
}

__global__ __launch_bounds__(64) XG2_BUILD_ATTR void k_build(DevTables T, DevVocab Vd, BuildPlan P, SlowScratch S) {
    extern __shared__ uint32_t lds[];                               // the item lists: (2 K + 2 WM) * 64 words, sized by the launch
    __shared__ uint32_t cls_words[64];                              // byte -> class, four a word
    const uint8_t* cls_bytes = reinterpret_cast<const uint8_t*>(cls_words);   // the same table, one byte an entry
    __shared__ uint8_t deferred[kBuildChunk];                       // tokens of the chunk for phase 2, as offsets from the chunk's first rank
    __shared__ uint32_t f_plane[128], f_rank[128];
    const uint32_t lane = threadIdx.x;
    cls_words[lane] = T.byte_class_words[lane];
    uint32_t n_follow = 0;                                          // same in every lane
    for (uint32_t chunk_idx = blockIdx.x; chunk_idx < P.n_chunks; chunk_idx += gridDim.x) {
        __syncthreads();                                            // one wave: orders the LDS traffic of the phases
        const uint4 chunk = P.chunk[2 * chunk_idx], chunk_b = P.chunk[2 * chunk_idx + 1];   // one 32-byte record: nothing else is loaded before the walk
        const uint32_t p = chunk.x;
        const uint32_t item0 = chunk_b.x;
        uint32_t* const row = reinterpret_cast<uint32_t*>(((uint64_t)chunk_b.w << 32) | chunk_b.z);
        // same for the whole chunk; that the start state itself can end its rule does not matter to a token (it has a byte)
        const bool walkable = chunk_b.y == 1 && (item0 & (F_BYTE | F_REF)) == F_BYTE;
        const bool root_instance = (item0 >> REF_BITS) == ROOT_ORIGIN;   // the start item is the plane's outermost rule instance
        const bool listed = chunk.w & kChunkListed;                 // ranks come from a list of long tokens
        const bool threaded = chunk.w & kChunkThreads;              // two thread descriptors follow the plane's items
        uint32_t n_work = chunk.z - chunk.y;
        // a token that left the outermost rule early and died: queued for the follow-language run, which starts
        // when 64 of them are there (`again` differs between lanes; everything else here is the same in all)
        auto queue_follow = [&](bool again, uint32_t rank) {
            const unsigned long long m = __ballot(again);
            if (!m) return;
            if (again) {
                const uint32_t at = n_follow + (uint32_t)__popcll(m & ((1ull << lane) - 1));
                f_plane[at] = p; f_rank[at] = rank;
            }
            n_follow += (uint32_t)__popcll(m);
            __syncthreads();
            if (n_follow >= 64) {
                n_follow -= 64;
                follow_batch(T, Vd, P, S, cls_words, lds, f_plane, f_rank, n_follow, 64, lane);
                __syncthreads();
            }
        };
        // what phase 1 does with such a token: the plain run would end dead with the early mark, so it is not made
        auto died_early = [&](bool yes, uint32_t rank) {
            if (yes) {
                const uint32_t id = Vd.perm[rank];
                store_left_early(row, Vd.W, id);
                if (!P.follow_filter) { store_class(row, Vd.W, id, RES_EARLY); yes = false; }
            }
            queue_follow(yes, rank);
        };
        if (chunk.w & kChunkDerive) {
            // partial cache hit: the plane's accepted row comes from a plane of the same structure built under another follow
            // language (copied by another kernel); of its tokens that left early and died -- mask words chunk.y .. chunk.z of
            // that plane's third row, one a lane -- those that this grammar's follow language can continue are uncertain here
            const uint32_t* base_left = reinterpret_cast<const uint32_t*>(((uint64_t)chunk_b.w << 32) | chunk_b.z);
            const uint32_t w = chunk.y + lane;
            uint32_t bits = w < chunk.z ? base_left[w] : 0u;
            while (__any(bits != 0)) {
                uint32_t rank = 0xFFFFFFFFu;
                if (bits) {
                    const uint32_t bit = (uint32_t)__ffs(bits) - 1;
                    bits &= bits - 1;
                    rank = Vd.rank[w * 32 + bit];
                }
                queue_follow(rank < Vd.n_sorted, rank);
            }
            continue;
        }
        if (walkable) {
            n_work = 0;
            for (uint32_t rank0 = chunk.y; rank0 < chunk.z; rank0 += 64) {
                uint32_t rank = rank0 + lane;
                int n = 0;
                uint4 tv = make_uint4(0, 0, 0, 0);
                if (rank < chunk.z) {
                    if (listed) rank = Vd.long_rank[rank];
                    n = (int)(Vd.off[rank + 1] - Vd.off[rank]); tv = Vd.tok16[rank];
                }
                bool defer = n > BuildStore::MAXLEN;                 // phase 2 hands it to the large-capacity kernel
                if (defer) n = 0;
                const WalkResult r = root_instance ? walk_tokens<true>(T.trans, T.n_classes, T.sink, cls_bytes, item0 & REF_MASK, tv, n)
                                                   : walk_tokens<false>(T.trans, T.n_classes, T.sink, cls_bytes, item0 & REF_MASK, tv, n);
                // a state that predicts, or that completes into a parent, is where the walk hands over to the recogniser
                defer |= n > 0 && (r.seen & (root_instance ? F_REF : (F_REF | F_FINAL))) != 0;
                const bool dead = r.state == T.sink;
                if (n > 0 && !dead && !defer) store_class(row, Vd.W, Vd.perm[rank], RES_ALIVE);      // reached its end alive
                // dead: rejected, unless the outermost rule could have ended on the way
                died_early(root_instance && n > 0 && dead && !defer && (r.seen_before_last & F_FINAL), rank);
                const unsigned long long m = __ballot(defer);
                if (defer) deferred[n_work + (uint32_t)__popcll(m & ((1ull << lane) - 1))] = (uint8_t)(rank0 + lane - chunk.y);
                n_work += (uint32_t)__popcll(m);
            }
            __syncthreads();
        } else if (threaded) {
            // Phase 1 for a start set of one or two scanning items that do not predict: each item is an automaton
            // thread; a thread of a waited-for instance that reaches a final state starts one thread of the outermost
            // instance at the state the host has looked up.  Three slots; anything else (a state that predicts, a
            // fourth thread) goes to phase 2.
            const uint4 pc = P.plane_ctx[p];
            const uint32_t* d = P.ctx_items + pc.x + pc.y;
            const uint32_t it_a = d[0], lead_a = d[1], it_b = d[2], lead_b = d[3];
            n_work = 0;
            for (uint32_t rank0 = chunk.y; rank0 < chunk.z; rank0 += 64) {
                uint32_t rank = rank0 + lane;
                bool defer = false;
                int n = 0;
                RegBytes tok;
                tok.v = make_uint4(0, 0, 0, 0);
                if (rank < chunk.z) {
                    if (listed) rank = Vd.long_rank[rank];
                    n = (int)(Vd.off[rank + 1] - Vd.off[rank]); tok.v = Vd.tok16[rank];
                }
                if (n > BuildStore::MAXLEN) { defer = true; n = 0; }
                uint32_t s0 = n > 0 ? it_a : kNoThread, s1 = n > 0 ? it_b : kNoThread, s2 = kNoThread;
                bool early = false;
                for (int i = 0; __any(i < n && !defer && (s0 & s1 & s2) != kNoThread); ++i) {
                    if (i < n && !defer && (s0 & s1 & s2) != kNoThread) {
                        const uint32_t cls = cls_bytes[tok.next()];
                        const bool more = i + 1 < n;
                        uint32_t start_a = kNoThread, start_b = kNoThread;
                        auto step = [&](uint32_t& s, uint32_t lead, uint32_t& start) {
                            if (s == kNoThread) return;
                            const uint32_t tgt = T.trans[(s & SID_MASK) * T.n_classes + cls];
                            if (tgt == T.sink) { s = kNoThread; return; }
                            if (tgt & F_REF) { defer = true; return; }
                            s = tgt | (s & ~REF_MASK);
                            if (tgt & F_FINAL) {
                                if ((s >> REF_BITS) == ROOT_ORIGIN) early |= more;
                                else start = lead;
                            }
                        };
                        uint32_t none = kNoThread;
                        step(s0, lead_a, start_a);
                        step(s1, lead_b, start_b);
                        step(s2, 0u, none);                          // only threads of the outermost instance get here
                        auto begin = [&](uint32_t item) {
                            if (item == kNoThread) return;
                            if (item & F_FINAL) early |= more;
                            if (item == s0 || item == s1 || item == s2) return;
                            if (s2 == kNoThread) s2 = item;
                            else if (s1 == kNoThread) s1 = item;
                            else if (s0 == kNoThread) s0 = item;
                            else defer = true;
                        };
                        begin(start_a);
                        begin(start_b);
                    }
                }
                bool dead_early = false;
                if (n > 0 && !defer) {
                    if ((s0 & s1 & s2) != kNoThread) store_class(row, Vd.W, Vd.perm[rank], RES_ALIVE);
                    else dead_early = early;
                }
                died_early(dead_early, rank);
                const unsigned long long m = __ballot(defer);
                if (defer) deferred[n_work + (uint32_t)__popcll(m & ((1ull << lane) - 1))] = (uint8_t)(rank0 + lane - chunk.y);
                n_work += (uint32_t)__popcll(m);
            }
            __syncthreads();
        }
        if (n_work == 0) continue;
        const DevCtx C = position_ctx(P, p);                        // only the recogniser needs the whole start set
        for (uint32_t base = 0; base < n_work; base += 64) {
            // level 0: 64 tokens of the list, one a lane; further levels: those of them that outgrew the item lists of the
            // level before, half as many at a time with twice the room (their offsets go through the part of the deferred
            // list that this batch has read)
            uint32_t cnt = min(64u, n_work - base);
            for (int level = 0; level < BUILD_LEVELS && cnt; ++level) {
                const uint32_t lanes = 64u >> level;
                const bool last = level == BUILD_LEVELS - 1;
                uint32_t n_next = 0;
                for (uint32_t off = 0; off < cnt; off += lanes) {
                    BuildStore st;
                    st.init(lds, lane, (int)P.list_k, (int)P.list_wm, level);
                    bool again = false, over = false;
                    uint32_t rank = 0, at = 0;                       // the token: sorted rank, and offset in the chunk
                    if (lane < lanes && off + lane < cnt) {
                        const uint32_t idx = base + off + lane;
                        at = (level > 0 || walkable || threaded) ? deferred[idx] : idx;
                        rank = listed ? Vd.long_rank[chunk.y + at] : chunk.y + at;
                        const int n = (int)(Vd.off[rank + 1] - Vd.off[rank]);
                        RegBytes tok;
                        tok.v = Vd.tok16[rank];
                        const int res = scan_token(T, cls_words, C, tok, n, st);
                        over = res & RES_OVERFLOW;
                        if (over && last) push_overflow(S, p, rank); // the large-capacity kernel takes it
                        else if (!over) {
                            // leaves the rule early and dies: it stays uncertain only if some context can take the rest of the token
                            const bool left_early = !(res & RES_ALIVE) && (res & RES_EARLY);
                            again = P.follow_filter && left_early;
                            if (left_early || !again) {
                                const uint32_t id = Vd.perm[rank];
                                if (left_early) store_left_early(row, Vd.W, id);
                                if (!again) store_class(row, Vd.W, id, res);
                            }
                        }
                    }
                    queue_follow(again, rank);
                    if (!last) {
                        const unsigned long long mo = __ballot(over);
                        if (mo) {
                            __syncthreads();
                            if (over) deferred[base + n_next + (uint32_t)__popcll(mo & ((1ull << lane) - 1))] = (uint8_t)at;
                            __syncthreads();
                            n_next += (uint32_t)__popcll(mo);
                        }
                    }
                }
                cnt = n_next;
            }
        }
    }
    __syncthreads();
    if (n_follow) follow_batch(T, Vd, P, S, cls_words, lds, f_plane, f_rank, 0, n_follow, lane);
}

// Both runs of one (plane, token) pair with the lists in `st`: the plain one and, if the token left the outermost
// rule early and died, the follow-language one.
template <class S>
__device__ int classify_slow(const DevTables& T, const DevVocab& Vd, const BuildPlan& P, const DevCtx& C, uint32_t off, int n, S& st) {
    st.reset();
    MemBytes tok{Vd.bytes + off};
    int res = scan_token<S, false, MemBytes>(T, T.byte_class_words, C, tok, n, st);
    if (!(res & (RES_ALIVE | RES_OVERFLOW)) && (res & RES_EARLY)) res |= RES_LEFT_EARLY;
    if (P.follow_filter && (res & RES_LEFT_EARLY)) {
        st.reset();
        int res2 = scan_token<S, true, MemBytes>(T, T.byte_class_words, C, tok, n, st);
        if (res2 & RES_OVERFLOW) res = RES_OVERFLOW;
        else if (!(res2 & RES_ALIVE)) res = RES_LEFT_EARLY;
    }
    return res;
}

__global__ __launch_bounds__(64) void k_build_slow(DevTables T, DevVocab Vd, BuildPlan P, SlowScratch S) {
    __shared__ uint32_t lds[MidStore::SLOTS * 64];
    const uint32_t gl = blockIdx.x * 64 + threadIdx.x;
    uint32_t count = S.count[0];
    if (count > S.list_cap) count = S.list_cap;
    MidStore mid;
    mid.init(lds + threadIdx.x);
    GlobalStore st;
    st.init(S.mem + gl, S.n_lanes, S.k_cap, S.wm_cap);
    for (uint32_t idx = gl; idx < count; idx += S.n_lanes) {
        if (*reinterpret_cast<volatile uint32_t*>(S.count + 1) & 2u) break;      // the build fails anyway: do not spend more on it
        const uint32_t p = S.list[2 * idx], rank = S.list[2 * idx + 1];
        const uint32_t off = Vd.off[rank];
        const int n = (int)(Vd.off[rank + 1] - off);
        DevCtx C = position_ctx(P, p);
        int res = S.k_cap >= (uint32_t)MidStore::K ? classify_slow(T, Vd, P, C, off, n, mid) : RES_OVERFLOW;   // (overflows at once if the token is too long for it)
        if (res & RES_OVERFLOW) res = classify_slow(T, Vd, P, C, off, n, st);
        if (res & RES_OVERFLOW) { atomicOr(S.count + 1, 2u); continue; }
        const uint32_t id = Vd.perm[rank];
        if (res & RES_LEFT_EARLY) store_left_early(P.plane_ptr[p], Vd.W, id);
        store_class(P, p, Vd.W, id, res);
    }
}

// Copies n 16-byte words from pinned host memory (read through its device address) to device memory: the per-call plan,
// tables and per-row records travel this way, without a trip through the copy engine.
__global__ __launch_bounds__(256) void k_upload(uint4* dst, const uint4* src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

__device__ __forceinline__ void expand_range(const uint4* range_a, const uint4* range_b, const uint32_t* first, uint32_t r, uint4* chunk) {
    const uint4 a = range_a[r], b = range_b[r];
    const uint32_t step = (a.w & kChunkDerive) ? kDeriveChunk : (a.w & kChunkHeavy) ? kHeavyChunk : kBuildChunk;
    uint4* out = chunk + 2 * (size_t)first[r];
    for (uint32_t lo = a.y; lo < a.z; lo += step, out += 2) {
        out[0] = make_uint4(a.x, lo, min(a.z, lo + step), a.w);
        out[1] = b;
    }
}

__global__ __launch_bounds__(256) void k_expand_chunks(const uint4* range_a, const uint4* range_b, const uint32_t* first, uint32_t n_ranges, uint4* chunk) {
    const uint32_t r = blockIdx.x * 256 + threadIdx.x;
    if (r < n_ranges) expand_range(range_a, range_b, first, r, chunk);
}

// Everything a build needs before its first kernel, in one launch of three independent parts: workgroups [0, nb_up) copy
// the plan (and tables) from pinned host memory, the next nb_zero clear the rows that the pool hands out for the first
// time, the rest write the chunk records, reading their ranges from the pinned host copy (not from the device copy that
// the first part is still writing).
__global__ __launch_bounds__(256) void k_stage(uint4* dst, const uint4* src, size_t n_up, uint32_t nb_up, StageZero Z, uint32_t nb_zero,
                                               const uint4* range_a, const uint4* range_b, const uint32_t* first, uint32_t n_ranges, uint4* chunk) {
    if (blockIdx.x < nb_up) {
        for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_up; i += (size_t)nb_up * 256) dst[i] = src[i];
    } else if (blockIdx.x < nb_up + nb_zero) {
        const size_t t = (size_t)(blockIdx.x - nb_up) * 256 + threadIdx.x, stride = (size_t)nb_zero * 256;
        for (uint32_t k = 0; k < Z.n; ++k) {
            uint32_t* p = Z.p[k];
            const size_t words = Z.words[k];
            if ((reinterpret_cast<uintptr_t>(p) & 15) == 0) {
                uint4* p4 = reinterpret_cast<uint4*>(p);
                for (size_t i = t; i < words / 4; i += stride) p4[i] = make_uint4(0, 0, 0, 0);
                for (size_t i = (words & ~(size_t)3) + t; i < words; i += stride) p[i] = 0u;
            } else {
                for (size_t i = t; i < words; i += stride) p[i] = 0u;
            }
        }
    } else {
        const uint32_t r = (blockIdx.x - nb_up - nb_zero) * 256 + threadIdx.x;
        if (r < n_ranges) expand_range(range_a, range_b, first, r, chunk);
    }
}

__global__ __launch_bounds__(256) void k_copy_masked(const CopyJob* jobs, uint32_t W) {
    const CopyJob j = jobs[blockIdx.y];
    const uint32_t w = blockIdx.x * 256 + threadIdx.x;
    if (w >= W) return;
    const uint32_t m = j.mask[w];
    if (!m) return;
    j.dst[w] |= j.src[w] & m;
    j.dst[W + w] |= j.src[W + w] & m;
    j.dst[2 * W + w] |= j.src[2 * W + w] & m;
}

__global__ __launch_bounds__(256) void k_copy_first_byte(const FirstByteCopyJob* jobs, const uint8_t* first_byte, uint32_t W) {
    __shared__ uint32_t bytes[8];
    const FirstByteCopyJob* j = jobs + blockIdx.y;
    if (threadIdx.x < 8) bytes[threadIdx.x] = j->bytes[threadIdx.x];
    __syncthreads();
    const uint32_t w = blockIdx.x * 256 + threadIdx.x;
    if (w >= W) return;
    const uint32_t* src = j->src;
    uint32_t* dst = j->dst;
    const uint32_t a = src[w], u = src[W + w], e = src[2 * W + w];
    uint32_t todo = a | u | e, m = 0;                               // only the tokens the source has a bit for matter
    while (todo) {
        const uint32_t bit = __ffs(todo) - 1;
        todo &= todo - 1;
        const uint32_t b = first_byte[w * 32 + bit];
        m |= ((bytes[b >> 5] >> (b & 31)) & 1u) << bit;
    }
    if (a & m) dst[w] |= a & m;
    if (u & m) dst[W + w] |= u & m;
    if (e & m) dst[2 * W + w] |= e & m;
}

// Partial cache hit: the accepted row and the left-early row of a plane are those of the plane it is derived from.
__global__ __launch_bounds__(256) void k_copy_structure(const CopyJob* jobs, uint32_t W) {
    const CopyJob j = jobs[blockIdx.y];
    const uint32_t w = blockIdx.x * 256 + threadIdx.x;
    if (w >= W) return;
    j.dst[w] = j.src[w];
    j.dst[2 * W + w] = j.src[2 * W + w];
}

// Per plane: set bits of the accepted and of the uncertain row, and the plane's list of uncertain tokens behind its
// three rows: word 0 = how many (the list holds them if that is at most kUncListWords - 1), then their token ids in no
// particular order.
__global__ __launch_bounds__(256) void k_plane_summary(uint32_t* const* plane_ptr, uint32_t n_pos, uint32_t W, uint32_t* counts) {
    __shared__ uint32_t part[2][4];
    __shared__ uint32_t n_list;
    const uint32_t p = blockIdx.x;
    if (p >= n_pos) return;
    uint32_t* row = plane_ptr[p];
    uint32_t* list = row + 3 * (size_t)W;
    if (threadIdx.x == 0) n_list = 0;
    __syncthreads();
    uint32_t a = 0, u = 0;
    for (uint32_t w = threadIdx.x; w < W; w += blockDim.x) {
        const uint32_t aw = row[w], uw = row[W + w];
        a += __popc(aw); u += __popc(uw);
        uint32_t c = uw & ~aw;
        if (c) {
            uint32_t at = atomicAdd(&n_list, (uint32_t)__popc(c));
            for (; c; c &= c - 1, ++at)
                if (at < kUncListWords - 1) list[1 + at] = w * 32 + (uint32_t)__ffs(c) - 1;
        }
    }
    for (int s = 32; s > 0; s >>= 1) { a += __shfl_down(a, s); u += __shfl_down(u, s); }
    if ((threadIdx.x & 63) == 0) { part[0][threadIdx.x >> 6] = a; part[1][threadIdx.x >> 6] = u; }
    __syncthreads();
    if (threadIdx.x == 0) {
        counts[2 * p] = part[0][0] + part[0][1] + part[0][2] + part[0][3];
        counts[2 * p + 1] = part[1][0] + part[1][1] + part[1][2] + part[1][3];
        list[0] = n_list;
    }
}

// The copies of the derived planes and the summary in one pass: a plane's words are read once, completed from the
// planes it takes bits from, written back where they changed, and counted and listed from the registers.  A workgroup
// takes FINISH_WORDS words of one plane; the plane's counts and the length of its list are summed with one device atomic
// per workgroup each (they start at zero: the counts arrive as zeros with the plan, the list with the cleared row).
constexpr uint32_t FINISH_ITER = 4, FINISH_WORDS = 256 * FINISH_ITER;
__global__ __launch_bounds__(256) void k_finish_planes(uint32_t* const* plane_ptr, const FinishJob* jobs, uint32_t n_pos, const uint8_t* first_byte,
                                                       uint32_t W, uint32_t* counts) {
    __shared__ uint32_t part[2][4];
    __shared__ uint32_t n_list, list_base;
    __shared__ uint32_t bytes[8];
    const uint32_t p = blockIdx.y;
    uint32_t* row = plane_ptr[p];
    uint32_t* list = row + 3 * (size_t)W;
    const FinishJob* job = jobs + p;
    const uint32_t* m_src = job->m_src;
    const uint32_t* m_mask = job->m_mask;
    const uint32_t* f_src = job->f_src;
    if (threadIdx.x == 0) n_list = 0;
    if (threadIdx.x < 8) bytes[threadIdx.x] = job->f_bytes[threadIdx.x];
    __syncthreads();
    uint32_t na = 0, nu = 0, cand[FINISH_ITER], at[FINISH_ITER];
#pragma unroll
    for (uint32_t it = 0; it < FINISH_ITER; ++it) {
        const uint32_t w = blockIdx.x * FINISH_WORDS + it * 256 + threadIdx.x;
        cand[it] = 0; at[it] = 0;
        if (w >= W) continue;
        const uint32_t a0 = row[w], u0 = row[W + w];
        uint32_t a = a0, u = u0, e = 0;                             // e: bits to add to the third row (it is not read for a plane that takes none)
        if (m_src) {
            const uint32_t m = m_mask[w];
            if (m) { a |= m_src[w] & m; u |= m_src[W + w] & m; e |= m_src[2 * W + w] & m; }
        }
        if (f_src) {
            const uint32_t sa = f_src[w], su = f_src[W + w], se = f_src[2 * W + w];
            uint32_t todo = sa | su | se, m = 0;                    // only the tokens the source has a bit for matter
            while (todo) {
                const uint32_t bit = __ffs(todo) - 1;
                todo &= todo - 1;
                const uint32_t b = first_byte[w * 32 + bit];
                m |= ((bytes[b >> 5] >> (b & 31)) & 1u) << bit;
            }
            a |= sa & m; u |= su & m; e |= se & m;
        }
        if (a != a0) row[w] = a;
        if (u != u0) row[W + w] = u;
        if (e) { const uint32_t e0 = row[2 * W + w]; if (e & ~e0) row[2 * W + w] = e0 | e; }
        na += __popc(a); nu += __popc(u);
        cand[it] = u & ~a;
        if (cand[it]) at[it] = atomicAdd(&n_list, (uint32_t)__popc(cand[it]));
    }
    for (int s = 32; s > 0; s >>= 1) { na += __shfl_down(na, s); nu += __shfl_down(nu, s); }
    if ((threadIdx.x & 63) == 0) { part[0][threadIdx.x >> 6] = na; part[1][threadIdx.x >> 6] = nu; }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t ta = part[0][0] + part[0][1] + part[0][2] + part[0][3], tu = part[1][0] + part[1][1] + part[1][2] + part[1][3];
        if (ta) atomicAdd(counts + 2 * p, ta);
        if (tu) atomicAdd(counts + 2 * p + 1, tu);
        list_base = n_list ? atomicAdd(list, n_list) : 0u;           // word 0 of the list: how many uncertain tokens the plane has
    }
    __syncthreads();
    if (n_list == 0) return;
#pragma unroll
    for (uint32_t it = 0; it < FINISH_ITER; ++it) {
        const uint32_t w = blockIdx.x * FINISH_WORDS + it * 256 + threadIdx.x;
        uint32_t k = list_base + at[it];
        for (uint32_t c = cand[it]; c; c &= c - 1, ++k)
            if (k < kUncListWords - 1) list[1 + k] = w * 32 + (uint32_t)__ffs(c) - 1;
    }
}

// ---- fill ------------------------------------------------------------------------------------------
// k_fill: one workgroup per row, in two teams of wavefronts that work side by side.
//   The union team streams: per mask word the OR of the accepted rows of the row's frontier planes, plus the
//   end-of-sequence bit, stored with 16-byte accesses.
//   The re-check team takes the uncertain tokens of the frontier planes from the short list every plane carries behind
//   its three rows (written by k_plane_summary), one token per lane, and runs the Earley routine from the row's full
//   context; what survives is kept in LDS until the union is stored, and OR-ed in afterwards.
// The two teams need nothing from each other until that point, so the latency of the re-check (a chain of dependent
// table loads) hides behind the streaming and the other way round.  A token that another frontier plane accepts is in
// the mask anyway and is not parsed: its lane looks the bit up in the accepted rows itself and does not wait for the union.
// A row with a frontier plane whose uncertain tokens do not fit its list (or with more candidates than the LDS list
// holds) takes the sequential way: the union team also reads the uncertain rows and lists the words with candidates,
// the re-check team starts when the union is done.
// Four wavefronts stream, two re-check with half of their lanes at work (measured: fewer lanes per wavefront, more
// wavefronts or another split of the six gain nothing; a larger workgroup lowers the number of rows a compute unit holds).
constexpr int FILL_OR_WAVES = 4, FILL_RECHECK_WAVES = 2;
constexpr int FILL_RECHECK_LANES = 32;                               // lanes at work in a wavefront of the re-check team
constexpr int FILL_COLS = FILL_RECHECK_WAVES * FILL_RECHECK_LANES;  // tokens the team parses at a time
constexpr int FILL_OR_THREADS = 64 * FILL_OR_WAVES;
constexpr int FILL_THREADS = 64 * (FILL_OR_WAVES + FILL_RECHECK_WAVES);
constexpr int FILL_BLOCK = 5;                          // steps of the union whose loads are issued together
constexpr int FILL_K = 8, FILL_WM = 12;
constexpr uint32_t FILL_SPARSE_CAP = 512;              // candidates of a row that the side-by-side way handles
constexpr uint32_t FILL_NONE = 0xFFFFFFFFu;
using FillStore = LdsStore<FILL_K, FILL_WM, FILL_COLS>;

__device__ __forceinline__ DevCtx row_ctx(const FillBatch& F, const FillRow& r) {
    DevCtx C;
    C.items = F.ctx_items + r.item_off;
    C.n_items = r.item_n;
    C.wait = F.ctx_wait + r.wait_base;
    C.wait_off = F.ctx_wait_off + r.waitoff_off;
    C.H = r.H;
    return C;
}

// Candidate bits of one mask word of row b go to the scratch word; the word's index goes to the row's own
// work list (one LDS atomic per wave with candidates: no atomics on device memory).
__device__ __forceinline__ void list_candidates(const FillBatch& F, uint32_t* n_listed, uint32_t* n_cand, uint32_t cand, uint32_t row_base, uint32_t w) {
    const unsigned long long has = __ballot(cand != 0);
    if (has) {
        const uint32_t lane = threadIdx.x & 63;
        const uint32_t leader = (uint32_t)__ffsll((long long)has) - 1;
        uint32_t base = 0;
        if (lane == leader) base = atomicAdd(n_listed, (uint32_t)__popcll(has));
        base = __shfl(base, (int)leader);
        if (cand) {
            atomicAdd(n_cand, (uint32_t)__popc(cand));
            F.cand_words[row_base + w] = cand;
            F.work_list[row_base + base + (uint32_t)__popcll(has & ((1ull << lane) - 1))] = w;
        }
    }
}

// One candidate token of row b against the row's full context.  A token the short lists cannot decide goes to the
// large-capacity list and counts as rejected here.
__device__ __forceinline__ bool recheck_token(const DevVocab& Vd, const SlowScratch& S, const DevTables& T, const uint32_t* cls_words, const DevCtx& C,
                                              uint32_t b, uint32_t id, FillStore& st) {
    const uint32_t rank = Vd.rank[id];
    if (rank >= Vd.n_sorted) return false;
    const int n = (int)(Vd.off[rank + 1] - Vd.off[rank]);
    RegBytes tok;
    tok.v = Vd.tok16[rank];
    st.reset();
    const int res = scan_token(T, cls_words, C, tok, n, st);
    if (res & RES_OVERFLOW) { push_overflow(S, b, id); return false; }
    return (res & RES_ALIVE) != 0;
}

// Entry with the smallest index whose inclusive prefix sum exceeds t (every lane of the wave calls this; incl is the
// lanes' non-decreasing prefix, lane 63 holds the total).
__device__ __forceinline__ uint32_t prefix_owner(uint32_t incl, uint32_t t) {
    uint32_t lo = 0, hi = 63;
#pragma unroll
    for (int it = 0; it < 6; ++it) {
        const uint32_t mid = (lo + hi) >> 1;
        const uint32_t v = (uint32_t)__shfl((int)incl, (int)mid);
        if (v > t) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// A thread of the union team handles WORDS consecutive mask words per step (4: 16-byte loads and stores, needs
// W % 4 == 0 and a 16-byte aligned bitmask row; 1: any layout).
template <int WORDS>
__global__ __launch_bounds__(FILL_THREADS) void k_fill(FillBatch F, DevVocab Vd, int32_t* bitmask, long long row_stride, SlowScratch S) {
    __shared__ uint32_t lds_store[FillStore::SLOTS * FILL_COLS];
    __shared__ uint32_t sh_surv[FILL_SPARSE_CAP];
    __shared__ uint32_t sh_cls[FILL_RECHECK_WAVES][64];               // byte classes of the row's grammar, a copy per wavefront of the re-check team
    __shared__ uint32_t n_listed, n_cand;
    const uint32_t b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const FillRow r = F.rows[b];
    const uint32_t front_off = r.front_off, front_n = r.front_n, flags = r.flags;
    const bool live = !(flags & 2u);
    if (threadIdx.x == 0) { n_listed = 0; n_cand = 0; }
    // the plan, worked out by every wavefront for itself: lane k looks at frontier plane k
    uint64_t addr = 1;
    uint32_t n_unc = 0;
    if (live && front_n <= 64 && lane < front_n) {
        addr = F.front_planes[front_off + lane];
        if (!(addr & 1)) n_unc = tab(reinterpret_cast<const uint32_t*>(addr) + 3 * (size_t)Vd.W);
    }
    const bool no_list = n_unc > kUncListWords - 1;                   // more uncertain tokens than the plane's list holds
    uint32_t incl = no_list ? 0u : n_unc;
    for (int d = 1; d < 64; d <<= 1) { const uint32_t up = (uint32_t)__shfl_up((int)incl, d); if ((int)lane >= d) incl += up; }
    const uint32_t total = (uint32_t)__shfl((int)incl, 63);
    const bool listed_way = live && front_n != 0 && (front_n > 64 || __any(no_list) || total > FILL_SPARSE_CAP);
    uint32_t* out = reinterpret_cast<uint32_t*>(bitmask) + (long long)b * row_stride;
    FillStore st;
    const uint32_t col = (wave - FILL_OR_WAVES) * FILL_RECHECK_LANES + lane;      // re-check team: this lane's place among the lanes at work
    const bool at_work = wave >= FILL_OR_WAVES && lane < FILL_RECHECK_LANES;
    if (at_work) st.init(lds_store + col);
    __syncthreads();

    if (wave < FILL_OR_WAVES) {
        const uint32_t eos_word = F.eos_id >> 5, eos_bit = 1u << (F.eos_id & 31);
        const uint32_t n_steps = (Vd.W / WORDS + FILL_OR_THREADS - 1) / FILL_OR_THREADS;   // same for every thread: the ballots see whole waves
        // FILL_BLOCK steps at a time: first every load of the block (plane after plane, so that a thread has several
        // independent loads in flight), then the candidates and the stores
        for (uint32_t step0 = 0; step0 < n_steps; step0 += FILL_BLOCK) {
            uint32_t acc[FILL_BLOCK][WORDS], unc[FILL_BLOCK][WORDS];
#pragma unroll
            for (int s = 0; s < FILL_BLOCK; ++s)
#pragma unroll
                for (int c = 0; c < WORDS; ++c) { acc[s][c] = 0; unc[s][c] = 0; }
            if (live)
                for (uint32_t k = 0; k < front_n; ++k) {
                    const uint64_t pa = F.front_planes[front_off + k];
                    const uint32_t* row = reinterpret_cast<const uint32_t*>(pa & ~(uint64_t)1);
                    const bool with_unc = listed_way && !(pa & 1);
#pragma unroll
                    for (int s = 0; s < FILL_BLOCK; ++s) {
                        const uint32_t v = (step0 + s) * FILL_OR_THREADS + threadIdx.x;
                        if (v >= Vd.W / WORDS) continue;
                        if (WORDS == 4) {
                            const uint4 a = tab(reinterpret_cast<const uint4*>(row) + v);
                            acc[s][0] |= a.x; acc[s][1 % WORDS] |= a.y; acc[s][2 % WORDS] |= a.z; acc[s][3 % WORDS] |= a.w;
                            if (with_unc) {
                                const uint4 u = tab(reinterpret_cast<const uint4*>(row + Vd.W) + v);
                                unc[s][0] |= u.x; unc[s][1 % WORDS] |= u.y; unc[s][2 % WORDS] |= u.z; unc[s][3 % WORDS] |= u.w;
                            }
                        } else {
                            acc[s][0] |= tab(row + v);
                            if (with_unc) unc[s][0] |= tab(row + Vd.W + v);
                        }
                    }
                }
#pragma unroll
            for (int s = 0; s < FILL_BLOCK; ++s) {
                if (step0 + s >= n_steps) break;                        // same for every thread
                const uint32_t v = (step0 + s) * FILL_OR_THREADS + threadIdx.x;
                const bool in_row = v < Vd.W / WORDS;
                uint32_t cand[WORDS], any = 0;
#pragma unroll
                for (int c = 0; c < WORDS; ++c) {
                    cand[c] = in_row ? (unc[s][c] & ~acc[s][c]) : 0u;
                    any |= cand[c];
                    if ((flags & 3u) && eos_word == v * WORDS + c) acc[s][c] |= eos_bit;
                }
                if (listed_way && __any(any != 0)) {                    // candidates are few: most wavefronts have none
#pragma unroll
                    for (int c = 0; c < WORDS; ++c) list_candidates(F, &n_listed, &n_cand, cand[c], b * Vd.W, v * WORDS + c);
                }
                if (in_row) {
                    if (WORDS == 4) reinterpret_cast<uint4*>(out)[v] = make_uint4(acc[s][0], acc[s][1 % WORDS], acc[s][2 % WORDS], acc[s][3 % WORDS]);
                    else out[v] = acc[s][0];
                }
            }
        }
    } else if (!listed_way && total != 0) {
        // side by side with the union: candidate t is entry t - (tokens of the planes before) of its plane's list
        const DevTables T = F.tables[r.tables_idx];
        const DevCtx C = row_ctx(F, r);
        sh_cls[wave - FILL_OR_WAVES][lane] = T.byte_class_words[lane];
        __builtin_amdgcn_wave_barrier();                              // one wave: its LDS operations complete in order
        for (uint32_t t0 = 0; t0 < total; t0 += FILL_COLS) {
            const uint32_t t = t0 + col;
            const bool mine = at_work && t < total;
            const uint32_t k = prefix_owner(incl, t);
            const uint32_t end_k = (uint32_t)__shfl((int)incl, (int)k), n_k = (uint32_t)__shfl((int)n_unc, (int)k);
            const uint32_t a_lo = (uint32_t)__shfl((int)(uint32_t)addr, (int)k), a_hi = (uint32_t)__shfl((int)(uint32_t)(addr >> 32), (int)k);
            uint32_t id = 0;
            if (mine) id = tab(reinterpret_cast<const uint32_t*>(((uint64_t)a_hi << 32) | a_lo) + 3 * (size_t)Vd.W + 1 + (t - (end_k - n_k)));
            // a token that a frontier plane accepts is in the mask already: no need to parse it
            uint32_t accepted = 0;
            for (uint32_t k2 = 0; k2 < front_n; ++k2) {
                const uint32_t p_lo = (uint32_t)__shfl((int)(uint32_t)addr, (int)k2), p_hi = (uint32_t)__shfl((int)(uint32_t)(addr >> 32), (int)k2);
                accepted |= tab(reinterpret_cast<const uint32_t*>((((uint64_t)p_hi << 32) | p_lo) & ~(uint64_t)1) + (id >> 5)) >> (id & 31);
            }
            if (mine) sh_surv[t] = !(accepted & 1u) && recheck_token(Vd, S, T, sh_cls[wave - FILL_OR_WAVES], C, b, id, st) ? id : FILL_NONE;
        }
    }
    __syncthreads();

    if (!listed_way) {
        for (uint32_t t = threadIdx.x; t < total; t += FILL_THREADS) {
            const uint32_t id = sh_surv[t];
            if (id != FILL_NONE) atomicOr(out + (id >> 5), 1u << (id & 31));
        }
        if (threadIdx.x == 0) F.row_count[b] = total;                   // every row writes its count: nothing to clear beforehand
        return;
    }
    if (threadIdx.x == 0) F.row_count[b] = n_cand;
    if (wave < FILL_OR_WAVES) return;
    // the sequential way: each wave of the re-check team takes as many listed words at a time as it has lanes at work
    // and spreads their set bits densely over those lanes
    const uint32_t count = n_listed;
    const uint32_t* wlist = F.work_list + b * Vd.W;
    const uint32_t* cands = F.cand_words + b * Vd.W;
    const DevTables T = F.tables[r.tables_idx];
    const DevCtx C = row_ctx(F, r);
    sh_cls[wave - FILL_OR_WAVES][lane] = T.byte_class_words[lane];
    __builtin_amdgcn_wave_barrier();
    for (uint32_t base = (wave - FILL_OR_WAVES) * FILL_RECHECK_LANES; base < count; base += FILL_COLS) {
        uint32_t idx = 0, cand = 0;
        if (lane < FILL_RECHECK_LANES && base + lane < count) { idx = wlist[base + lane]; cand = cands[idx]; }
        uint32_t pre = (uint32_t)__popc(cand);
        for (int d = 1; d < 64; d <<= 1) { const uint32_t up = (uint32_t)__shfl_up((int)pre, d); if ((int)lane >= d) pre += up; }
        const uint32_t n_tok = (uint32_t)__shfl((int)pre, 63);
        for (uint32_t t0 = 0; t0 < n_tok; t0 += FILL_RECHECK_LANES) {
            const uint32_t my = t0 + lane;
            const uint32_t j = prefix_owner(pre, my);
            uint32_t c = (uint32_t)__shfl((int)cand, (int)j);
            const uint32_t end_j = (uint32_t)__shfl((int)pre, (int)j), w = (uint32_t)__shfl((int)idx, (int)j);
            if (lane < FILL_RECHECK_LANES && my < n_tok) {
                uint32_t skip = my - (end_j - (uint32_t)__popc(c));
                while (skip--) c &= c - 1;                             // drop the lowest set bits that other lanes take
                const uint32_t bit = __ffs(c) - 1;
                if (recheck_token(Vd, S, T, sh_cls[wave - FILL_OR_WAVES], C, b, w * 32 + bit, st)) atomicOr(out + w, 1u << bit);
            }
        }
    }
}

__global__ __launch_bounds__(64) void k_recheck_slow(FillBatch F, DevVocab Vd, int32_t* bitmask, long long row_stride, SlowScratch S) {
    __shared__ uint32_t lds[MidStore::SLOTS * 64];
    const uint32_t gl = blockIdx.x * 64 + threadIdx.x;
    if (F.zero_words && gl < 4) F.zero_words[gl] = 0;                   // the words the next call counts in
    uint32_t count = S.count[0];
    if (count > S.list_cap) count = S.list_cap;
    MidStore mid;
    mid.init(lds + threadIdx.x);
    GlobalStore st;
    st.init(S.mem + gl, S.n_lanes, S.k_cap, S.wm_cap);
    for (uint32_t idx = gl; idx < count; idx += S.n_lanes) {
        const uint32_t b = S.list[2 * idx], id = S.list[2 * idx + 1];
        const FillRow r = F.rows[b];
        const uint32_t rank = Vd.rank[id];
        if (rank >= Vd.n_sorted) continue;
        const uint32_t off = Vd.off[rank];
        const int n = (int)(Vd.off[rank + 1] - off);
        const DevTables T = F.tables[r.tables_idx];
        MemBytes tok{Vd.bytes + off};
        mid.reset();
        int res = S.k_cap >= (uint32_t)MidStore::K ? scan_token<MidStore, false, MemBytes>(T, T.byte_class_words, row_ctx(F, r), tok, n, mid) : RES_OVERFLOW;
        if (res & RES_OVERFLOW) {
            st.reset();
            res = scan_token<GlobalStore, false, MemBytes>(T, T.byte_class_words, row_ctx(F, r), tok, n, st);
        }
        if (res & RES_OVERFLOW) {
            // undecided: the bit stays 0, and the call must not pass for complete.  The pair goes to the host's list (it
            // can decide it with its own parser), a slot on the device is marked unusable.
            atomicOr(S.count + 1, 2u);
            if (S.mark_rows) S.mark_rows[b].pad[1] = 2u;
            if (S.unresolved) {                                      // plain stores only: the list is host memory
                const uint32_t at = atomicAdd(S.count + 2, 1u);
                S.unresolved[0] = 1u;
                if (at < S.unresolved_cap) { S.unresolved[2 + 2 * at] = b; S.unresolved[3 + 2 * at] = id; }
                else S.unresolved[1] = 1u;
            }
            continue;
        }
        if (res & RES_ALIVE) atomicOr(reinterpret_cast<uint32_t*>(bitmask) + (long long)b * row_stride + (id >> 5), 1u << (id & 31));
    }
}

// ---- matchers on the device ------------------------------------------------------------------------
// k_accept: one wavefront per matcher slot.  The lanes bring the slot's context into LDS, lane 0 takes the sampled token
// through the recogniser and writes the slot's next context and frontier planes (accept_core.hpp) into an LDS staging
// area, with its item lists, the renumbering table and the frontier staging in LDS too, and the lanes copy the result
// out.  A token or context too large for that runs again with everything in device memory.  A slot whose capacity is
// exceeded gets a sticky error and answers XG2_EOVERFLOW until it is reset.
constexpr int ACCEPT_K = 64, ACCEPT_WM = 256, ACCEPT_MAXLEN = 48;  // lane 0's item lists
struct OneLaneStore {
    static constexpr int K = ACCEPT_K, WM = ACCEPT_WM, MAXLEN = ACCEPT_MAXLEN, WORDS = 2 * ACCEPT_K + 2 * ACCEPT_WM + ACCEPT_MAXLEN + 1;
    uint32_t* cur; uint32_t* nxt; uint32_t* wait; uint32_t* ws;
    __device__ void init(uint32_t* base) { cur = base; nxt = base + K; wait = base + 2 * K; ws = base + 2 * K + 2 * WM; }
    __device__ uint32_t get_cur(int k) const { return cur[k]; }
    __device__ void set_cur(int k, uint32_t v) { cur[k] = v; }
    __device__ uint32_t get_nxt(int k) const { return nxt[k]; }
    __device__ void set_nxt(int k, uint32_t v) { nxt[k] = v; }
    __device__ uint32_t wait_rule(int k) const { return wait[2 * k]; }
    __device__ uint32_t wait_tgt(int k) const { return wait[2 * k + 1]; }
    __device__ void set_wait(int k, uint32_t rule, uint32_t tgt) { wait[2 * k] = rule; wait[2 * k + 1] = tgt; }
    __device__ void swap() { uint32_t* t = cur; cur = nxt; nxt = t; }
    __device__ bool charge(int) { return true; }
    __device__ void reset() {}
    __device__ void set_wstart(int j, uint32_t v) { ws[j] = v; }
    __device__ uint32_t get_wstart(int j) const { return ws[j]; }
};
template <int N_MAP, int N_FRONT>
struct OneLaneScratchX {
    uint8_t* map; uint64_t* front;
    __device__ uint32_t map_cap() const { return N_MAP; }
    __device__ uint32_t front_cap() const { return N_FRONT; }
    __device__ uint32_t map_get(uint32_t i) const { return map[i]; }
    __device__ void map_set(uint32_t i, uint32_t v) { map[i] = (uint8_t)v; }
    __device__ uint64_t front_get(uint32_t k) const { return front[k]; }
    __device__ void front_set(uint32_t k, uint64_t v) { front[k] = v; }
};
struct GlobalScratchX {
    uint8_t* map; uint64_t* front; size_t stride; uint32_t n_map, n_front;
    __device__ uint32_t map_cap() const { return n_map; }
    __device__ uint32_t front_cap() const { return n_front; }
    __device__ uint32_t map_get(uint32_t i) const { return map[(size_t)i * stride]; }
    __device__ void map_set(uint32_t i, uint32_t v) { map[(size_t)i * stride] = (uint8_t)v; }
    __device__ uint64_t front_get(uint32_t k) const { return front[(size_t)k * stride]; }
    __device__ void front_set(uint32_t k, uint64_t v) { front[(size_t)k * stride] = v; }
};

__device__ __forceinline__ void start_sequence(const BatchDev& D, uint32_t b, uint32_t cache_idx, uint32_t lane, uint32_t n_lanes) {
    const CacheDev& Cd = D.caches[cache_idx];
    FillRow r{};
    r.front_off = b * D.KF; r.front_n = Cd.start_n_front;
    r.item_off = b * D.KI; r.item_n = Cd.start_n_items;
    r.wait_base = b * D.KW; r.waitoff_off = b * (D.KH + 1); r.H = Cd.start_H;
    r.tables_idx = cache_idx; r.flags = Cd.start_flags;
    r.pad[0] = 0; r.pad[1] = 0; r.pad[2] = 0;
    for (uint32_t k = lane; k < Cd.start_n_front; k += n_lanes) D.front[r.front_off + k] = Cd.start_front[k];
    for (uint32_t k = lane; k < Cd.start_n_items; k += n_lanes) D.items[r.item_off + k] = Cd.start_items[k];
    for (uint32_t k = lane; k <= Cd.start_H; k += n_lanes) D.wait_off[r.waitoff_off + k] = Cd.start_wait_off[k];
    const uint32_t n_wait = Cd.start_wait_off[Cd.start_H];
    for (uint32_t k = lane; k < n_wait; k += n_lanes) D.wait[r.wait_base + k] = Cd.start_wait[k];
    if (lane == 0) D.rows[b] = r;
}

__global__ __launch_bounds__(256) void k_batch_assign(BatchDev D, const int32_t* rows, uint32_t n, uint32_t cache_idx) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t b = rows ? (uint32_t)rows[i] : i;
    if (b < D.B) start_sequence(D, b, cache_idx, 0, 1);
}

constexpr uint32_t ACC_KI = kSlotItems, ACC_KH = kSlotSets, ACC_KW = kSlotWaits, ACC_KF = kSlotPlanes;     // the slot capacities the LDS staging is laid out for
__global__ __launch_bounds__(64) void k_accept(BatchDev D, DevVocab Vd, uint32_t eos_id, const int32_t* token_ids, int32_t* status) {
    __shared__ uint32_t in_items[ACC_KI], in_wait_off[ACC_KH + 1], out_items[ACC_KI], out_wait_off[ACC_KH + 1];
    __shared__ uint2 in_wait[ACC_KW], out_wait[ACC_KW];
    __shared__ uint64_t out_front[ACC_KF], x_front[ACC_KF];
    __shared__ uint32_t lists[OneLaneStore::WORDS];
    __shared__ uint8_t x_map[ACC_KH + ACCEPT_MAXLEN + 4];
    __shared__ uint32_t cls_words[64];
    __shared__ int sh_acc;
    __shared__ uint32_t sh_out[4];                                 // n_items, H, n_front, root_done
    const uint32_t lane = threadIdx.x, b = blockIdx.x;              // one wavefront per slot: everything below is the same in all lanes
    const int32_t tok = token_ids[b];
    int32_t code = kAccOk;
    FillRow r = D.rows[b];
    if (tok == kTokenReset) start_sequence(D, b, r.tables_idx, lane, 64);
    else if (tok < 0) code = kAccOk;                                 // nothing for this slot
    else if (r.pad[1]) code = kAccOverflow;                          // unusable until reset
    else if ((r.flags & 2u) || (uint32_t)tok >= Vd.V) code = kAccInvalid;
    else if ((uint32_t)tok == eos_id) {
        if (!(r.flags & 1u)) code = kAccRejected;
        else if (lane == 0) D.rows[b].flags = r.flags | 2u;          // the sequence ends here
    } else {
        const uint32_t rank = Vd.rank[tok];
        if (rank >= Vd.n_sorted) code = kAccRejected;                // special and empty tokens are never allowed
        else {
            const uint32_t off = Vd.off[rank];
            const int n = (int)(Vd.off[rank + 1] - off);
            const uint32_t nb = r.pad[0] ^ 1u;
            const CacheDev Cd = D.caches[r.tables_idx];             // by value: no reload after every store
            const size_t slot = (size_t)nb * D.B + b;
            // the byte classes and the slot's context into LDS
            cls_words[lane] = Cd.T.byte_class_words[lane];
            const uint32_t n_wait_in = D.wait_off[r.waitoff_off + r.H];
            for (uint32_t k = lane; k < r.item_n; k += 64) in_items[k] = D.items[r.item_off + k];
            for (uint32_t k = lane; k <= r.H; k += 64) in_wait_off[k] = D.wait_off[r.waitoff_off + k];
            for (uint32_t k = lane; k < n_wait_in; k += 64) in_wait[k] = D.wait[r.wait_base + k];
            __syncthreads();
            if (lane == 0) {
                MatcherIn in{in_items, r.item_n, in_wait, in_wait_off, r.H};
                MatcherOut out{out_items, out_wait, out_wait_off, out_front, ACC_KI, ACC_KH, ACC_KW, ACC_KF, 0, 0, 0, 0};
                OneLaneStore st;
                st.init(lists);
                OneLaneScratchX<ACC_KH + ACCEPT_MAXLEN, ACC_KF> x{x_map, x_front};
                int acc = accept_token(Cd, cls_words, in, Vd.bytes + off, n, st, x, out);
                if (acc == ACC_RETRY) {
                    // lists in device memory, results straight to the slot's other buffer
                    MatcherIn gin{D.items + r.item_off, r.item_n, D.wait + r.wait_base, D.wait_off + r.waitoff_off, r.H};
                    MatcherOut gout{D.items + slot * D.KI, D.wait + slot * D.KW, D.wait_off + slot * (D.KH + 1), D.front + (size_t)b * D.KF,
                                    D.KI, D.KH, D.KW, D.KF, 0, 0, 0, 0};
                    GlobalStore gs;
                    gs.init(D.slow_mem + b, D.B);
                    GlobalScratchX gx{D.slow_map + b, D.slow_front + b, D.B, D.KH + kSlowMaxLen + 1, D.KF};
                    acc = accept_token(Cd, cls_words, gin, Vd.bytes + off, n, gs, gx, gout);
                    out.n_items = gout.n_items; out.H = gout.H; out.n_front = gout.n_front; out.root_done = gout.root_done;
                    if (acc == ACC_OK) acc = -1;                     // done, nothing to copy out
                }
                sh_acc = acc;
                sh_out[0] = out.n_items; sh_out[1] = out.H; sh_out[2] = out.n_front; sh_out[3] = out.root_done;
            }
            __syncthreads();
            const int acc = sh_acc;
            if (acc == ACC_OK || acc == -1) {
                const uint32_t n_items = sh_out[0], H = sh_out[1], n_front = sh_out[2];
                if (acc == ACC_OK) {
                    for (uint32_t k = lane; k < n_items; k += 64) D.items[slot * D.KI + k] = out_items[k];
                    for (uint32_t k = lane; k <= H; k += 64) D.wait_off[slot * (D.KH + 1) + k] = out_wait_off[k];
                    const uint32_t n_wait = out_wait_off[H];
                    for (uint32_t k = lane; k < n_wait; k += 64) D.wait[slot * D.KW + k] = out_wait[k];
                    for (uint32_t k = lane; k < n_front; k += 64) D.front[(size_t)b * D.KF + k] = out_front[k];
                }
                if (lane == 0) {
                    r.front_n = n_front;
                    r.item_off = (uint32_t)(slot * D.KI); r.item_n = n_items;
                    r.wait_base = (uint32_t)(slot * D.KW); r.waitoff_off = (uint32_t)(slot * (D.KH + 1)); r.H = H;
                    r.flags = sh_out[3];
                    r.pad[0] = nb;
                    D.rows[b] = r;
                }
            } else if (acc == ACC_REJECTED) code = kAccRejected;
            else { if (lane == 0) D.rows[b].pad[1] = 1u; code = kAccOverflow; }   // a capacity of the slot (or of the device-memory lists) was exceeded
        }
    }
    if (status && lane == 0) status[b] = code;
}

// ---- apply -----------------------------------------------------------------------------------------
// One 16-byte vector per thread per step: 4 fp32 or 8 bf16.  A vector whose tokens are all allowed is
// left alone (no read, no write); one whose tokens are all disallowed is overwritten without a read;
// only mixed vectors are read, merged and written back.
constexpr int APPLY_THREADS = 256, APPLY_VECS = 4;

template <int EPV /* elements per 16-byte vector */>
__global__ __launch_bounds__(APPLY_THREADS) void k_apply_vec(uint4* logits, long long row_stride_vecs, int n_vecs,
                                                             const uint32_t* bitmask, long long bm_stride) {
    const long long b = blockIdx.y;
    uint4* row = logits + b * row_stride_vecs;
    const uint32_t* bm = bitmask + b * bm_stride;
    const int v0 = blockIdx.x * (APPLY_THREADS * APPLY_VECS) + threadIdx.x;
#pragma unroll
    for (int j = 0; j < APPLY_VECS; ++j) {
        const int v = v0 + j * APPLY_THREADS;
        if (v >= n_vecs) break;
        const int e0 = v * EPV;
        const uint32_t bits = (bm[e0 >> 5] >> (e0 & 31)) & ((1u << EPV) - 1);
        if (bits == (1u << EPV) - 1) continue;
        uint4 x;
        if (EPV == 4) {
            const uint32_t NINF = 0xFF800000u;
            if (bits == 0) x = make_uint4(NINF, NINF, NINF, NINF);
            else {
                x = row[v];
                if (!(bits & 1)) x.x = NINF;
                if (!(bits & 2)) x.y = NINF;
                if (!(bits & 4)) x.z = NINF;
                if (!(bits & 8)) x.w = NINF;
            }
        } else {
            const uint32_t NINF2 = 0xFF80FF80u;
            if (bits == 0) x = make_uint4(NINF2, NINF2, NINF2, NINF2);
            else {
                x = row[v];
                auto merge = [](uint32_t w, uint32_t two) {
                    if (!(two & 1)) w = (w & 0xFFFF0000u) | 0xFF80u;
                    if (!(two & 2)) w = (w & 0x0000FFFFu) | 0xFF800000u;
                    return w;
                };
                x.x = merge(x.x, bits); x.y = merge(x.y, bits >> 2); x.z = merge(x.z, bits >> 4); x.w = merge(x.w, bits >> 6);
            }
        }
        row[v] = x;
    }
}

// Any alignment, any stride; also the tail after the last whole vector.
template <typename E>
__global__ __launch_bounds__(256) void k_apply_scalar(E* logits, long long row_stride, int v_begin, int V,
                                                      const uint32_t* bitmask, long long bm_stride, E ninf) {
    const long long b = blockIdx.y;
    const int v = v_begin + blockIdx.x * 256 + threadIdx.x;
    if (v >= V) return;
    if (!((bitmask[b * bm_stride + (v >> 5)] >> (v & 31)) & 1u)) logits[b * row_stride + v] = ninf;
}

}  // namespace

// ---- scratch of the entry point that allocates nothing ---------------------------------------------
// One array per GPU the library runs on, held until the process ends.  In host code the array's name is only
// a stand-in: the device address comes from hipGetSymbolAddress, once per device, and only that address is
// handed to kernels and copies.
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

hipError_t noalloc_scratch(void** ptr_out) {
    constexpr int kMaxDevices = 64;
    static void* ptr_of[kMaxDevices] = {};
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(mu);
    if (!ptr_of[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        ptr_of[dev] = p;
    }
    *ptr_out = ptr_of[dev];
    return hipSuccess;
}

void launch_expand_chunks(const uint4* range_a_dev, const uint4* range_b_dev, const uint32_t* first_dev, uint32_t n_ranges,
                          uint4* chunk_dev, hipStream_t stream) {
    if (!n_ranges) return;
    hipLaunchKernelGGL(k_expand_chunks, dim3((n_ranges + 255) / 256), dim3(256), 0, stream, range_a_dev, range_b_dev, first_dev, n_ranges, chunk_dev);
}

void launch_stage(void* dst_dev, const void* src_host_mapped, size_t bytes, const StageZero& Z, const uint4* range_a_host_mapped,
                  const uint4* range_b_host_mapped, const uint32_t* first_host_mapped, uint32_t n_ranges, uint4* chunk_dev, hipStream_t stream) {
    const size_t n = bytes / sizeof(uint4);
    const uint32_t nb_up = (uint32_t)std::min<size_t>((n + 255) / 256, 2048);
    size_t zero_words = 0;
    for (uint32_t k = 0; k < Z.n; ++k) zero_words += Z.words[k];
    const uint32_t nb_zero = (uint32_t)std::min<size_t>((zero_words / 4 + 255) / 256, 2048);
    const uint32_t nb_exp = (n_ranges + 255) / 256;
    if (nb_up + nb_zero + nb_exp == 0) return;
    hipLaunchKernelGGL(k_stage, dim3(nb_up + nb_zero + nb_exp), dim3(256), 0, stream, static_cast<uint4*>(dst_dev), static_cast<const uint4*>(src_host_mapped), n,
                       nb_up, Z, nb_zero, range_a_host_mapped, range_b_host_mapped, first_host_mapped, n_ranges, chunk_dev);
}

void launch_build(const DevTables& T, const DevVocab& Vd, BuildPlan P, const SlowScratch& S, hipStream_t stream) {
    if (P.n_chunks == 0) return;
    // Short item lists let a compute unit hold more workgroups, which is what hides the latency of the automaton
    // walks' dependent table loads when there is far more work than the device holds at once; long ones spare the
    // tokens that need them a second run at half width, which is what counts when the launch is a few chunks per
    // wave slot and lasts as long as its slowest workgroup.
    static const uint32_t wave_slots = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        return (uint32_t)cus * 32u;                                 // 4 SIMDs of 8 wave slots each
    }();
    P.large_lists = P.n_chunks <= 4 * wave_slots ? 1u : 0u;
#ifdef XG2_BUILD_FORCE_LISTS
    P.large_lists = XG2_BUILD_FORCE_LISTS;
#endif
    P.list_k = P.large_lists ? BUILD_K_LARGE : BUILD_K_SMALL;
    P.list_wm = P.large_lists ? BUILD_WM_LARGE : BUILD_WM_SMALL;
    const uint32_t lds_bytes = (2 * P.list_k + 2 * P.list_wm) * 64 * sizeof(uint32_t);
    // Workgroup g takes chunks g, g + grid, ...  At least one workgroup per wave slot of the device; a large launch is cut
    // into shares of about a dozen chunks, small enough for the hardware to even out the load as workgroups end and
    // large enough for a workgroup's tokens for the follow-language run to fill whole batches (measured: 8,192 for the
    // 10,063 chunks of the repetition workload, 65,536 for the 856,956 of the dispatch workload).
    uint32_t grid = std::min(P.n_chunks, std::max(wave_slots, std::min(P.n_chunks / 12, 8 * wave_slots)));
#ifdef XG2_TUNE
    if (const char* e = getenv("XG2_BUILD_GRID")) grid = std::min<uint32_t>(P.n_chunks, (uint32_t)atoi(e));
    if (getenv("XG2_DEBUG_PLAN")) fprintf(stderr, "launch: chunks %u grid %u lds %u\n", P.n_chunks, grid, lds_bytes);
#endif
    hipLaunchKernelGGL(k_build, dim3(grid), dim3(64), lds_bytes, stream, T, Vd, P, S);
}

void launch_build_slow(const DevTables& T, const DevVocab& Vd, const BuildPlan& P, const SlowScratch& S, hipStream_t stream) {
    hipLaunchKernelGGL(k_build_slow, dim3(S.n_lanes / 64), dim3(64), 0, stream, T, Vd, P, S);
}

void launch_accept(const BatchDev& D, const DevVocab& Vd, uint32_t eos_id, const int32_t* token_ids_dev, int32_t* status_dev, hipStream_t stream) {
    if (!D.B || D.KI != ACC_KI || D.KH != ACC_KH || D.KW != ACC_KW || D.KF != ACC_KF) return;
    hipLaunchKernelGGL(k_accept, dim3(D.B), dim3(64), 0, stream, D, Vd, eos_id, token_ids_dev, status_dev);
}

void launch_batch_assign(const BatchDev& D, const int32_t* rows_dev, uint32_t n, uint32_t cache_idx, hipStream_t stream) {
    if (!n) return;
    hipLaunchKernelGGL(k_batch_assign, dim3((n + 255) / 256), dim3(256), 0, stream, D, rows_dev, n, cache_idx);
}

void launch_upload(void* dst_dev, const void* src_host_mapped, size_t bytes, hipStream_t stream) {
    const size_t n = bytes / sizeof(uint4);
    if (!n) return;
    const uint32_t grid = (uint32_t)std::min<size_t>((n + 255) / 256, 2048);
    hipLaunchKernelGGL(k_upload, dim3(grid), dim3(256), 0, stream, static_cast<uint4*>(dst_dev), static_cast<const uint4*>(src_host_mapped), n);
}

void launch_copy_masked(const CopyJob* jobs_dev, uint32_t n_jobs, uint32_t W, hipStream_t stream) {
    if (!n_jobs) return;
    for (uint32_t first = 0; first < n_jobs; first += 65535) {      // grid.y limit
        const uint32_t n = std::min<uint32_t>(65535, n_jobs - first);
        hipLaunchKernelGGL(k_copy_masked, dim3((W + 255) / 256, n), dim3(256), 0, stream, jobs_dev + first, W);
    }
}

void launch_copy_structure(const CopyJob* jobs_dev, uint32_t n_jobs, uint32_t W, hipStream_t stream) {
    for (uint32_t first = 0; first < n_jobs; first += 65535) {      // grid.y limit
        const uint32_t n = std::min<uint32_t>(65535, n_jobs - first);
        hipLaunchKernelGGL(k_copy_structure, dim3((W + 255) / 256, n), dim3(256), 0, stream, jobs_dev + first, W);
    }
}

void launch_copy_first_byte(const FirstByteCopyJob* jobs_dev, uint32_t n_jobs, const uint8_t* first_byte_dev, uint32_t W, hipStream_t stream) {
    for (uint32_t first = 0; first < n_jobs; first += 65535) {      // grid.y limit
        const uint32_t n = std::min<uint32_t>(65535, n_jobs - first);
        hipLaunchKernelGGL(k_copy_first_byte, dim3((W + 255) / 256, n), dim3(256), 0, stream, jobs_dev + first, first_byte_dev, W);
    }
}

void launch_plane_summary(uint32_t* const* plane_ptr_dev, uint32_t n_pos, uint32_t W, uint32_t* counts_dev, hipStream_t stream) {
    if (n_pos == 0) return;
    hipLaunchKernelGGL(k_plane_summary, dim3(n_pos), dim3(256), 0, stream, plane_ptr_dev, n_pos, W, counts_dev);
}

void launch_finish_planes(uint32_t* const* plane_ptr_dev, const FinishJob* jobs_dev, uint32_t n_pos, const uint8_t* first_byte_dev, uint32_t W,
                          uint32_t* counts_dev, hipStream_t stream) {
    for (uint32_t first = 0; first < n_pos; first += 65535) {       // grid.y limit
        const uint32_t n = std::min<uint32_t>(65535, n_pos - first);
        hipLaunchKernelGGL(k_finish_planes, dim3((W + FINISH_WORDS - 1) / FINISH_WORDS, n), dim3(256), 0, stream, plane_ptr_dev + first, jobs_dev + first, n,
                           first_byte_dev, W, counts_dev + 2 * (size_t)first);
    }
}

void launch_fill(const FillBatch& F, const DevVocab& Vd, int32_t* bitmask_dev, int64_t row_stride_words,
                 const SlowScratch& S, hipStream_t stream) {
    if (F.B == 0) return;
    const bool wide = Vd.W % 4 == 0 && row_stride_words % 4 == 0 && ((uintptr_t)bitmask_dev & 15) == 0;   // plane rows are 16-byte aligned when W % 4 == 0
    if (wide) hipLaunchKernelGGL(k_fill<4>, dim3(F.B), dim3(FILL_THREADS), 0, stream, F, Vd, bitmask_dev, (long long)row_stride_words, S);
    else hipLaunchKernelGGL(k_fill<1>, dim3(F.B), dim3(FILL_THREADS), 0, stream, F, Vd, bitmask_dev, (long long)row_stride_words, S);
}

void launch_recheck_slow(const FillBatch& F, const DevVocab& Vd, int32_t* bitmask_dev, int64_t row_stride_words,
                         const SlowScratch& S, hipStream_t stream) {
    hipLaunchKernelGGL(k_recheck_slow, dim3(S.n_lanes / 64), dim3(64), 0, stream, F, Vd, bitmask_dev, (long long)row_stride_words, S);
}

void launch_apply(void* logits_dev, int32_t dtype, int32_t B, int32_t V, int64_t row_stride_elems,
                  const int32_t* bitmask_dev, int64_t bm_row_stride_words, hipStream_t stream) {
    if (B == 0 || V == 0) return;
    const int esize = dtype == 0 ? 4 : 2;
    const int epv = 16 / esize;
    const bool aligned = (reinterpret_cast<uintptr_t>(logits_dev) % 16 == 0) && ((row_stride_elems * esize) % 16 == 0);
    const int n_vecs = aligned ? V / epv : 0;
    const uint32_t* bm = reinterpret_cast<const uint32_t*>(bitmask_dev);
    if (n_vecs > 0) {
        dim3 grid((n_vecs + APPLY_THREADS * APPLY_VECS - 1) / (APPLY_THREADS * APPLY_VECS), B);
        if (dtype == 0)
            hipLaunchKernelGGL(k_apply_vec<4>, grid, dim3(APPLY_THREADS), 0, stream, (uint4*)logits_dev,
                               (long long)(row_stride_elems / 4), n_vecs, bm, (long long)bm_row_stride_words);
        else
            hipLaunchKernelGGL(k_apply_vec<8>, grid, dim3(APPLY_THREADS), 0, stream, (uint4*)logits_dev,
                               (long long)(row_stride_elems / 8), n_vecs, bm, (long long)bm_row_stride_words);
    }
    const int v_begin = n_vecs * epv;
    if (v_begin < V) {
        dim3 grid((V - v_begin + 255) / 256, B);
        if (dtype == 0)
            hipLaunchKernelGGL(k_apply_scalar<uint32_t>, grid, dim3(256), 0, stream, (uint32_t*)logits_dev, (long long)row_stride_elems,
                               v_begin, V, bm, (long long)bm_row_stride_words, 0xFF800000u);
        else
            hipLaunchKernelGGL(k_apply_scalar<uint16_t>, grid, dim3(256), 0, stream, (uint16_t*)logits_dev, (long long)row_stride_elems,
                               v_begin, V, bm, (long long)bm_row_stride_words, (uint16_t)0xFF80);
    }
}

}  // namespace xg2
