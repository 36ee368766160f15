// Launchers of the gfx950 kernels.  Plain pointers and sizes only; every pointer named *_dev is
// device memory.  All launches go to `stream`; none of them synchronises.
#pragma once
#include <cstdint>
#include <hip/hip_runtime.h>

namespace xg2 {

struct DevTables {                       // packed grammar tables (see tables.hpp for the word layout)
    const uint4* state;                  // {rule, expansion offset, n_items, n_triples}: loaded only for states with
                                         // rule edges (what entering them adds) and for completing items (their rule)
    const uint32_t* exp_list;            // expansions: item words, then {rule, target} pairs
    const uint32_t* trans;               // [(n_states + 1) * n_classes] state reference of the byte target, or `sink`
    const uint32_t* byte_class_words;    // [64] byte -> class, four per word
    uint32_t n_classes;
    uint32_t sink;                       // the state (without flags) that missing edges lead to; its own row leads back to it
    const uint32_t* site_off;            // per rule: states in which referencing rules continue (CSR)
    const uint32_t* site_tgt;
};

struct DevVocab {                        // byte-sorted vocabulary in HBM
    const uint8_t* bytes;                // concatenated token bytes in sorted order
    const uint32_t* off;                 // [n_sorted + 1]
    const uint4* tok16;                  // [n_sorted] first 16 bytes of each token, zero padded: one coalesced load
                                         // instead of sixteen byte loads for the tokens the LDS path handles
    const uint32_t* perm;                // sorted rank -> token id
    const uint32_t* rank;                // token id -> sorted rank, 0xFFFFFFFF for tokens never checked
    const uint32_t* long_rank;           // per length bound d, ascending: the sorted ranks of the tokens longer than d bytes
    uint32_t n_sorted;                   // checkable tokens (non-special, non-empty)
    uint32_t V, W;
};

// Work plan of one cache build.  A chunk is a record of two uint4: the first {plane, first rank, end rank, flags}, the
// second what the automaton walk needs of the plane without a further load {first item of the start set, number of
// its items, row address low, row address high}.  Below, chunk[c] stands for the first half of record c.
// Chunk c covers sorted ranks [chunk[c].y, chunk[c].z) of plane chunk[c].x
// (at most kBuildChunk tokens, all with a first byte the plane's start set can read); with bit 0 of chunk[c].w
// set, y and z index DevVocab::long_rank instead and the ranks are read from there (a plane that needs only
// its long tokens checked).  The workgroups of a persistent grid take chunks round-robin.  plane_ctx[k] = {first item, number of items, first wait offset, H} describes the closed start
// set of plane k as a scan context (H = 1: the position alone; H = 2: the position inside one level of
// referencing rule).  ctx_wait holds, set after set, what the waiting items wait for as pairs
// {rule, state reference of the target | origin << 21}; ctx_wait_off counts pairs.  With bit 2 of chunk[c].w set,
// four more words follow the plane's items in ctx_items: {item a, lead a, item b or kNoThread, lead b}, the start
// set's one or two scanning items and, for an item of a waited-for instance, the item of the outermost instance
// that its end leads to (the only wait entry of its rule; neither predicts) — the kernel walks these as threads.
#ifndef XG2_BUILD_CHUNK
#define XG2_BUILD_CHUNK 128
#endif
constexpr uint32_t kBuildChunk = XG2_BUILD_CHUNK;
#ifndef XG2_HEAVY_CHUNK
#define XG2_HEAVY_CHUNK XG2_BUILD_CHUNK
#endif
constexpr uint32_t kHeavyChunk = XG2_HEAVY_CHUNK;             // chunk size of planes whose tokens all take the Earley steps
static_assert(kHeavyChunk <= kBuildChunk && kBuildChunk <= 256, "the deferred list is sized for kBuildChunk and holds one-byte offsets");
struct BuildPlan {
    const uint4* chunk; uint32_t n_chunks;                      // 2 * n_chunks uint4
    const uint4* plane_ctx;                                     // [n_planes]
    const uint32_t* ctx_items; const uint2* ctx_wait; const uint32_t* ctx_wait_off;
    uint32_t* const* plane_ptr;                                 // [n_planes] accepted row; uncertain row at + W words, left-early row at + 2 W
    uint32_t follow_filter;                                     // drop uncertain tokens that no reference site can continue
    uint32_t large_lists, list_k, list_wm;                      // set by launch_build: long or short item lists; item and wait-entry capacity a lane
};

struct FillRow;
struct SlowScratch {                     // large-capacity per-lane Earley scratch in device memory
    uint32_t* mem; uint32_t n_lanes;     // mem holds n_lanes * kSlowSlots words
    uint32_t* list; uint32_t list_cap;   // overflow work list: pairs (a, b)
    uint32_t* count;                     // [0] = entries in list, [1] = sticky error flag
    uint32_t k_cap, wm_cap;              // item and wait-entry capacity in use (at most kSlowK, kSlowWM; smaller only in tests
                                         // of the overflow handling); below the LDS lists' 16 / 32 those are skipped
    // fill only: where the (row, token) pairs that even these lists could not decide are reported: a counter and a list in
    // pinned host memory (device-side address; null: not reported), and, for matchers on the device, the slots' rows
    uint32_t* unresolved; uint32_t unresolved_cap;       // [0] = 1 if any, [1] = 1 if more than fit; pairs from word 2 on (the host presets them to ~0)
    FillRow* mark_rows;                                  // not null: rows[b].pad[1] gets the sticky error
};
constexpr uint32_t kSlowK = 256, kSlowWM = 1024, kSlowMaxLen = 1024;
constexpr uint32_t kSlowSearchBudget = 1u << 20;     // list entries one token may compare against in the device-memory lists
constexpr uint32_t kSlowSlots = 2 * kSlowK + 2 * kSlowWM + kSlowMaxLen + 1;

constexpr uint32_t kChunkListed = 1u, kChunkHeavy = 2u, kChunkThreads = 4u, kChunkDerive = 8u;   // bits of chunk[c].w
constexpr uint32_t kDeriveChunk = 64;                        // mask words of a derive chunk: y and z are word indices there, and the second
                                                             // half of the record holds the address of the base plane's third row
constexpr uint32_t kNoThread = 0xFFFFFFFFu;                  // an empty slot of the thread walk (what the transition table holds for "no edge")

// dst gets, for the tokens in mask (token ids, W words), the bits src holds: all three rows of a plane at once
// (accepted at [0, W), uncertain at [W, 2 W), left early at [2 W, 3 W)).  The mask bits of dst must be clear before.
struct CopyJob { uint32_t* dst; const uint32_t* src; const uint32_t* mask; uint64_t pad; };
void launch_copy_masked(const CopyJob* jobs_dev, uint32_t n_jobs, uint32_t W, hipStream_t stream);
// dst gets src's accepted row and left-early row whole (mask unused): what a plane derived from another one shares with it.
void launch_copy_structure(const CopyJob* jobs_dev, uint32_t n_jobs, uint32_t W, hipStream_t stream);
// The same with the mask given by first bytes: dst gets the bits src holds for the tokens whose first byte is in the
// set `bytes` (256 bits).  first_byte_dev: first byte of every token id, padded to W * 32 entries.
struct FirstByteCopyJob { uint32_t* dst; const uint32_t* src; uint32_t bytes[8]; };
void launch_copy_first_byte(const FirstByteCopyJob* jobs_dev, uint32_t n_jobs, const uint8_t* first_byte_dev, uint32_t W, hipStream_t stream);

// Writes the chunk records of a build: thread r cuts range_a[r] = {plane, first rank, end rank, flags} into chunks of
// kBuildChunk (kHeavyChunk with kChunkHeavy) ranks, records first[r], first[r] + 1, ..., each followed by range_b[r].
void launch_expand_chunks(const uint4* range_a_dev, const uint4* range_b_dev, const uint32_t* first_dev, uint32_t n_ranges,
                          uint4* chunk_dev, hipStream_t stream);
// One launch for what a build needs first: the copy of `bytes` (a multiple of 16) from pinned host memory (given by its
// device address) to dst_dev, the clearing of up to kStageZeroRanges ranges of words, and the chunk records (as
// launch_expand_chunks, but reading the ranges through the device addresses of their pinned host copies).
constexpr uint32_t kStageZeroRanges = 8;
struct StageZero { uint32_t* p[kStageZeroRanges]; uint64_t words[kStageZeroRanges]; uint32_t n; };
void launch_stage(void* dst_dev, const void* src_host_mapped, size_t bytes, const StageZero& Z, const uint4* range_a_host_mapped,
                  const uint4* range_b_host_mapped, const uint32_t* first_host_mapped, uint32_t n_ranges, uint4* chunk_dev, hipStream_t stream);
void launch_build(const DevTables& T, const DevVocab& Vd, BuildPlan P, const SlowScratch& S, hipStream_t stream);
void launch_build_slow(const DevTables& T, const DevVocab& Vd, const BuildPlan& P, const SlowScratch& S, hipStream_t stream);
// What a freshly classed plane still lacks: the bits it takes from other planes (either kind, or none: null sources).
// m_src under the token mask m_mask (all three rows, as launch_copy_masked); f_src for the tokens whose first byte is in
// f_bytes (as launch_copy_first_byte).  The sources must not themselves be planes that take bits in the same launch.
struct FinishJob { const uint32_t* m_src; const uint32_t* m_mask; const uint32_t* f_src; uint32_t f_bytes[8]; uint32_t pad[2]; };
// One pass over every built plane: the copies above, then what launch_plane_summary does, on the words in registers.
void launch_finish_planes(uint32_t* const* plane_ptr_dev, const FinishJob* jobs_dev, uint32_t n_pos, const uint8_t* first_byte_dev, uint32_t W,
                          uint32_t* counts_dev, hipStream_t stream);
// A plane in device memory: three rows of W words (accepted, uncertain, left early) and behind them the list of its
// uncertain tokens: word 0 = how many (the list holds them if that is at most kUncListWords - 1), then their token ids.
constexpr uint32_t kUncListWords = 64;
constexpr size_t plane_words(uint32_t W) { return 3 * (size_t)W + kUncListWords; }
// counts_dev[2p], counts_dev[2p + 1] = set bits of the accepted and of the uncertain row of plane p; also writes the
// plane's list of uncertain tokens
void launch_plane_summary(uint32_t* const* plane_ptr_dev, uint32_t n_pos, uint32_t W, uint32_t* counts_dev, hipStream_t stream);

// One row of a fill batch.
struct FillRow {
    uint32_t front_off, front_n;         // into front_planes
    uint32_t item_off, item_n;           // into ctx_items
    uint32_t wait_base;                  // into ctx_wait (pairs)
    uint32_t waitoff_off, H;             // into ctx_wait_off ([H + 1] entries, relative to wait_base)
    uint32_t tables_idx;                 // into tables
    uint32_t flags;                      // bit 0: root can end, bit 1: terminated
    uint32_t pad[3];
};
struct FillBatch {
    const FillRow* rows; uint32_t B;
    const uint64_t* front_planes;        // device addresses of accepted rows (uncertain at + W words, list of uncertain tokens at + 3 W);
                                         // bit 0 set: only the accepted row counts (root instance)
    const uint32_t* ctx_items; const uint2* ctx_wait; const uint32_t* ctx_wait_off;
    const DevTables* tables;
    uint32_t eos_id;
    // re-check scratch: candidate bits of every mask word; per row, the indices of the non-zero ones and their count
    uint32_t* cand_words;                // [B * W]
    uint32_t* work_list;                 // [B * W], row b's list starts at b * W
    uint32_t* row_count;                 // [B], written by the fill kernel: candidate tokens of the row
    uint32_t* zero_words;                // if not null: four words the large-capacity kernel clears for the next call (the overflow
                                         // list's length and flag, where no upload brings them in as zeros: two sets take turns)
};
void launch_fill(const FillBatch& F, const DevVocab& Vd, int32_t* bitmask_dev, int64_t row_stride_words,
                 const SlowScratch& S, hipStream_t stream);
void launch_recheck_slow(const FillBatch& F, const DevVocab& Vd, int32_t* bitmask_dev, int64_t row_stride_words,
                         const SlowScratch& S, hipStream_t stream);

// ---- matchers that live on the device ------------------------------------------------------------------------
// What a matcher needs of its mask cache besides the tables: the plane of every (state) and (state, state the
// referencing rule continues in), as device addresses of accepted rows with bit 0 = "only the accepted row counts"
// (an all-zero uncertain row), and the matcher state a new sequence starts from.
struct CacheDev {
    DevTables T;
    const uint64_t* plain_row;           // [n_states] plane of a position without context (root rule, or context depth 1), 0 = none
    const uint32_t* pair_off;            // [n_states + 1] CSR over states: the planes of the state under its referencing sites
    const uint32_t* pair_key;            //   state id the referencing rule continues in, ascending within a state
    const uint64_t* pair_row;
    uint32_t context_depth;
    uint32_t start_n_items, start_H, start_n_front, start_flags;
    const uint32_t* start_items; const uint2* start_wait; const uint32_t* start_wait_off; const uint64_t* start_front;
};
// B matcher slots of fixed capacity.  Slot b's state is what FillRow b points at: its frontier planes at front[b * KF ..],
// and its parser context (items of the current closed set that can scan; per reachable older set what its waiting items
// wait for) in one of two buffers, c = rows[b].pad[0]: items[(c * B + b) * KI ..], wait[(c * B + b) * KW ..],
// wait_off[(c * B + b) * (KH + 1) ..].  Accepting a token writes the other buffer and switches.  rows[b].pad[1] holds a
// sticky error (a capacity was exceeded: the slot is unusable until it is reset), rows[b].tables_idx the slot's cache.
constexpr uint32_t kSlotItems = 64, kSlotSets = 240, kSlotWaits = 512, kSlotPlanes = 32;   // capacities of a matcher slot
struct BatchDev {
    uint32_t B, KI, KH, KW, KF;                          // KI .. KF: the four capacities above
    FillRow* rows;
    uint64_t* front; uint32_t* items; uint2* wait; uint32_t* wait_off;
    const CacheDev* caches; const DevTables* tables;     // [number of caches in use] (tables: the same DevTables, as fill wants them)
    uint32_t* slow_mem;                                   // item lists in device memory for tokens the LDS lists cannot take: B * kSlowSlots words
    uint8_t* slow_map;                                    // and the set renumbering table: B * (KH + kSlowMaxLen + 1) bytes
    uint64_t* slow_front;                                 // B * KF staging words
};
constexpr int32_t kTokenReset = -2;      // xg2_batch_accept_tokens: "start a new sequence in this slot"
// status codes written per slot (the XG2_* values of the C ABI)
constexpr int32_t kAccOk = 0, kAccInvalid = -1, kAccRejected = -3, kAccOverflow = -4;
void launch_accept(const BatchDev& D, const DevVocab& Vd, uint32_t eos_id, const int32_t* token_ids_dev, int32_t* status_dev, hipStream_t stream);
// rows_dev (n of them; nullptr = slots 0 .. n - 1) start a new sequence of cache `cache_idx`
void launch_batch_assign(const BatchDev& D, const int32_t* rows_dev, uint32_t n, uint32_t cache_idx, hipStream_t stream);

// Copies `bytes` (a multiple of 16) from pinned host memory, given by its device-side address, to device memory with
// a kernel: for the small per-call uploads this has less latency than the copy engine.
void launch_upload(void* dst_dev, const void* src_host_mapped, size_t bytes, hipStream_t stream);

// The entry point that allocates nothing works in a fixed device array of the library (one per GPU, kept until the
// process ends) instead of buffers that grow with the batch: staging of the per-row records, candidate words and
// work lists, row counts, the overflow list and the large-capacity item lists.  noalloc_scratch gives the array's
// device address on the current device (looked up once per device).
constexpr size_t kNoAllocStagingBytes = (size_t)1 << 20;            // per-row records, frontier planes, context slices
constexpr size_t kNoAllocMaskWords = (size_t)1 << 20;               // rows x ceil(V/32) of one call
constexpr size_t kNoAllocMaxRows = 4096;
constexpr uint32_t kNoAllocSlowLanes = 256, kNoAllocListCap = 1u << 16;
constexpr size_t kNoAllocScratchBytes = kNoAllocStagingBytes + 2 * kNoAllocMaskWords * 4 + kNoAllocMaxRows * 4
                                        + (size_t)kNoAllocListCap * 8 + (size_t)kNoAllocSlowLanes * kSlowSlots * 4;
hipError_t noalloc_scratch(void** ptr_out);

void launch_apply(void* logits_dev, int32_t dtype, int32_t B, int32_t V, int64_t row_stride_elems,
                  const int32_t* bitmask_dev, int64_t bm_row_stride_words, hipStream_t stream);

}  // namespace xg2
