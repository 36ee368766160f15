// C ABI of libxg2mask.so (see include/xg2mask.h): argument checking, handle lifetime, host-side
// planning of the cache build and of a fill batch, and the launches.  There is no CPU fallback for any
// kernel: without a HIP device the device calls fail with XG2_EHIP.
#include "../../include/xg2mask.h"

#include <algorithm>
#include <array>
#include <atomic>
#include <chrono>
#include <cstring>
#include <deque>
#include <map>
#include <set>
#include <memory>
#include <mutex>
#include <numeric>
#include <string>
#include <condition_variable>
#include <functional>
#include <thread>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include <hip/hip_runtime.h>

#include "device.hpp"
#include "grammar.hpp"
#include "tables.hpp"

using namespace xg2;

namespace {

thread_local std::string g_error;
int32_t fail(int32_t code, const std::string& msg) { g_error = msg; return code; }

struct HipError : std::runtime_error { using std::runtime_error::runtime_error; };
#define HIP_CHECK(expr)                                                                              \
    do {                                                                                             \
        hipError_t e_ = (expr);                                                                      \
        if (e_ != hipSuccess) throw HipError(std::string(#expr) + ": " + hipGetErrorString(e_));     \
    } while (0)

template <typename T>
struct DevBuf {                                    // owning device array
    T* p = nullptr; size_t n = 0;
    DevBuf() = default;
    DevBuf(const DevBuf&) = delete;
    DevBuf& operator=(const DevBuf&) = delete;
    ~DevBuf() { if (p) (void)hipFree(p); }
    void alloc(size_t count) {
        if (p) { (void)hipFree(p); p = nullptr; }
        n = count;
        if (count) HIP_CHECK(hipMalloc((void**)&p, count * sizeof(T)));
    }
    void upload(const std::vector<T>& v, hipStream_t s) {
        alloc(std::max<size_t>(v.size(), 1));
        if (!v.empty()) HIP_CHECK(hipMemcpyAsync(p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice, s));
    }
};

// Pinned host memory to device memory on `stream`: small blocks by a copy kernel that reads the host memory through its
// device-side address (less latency than the copy engine), large ones by the runtime.  bytes: a multiple of 16.
constexpr size_t kUploadByKernelMax = (size_t)4 << 20;
inline void upload_pinned(void* dev, void* host, size_t bytes, hipStream_t stream) {
    if (bytes <= kUploadByKernelMax) {
        void* mapped = nullptr;
        HIP_CHECK(hipHostGetDevicePointer(&mapped, host, 0));
        launch_upload(dev, mapped, bytes, stream);
    } else {
        HIP_CHECK(hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, stream));
    }
}

// Several host arrays laid out back to back (256-byte aligned) in one pinned buffer, moved to the device
// with one copy.
// A build does not wait for its kernels, so the pinned host buffer, the device buffer (for uploads that need not
// outlive the build), the pinned words its results come back in and its events belong to one staging set from the
// moment the build is enqueued until it has been looked at (finalised); sets are kept and handed out again
// (allocating them costs more than a small build).
struct StagingSet {
    uint8_t* host = nullptr; size_t host_cap = 0;
    uint8_t* dev = nullptr; size_t dev_cap = 0;
    uint32_t* res = nullptr; size_t res_cap = 0;                // pinned: overflow counter and flag, bit counts per built plane
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};   // around the build, around its classification kernel, results copied
    bool in_use = false;
    void ensure_events() { for (hipEvent_t& e : ev) if (!e) HIP_CHECK(hipEventCreate(&e)); }
    void ensure_res(size_t words) {
        if (res_cap >= words) return;
        if (res) (void)hipHostFree(res);
        res = nullptr; res_cap = 0;
        const size_t cap = std::max<size_t>(words * 2, 1024);
        HIP_CHECK(hipHostMalloc((void**)&res, cap * sizeof(uint32_t), hipHostMallocDefault));
        res_cap = cap;
    }
};
struct StagingPool {
    std::mutex mu;
    std::vector<std::unique_ptr<StagingSet>> sets;
    StagingSet* acquire() {
        std::lock_guard<std::mutex> lk(mu);
        for (auto& p : sets) if (!p->in_use) { p->in_use = true; return p.get(); }
        sets.emplace_back(new StagingSet());
        sets.back()->in_use = true;
        return sets.back().get();
    }
    void release(StagingSet* s) { std::lock_guard<std::mutex> lk(mu); s->in_use = false; }
};
StagingPool& staging_pool() { static StagingPool* s = new StagingPool(); return *s; }
// test aid: off = a build uses one launch per step (clear, upload, chunk records; copy kernels, summary) even where one would do
std::atomic<bool>& build_fusion() { static std::atomic<bool> on{true}; return on; }

struct Packer {
    struct Seg { const void* src; size_t bytes, off; };
    std::vector<Seg> segs;
    size_t total = 0;
    uint8_t* host = nullptr;
    uint8_t* dev = nullptr;
    template <typename T> size_t add(const std::vector<T>& v) {
        size_t off = total;
        segs.push_back({v.data(), v.size() * sizeof(T), off});
        total = (total + v.size() * sizeof(T) + 255) & ~(size_t)255;
        return off;
    }
    // room in the device block behind the uploaded arrays, written by kernels only
    size_t reserved = 0;
    size_t reserve(size_t bytes) {
        const size_t off = total + reserved;
        reserved = (reserved + bytes + 255) & ~(size_t)255;
        return off;
    }
    // own_dev: the device block is allocated for this upload and belongs to the caller afterwards
    void stage(bool own_dev, StagingSet& S) {
        const size_t n = std::max<size_t>(total, 256), n_dev = n + reserved;
        if (S.host_cap < n) {
            if (S.host) (void)hipHostFree(S.host);
            S.host = nullptr; S.host_cap = 0;
            const size_t cap = std::max<size_t>(n + n / 2, (size_t)1 << 20);
            HIP_CHECK(hipHostMalloc((void**)&S.host, cap, hipHostMallocDefault));
            S.host_cap = cap;
        }
        host = S.host;
        if (own_dev) {
            HIP_CHECK(hipMalloc((void**)&dev, n_dev));
        } else {
            if (S.dev_cap < n_dev) {
                if (S.dev) (void)hipFree(S.dev);
                S.dev = nullptr; S.dev_cap = 0;
                const size_t cap = std::max<size_t>(n_dev + n_dev / 2, (size_t)1 << 20);
                HIP_CHECK(hipMalloc((void**)&S.dev, cap));
                S.dev_cap = cap;
            }
            dev = S.dev;
        }
        for (const Seg& s : segs) if (s.bytes) std::memcpy(host + s.off, s.src, s.bytes);
    }
    void copy(hipStream_t stream) { if (total) upload_pinned(dev, host, total, stream); }
    template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(dev + off); }
};

// What the entry point that allocates nothing needs besides the fixed device array: two pinned host buffers for the
// per-row records and an event each, made when the first vocabulary goes to the device (set-up), never in the entry
// point itself.
struct NoAllocHost {
    std::mutex mu;
    bool ready = false;
    uint8_t* host[2] = {nullptr, nullptr};
    hipEvent_t done[2] = {nullptr, nullptr};
    bool in_flight[2] = {false, false};
    int next = 0;
    void* scratch_dev = nullptr;
    void setup() {
        std::lock_guard<std::mutex> lk(mu);
        if (ready) return;
        HIP_CHECK(noalloc_scratch(&scratch_dev));
        for (int k = 0; k < 2; ++k) {
            HIP_CHECK(hipHostMalloc((void**)&host[k], kNoAllocStagingBytes, hipHostMallocDefault));
            HIP_CHECK(hipEventCreateWithFlags(&done[k], hipEventDisableTiming));
        }
        ready = true;
    }
};
NoAllocHost& noalloc_host() { static NoAllocHost* h = new NoAllocHost(); return *h; }

void require_device() {
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || n <= 0) throw HipError("no HIP device available (the mask cache runs on the GPU only)");
}

// ---- vocabulary --------------------------------------------------------------------------------------
struct VocabImpl {
    int32_t V = 0, eos = 0;
    uint32_t W = 0;
    std::vector<uint8_t> bytes;                 // id order
    std::vector<uint64_t> offs;
    std::vector<uint8_t> special;               // [V] 1 = never allowed by a plane (special or empty)
    // byte-sorted layout
    std::vector<uint32_t> perm, rank, s_off;
    std::vector<uint8_t> s_bytes;
    uint32_t fb_start[257];                     // first sorted rank whose first byte is >= b
    uint32_t n_sorted = 0;
    uint32_t max_len = 0;                       // longest checkable token, in bytes
    // device copy (made at first use)
    std::mutex mu;
    bool on_device = false;
    DevBuf<uint8_t> d_bytes; DevBuf<uint32_t> d_off, d_perm, d_rank; DevBuf<uint4> d_tok16;
    DevVocab dv{};
    // per length bound d = 1 .. near_depths: the sorted ranks of the tokens longer than d bytes (ascending; list d is
    // long_rank[long_off[d] .. long_off[d + 1])), and on the device also the mask, in token ids, of the checkable tokens
    // of at most d bytes (row d - 1 of d_short_mask)
    uint32_t near_depths = 0;
    std::vector<uint32_t> long_rank, long_off;
    std::vector<uint64_t> long_bytes;           // long_bytes[i] = bytes of the tokens long_rank[0 .. i) (for the statistics of a build)
    void extend_long_bytes() {
        if (long_bytes.empty()) long_bytes.push_back(0);
        for (size_t i = long_bytes.size() - 1; i < long_rank.size(); ++i) {
            const uint32_t r = long_rank[i];
            long_bytes.push_back(long_bytes.back() + (r < n_sorted ? s_off[r + 1] - s_off[r] : 0u));
        }
    }
    DevBuf<uint32_t> d_long_rank, d_short_mask;
    DevBuf<uint8_t> d_first_byte;               // first byte of every token id (0 for the empty ones), W * 32 entries
    // per byte set asked for so far: the sorted ranks of the tokens that contain a byte of the set (ascending, appended
    // to long_rank) and, on the device, the mask in token ids of the checkable tokens that contain none
    struct ByteSetList { std::array<uint32_t, 8> bytes; uint32_t off, n; std::unique_ptr<DevBuf<uint32_t>> d_without; };
    std::vector<ByteSetList> byte_lists;
    // The caller serialises (the mutex of the large-capacity scratch) and no kernel is in flight on the lists.
    int32_t list_of_tokens_with(const std::array<uint32_t, 8>& bytes) {
        for (size_t k = 0; k < byte_lists.size(); ++k) if (byte_lists[k].bytes == bytes) return (int32_t)k;
        ByteSetList bl;
        bl.bytes = bytes;
        bl.off = (uint32_t)long_rank.size();
        std::vector<uint32_t> without(W, 0u);
        for (uint32_t r = 0; r < n_sorted; ++r) {
            bool has = false;
            for (uint32_t k = s_off[r]; k < s_off[r + 1] && !has; ++k) has = (bytes[s_bytes[k] >> 5] >> (s_bytes[k] & 31)) & 1u;
            if (has) long_rank.push_back(r);
            else without[perm[r] >> 5] |= 1u << (perm[r] & 31);
        }
        bl.n = (uint32_t)long_rank.size() - bl.off;
        extend_long_bytes();
        bl.d_without.reset(new DevBuf<uint32_t>());
        bl.d_without->upload(without, nullptr);
        HIP_CHECK(hipDeviceSynchronize());                           // builds in flight read the list that is replaced here
        d_long_rank.upload(long_rank, nullptr);
        HIP_CHECK(hipStreamSynchronize(nullptr));
        dv.long_rank = d_long_rank.p;
        byte_lists.push_back(std::move(bl));
        return (int32_t)byte_lists.size() - 1;
    }

    const uint8_t* tok(int32_t id) const { return bytes.data() + offs[(size_t)id]; }
    size_t len(int32_t id) const { return (size_t)(offs[(size_t)id + 1] - offs[(size_t)id]); }

    void ensure_device() {
        std::lock_guard<std::mutex> lk(mu);
        if (on_device) return;
        require_device();
        std::vector<uint8_t> padded = s_bytes;
        padded.resize(s_bytes.size() + 32, 0);
        d_bytes.upload(padded, nullptr);
        d_off.upload(s_off, nullptr);
        d_perm.upload(perm, nullptr);
        d_rank.upload(rank, nullptr);
        std::vector<uint4> tok16(n_sorted, make_uint4(0, 0, 0, 0));
        for (uint32_t r = 0; r < n_sorted; ++r)
            std::memcpy(&tok16[r], s_bytes.data() + s_off[r], std::min<size_t>(16, s_off[r + 1] - s_off[r]));
        d_tok16.upload(tok16, nullptr);
        near_depths = max_len > 1 ? std::min<uint32_t>(max_len - 1, (uint32_t)kMaxNearDepth) : 0;
        long_off.assign((size_t)near_depths + 2, 0);
        std::vector<uint32_t> short_mask((size_t)std::max<uint32_t>(near_depths, 1) * W, 0u);
        for (uint32_t d = 1; d <= near_depths; ++d) {
            long_off[d] = (uint32_t)long_rank.size();
            for (uint32_t r = 0; r < n_sorted; ++r) {
                if (s_off[r + 1] - s_off[r] > d) long_rank.push_back(r);
                else short_mask[(size_t)(d - 1) * W + (perm[r] >> 5)] |= 1u << (perm[r] & 31);
            }
        }
        long_off[(size_t)near_depths + 1] = (uint32_t)long_rank.size();
        if (long_rank.empty()) long_rank.push_back(0);
        extend_long_bytes();
        d_long_rank.upload(long_rank, nullptr);
        d_short_mask.upload(short_mask, nullptr);
        std::vector<uint8_t> first_byte((size_t)W * 32, 0);
        for (int32_t i = 0; i < V; ++i) if (len(i)) first_byte[(size_t)i] = tok(i)[0];
        d_first_byte.upload(first_byte, nullptr);
        HIP_CHECK(hipStreamSynchronize(nullptr));
        dv.long_rank = d_long_rank.p;
        dv.tok16 = d_tok16.p;
        dv.bytes = d_bytes.p; dv.off = d_off.p; dv.perm = d_perm.p; dv.rank = d_rank.p;
        dv.n_sorted = n_sorted; dv.V = (uint32_t)V; dv.W = W;
        noalloc_host().setup();
        on_device = true;
    }
};

// ---- lowered grammar ---------------------------------------------------------------------------------
struct GrammarImpl {
    Grammar g;
    FlatTables ft;
    std::vector<std::string> rule_names;
};

// ---- large-capacity scratch shared by the slow kernels (one per process; calls are serialised) --------
struct SlowImpl {
    std::mutex mu;
    DevBuf<uint32_t> mem, list;                 // the counter and flag of the list belong to each call's upload
    SlowScratch s{};
    bool ready = false;
    uint32_t k_cap = kSlowK, wm_cap = kSlowWM;  // capacities in use (lowered only by the test hook)
    void ensure() {
        s.k_cap = k_cap; s.wm_cap = wm_cap;
        if (ready) return;
        s.n_lanes = 64 * 64;
        s.list_cap = 1u << 20;
        mem.alloc((size_t)s.n_lanes * kSlowSlots);
        list.alloc((size_t)s.list_cap * 2);
        s.mem = mem.p; s.list = list.p; s.count = nullptr;
        ready = true;
    }
};
SlowImpl& slow() { static SlowImpl* s = new SlowImpl(); return *s; }             // of the fill calls
SlowImpl& build_slow() { static SlowImpl* s = new SlowImpl(); return *s; }       // of the cache builds (which may run beside a fill)
// The library's own stream (default priority) for the builds that fill calls issue just in time.
hipStream_t jit_stream() {
    static hipStream_t s = [] {
        hipStream_t st = nullptr;
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) st = nullptr;
        return st;
    }();
    return s;
}

// ---- cross-grammar pool -------------------------------------------------------------------------------
// A plane is identified by (pool entry of the position's rule, canonical state, pool entry of the
// referencing rule or -1, canonical state the referencing rule continues in or -1).
using PlaneKey = std::array<int64_t, 5>;   // the fifth word: follow signature of the outermost rule (0 = unfiltered)
struct PoolImpl;
// One enqueued cache build.  Compile (and a fill that builds just in time) returns once the kernels are enqueued; whoever
// needs their outcome next (statistics, planes copied to the host, the next compile or fill) finalises the ticket: waits for
// its last event, reads the counters the device copied to pinned memory, and either marks the planes' rows as good
// (noting the ones without uncertain tokens) or, if item sets overflowed even the large-capacity lists, takes the rows
// out of the pool again and fails every cache that uses them.
struct BuildTicket {
    StagingSet* staging = nullptr;
    std::shared_ptr<PoolImpl> pool;
    hipStream_t stream = nullptr;
    std::vector<uint32_t*> rows;                                // the rows being built, with their keys in the pool
    std::vector<PlaneKey> keys;
    std::vector<uint32_t*> borrowed;                            // rows of other planes this build reads: kept from eviction until it is looked at
    int64_t partial_hits = 0;                                   // planes derived from a plane of the same structure
    int64_t executed = 0, executed_bytes = 0;
    double host_ms = 0;
    int state = 0;                                              // 0 enqueued, 1 good, 2 failed
    int64_t slow = 0, n_accepted = 0, n_uncertain = 0;
    float device_ms = 0.f, kernel_ms = 0.f;
    bool timed_kernel = false;                                  // events were recorded around the classification kernel
    ~BuildTicket() { if (staging) { (void)hipEventSynchronize(staging->ev[4]); staging_pool().release(staging); } }
};
// Builds follow one another on the device whatever streams they were given: each waits for the event of the one before
// (they share the large-capacity scratch, and a later one may copy from rows an earlier one writes).
struct BuildChain { std::mutex mu; std::shared_ptr<BuildTicket> last; };
BuildChain& build_chain() { static BuildChain* c = new BuildChain(); return *c; }

struct PoolImpl {
    size_t max_bytes = 0;
    std::mutex mu;
    std::shared_ptr<VocabImpl> vocab;           // bound at first use
    struct Entry { uint64_t hash; std::string text; };
    std::vector<Entry> entries;
    std::unordered_multimap<uint64_t, int> by_hash;
    std::map<PlaneKey, uint32_t*> rows;
    // per structure (the key without its follow signature), one row built under the follow filter: what a plane of the same
    // structure under another follow language is derived from (section 3.3: partial cache hit)
    std::map<std::array<int64_t, 4>, uint32_t*> by_structure;
    std::unordered_set<const uint32_t*> no_uncertain;      // rows whose uncertain plane is all zero (need not be read)
    // bounded-bisimulation classes of interned rules, in canonical state numbers: (entry, token-length budget) -> for
    // canonical state c, the canonical state of its representative
    struct ClassMemo { std::vector<int32_t> rep, base, depth; };            // by canonical state number
    std::map<std::pair<int, int32_t>, ClassMemo> class_memo;
    // rows in use: by how many live caches, and when last taken into a cache.  When max_bytes is reached, rows that no
    // live cache uses are given up, least recently used first, and their memory is handed out again.
    struct RowMeta { PlaneKey key; int32_t refs; uint64_t stamp; };
    std::unordered_map<const uint32_t*, std::shared_ptr<BuildTicket>> building;   // rows whose build has not been finalised
    std::deque<std::shared_ptr<BuildTicket>> pending;                             // tickets not finalised yet, oldest first
    std::unordered_map<const uint32_t*, RowMeta> meta;
    std::vector<uint32_t*> free_rows;
    uint64_t clock = 0;
    int64_t n_evicted = 0;
    struct WordsHash { size_t operator()(const std::vector<uint64_t>& v) const { uint64_t h = 0x9E3779B97F4A7C15ull; for (uint64_t w : v) h = hash_combine(h, w); return (size_t)h; } };
    std::unordered_map<std::vector<uint64_t>, uint64_t, WordsHash> follow_nodes;    // exact interning of follow-language descriptions
    std::unordered_map<int, std::vector<uint64_t>> follow_unfold;   // per interned rule: value of (depth, canonical state), 0 = not known yet
    std::vector<void*> slabs;
    // memory to clear before the next build writes to it: freshly allocated slabs and rows taken from the free list.
    // The build enqueues the fills inside its timed region (skipped tokens rely on the zeros).
    std::vector<std::pair<void*, size_t>> to_zero;
    void flush_zero(hipStream_t stream) {
        for (auto& z : to_zero) HIP_CHECK(hipMemsetAsync(z.first, 0, z.second, stream));
        to_zero.clear();
    }
    uint8_t* slab_cur = nullptr; size_t slab_left = 0;
    size_t device_bytes = 0;
    int64_t n_rows = 0;
    ~PoolImpl() { for (void* s : slabs) (void)hipFree(s); }

    // exact interning: same hash AND same serialisation
    int intern(uint64_t hash, const std::string& text, bool shareable) {
        if (shareable) {
            auto range = by_hash.equal_range(hash);
            for (auto it = range.first; it != range.second; ++it)
                if (entries[(size_t)it->second].text == text) return it->second;
        }
        entries.push_back({hash, shareable ? text : std::string()});
        int id = (int)entries.size() - 1;
        if (shareable) by_hash.emplace(hash, id);
        return id;
    }
    void take(uint32_t* row, const PlaneKey& key) {              // a cache starts using the row
        RowMeta& m = meta[row];
        if (m.refs == 0 && m.stamp == 0) m.key = key;
        ++m.refs;
        m.stamp = ++clock;
    }
    void release(const uint32_t* row) {
        auto it = meta.find(row);
        if (it != meta.end() && it->second.refs > 0) --it->second.refs;
    }
    void forget(uint32_t* row) {                                 // the row's content is void: its memory can be reused
        auto it = meta.find(row);
        if (it != meta.end()) {
            const PlaneKey& k = it->second.key;
            auto bs = by_structure.find({k[0], k[1], k[2], k[3]});
            if (bs != by_structure.end() && bs->second == row) by_structure.erase(bs);
            rows.erase(k); meta.erase(it);
        }
        no_uncertain.erase(row);
        free_rows.push_back(row);
        --n_rows;
    }
    // rows_ahead: how many rows the caller is about to ask for, this one included (sizes a new slab: what is
    // allocated is zeroed by the build that first uses it, so a small build should not pay for a large slab)
    uint32_t* alloc_row(size_t row_bytes, size_t rows_ahead = 1) {
        if (free_rows.empty() && slab_left < row_bytes) {
            size_t want = std::min<size_t>(std::max<size_t>({row_bytes * 64, (size_t)8 << 20, rows_ahead * row_bytes}), (size_t)256 << 20);
            want = std::max(want, row_bytes);
            if (max_bytes && device_bytes + want > max_bytes) want = row_bytes * 16;
            if (max_bytes && device_bytes + want > max_bytes) want = row_bytes;
            if (max_bytes && device_bytes + want > max_bytes) {
                // full: give up the least recently used rows that no live cache uses (a batch, so that the scan is rare)
                std::vector<std::pair<uint64_t, uint32_t*>> idle;
                for (auto& kv : meta) if (kv.second.refs == 0) idle.emplace_back(kv.second.stamp, const_cast<uint32_t*>(kv.first));
                if (idle.empty()) throw std::length_error("cross-grammar pool is full (max_bytes reached and every row is in use)");
                const size_t batch = std::min<size_t>(idle.size(), std::max<size_t>(64, idle.size() / 8));
                std::partial_sort(idle.begin(), idle.begin() + (long)batch, idle.end());
                for (size_t k = 0; k < batch; ++k) { forget(idle[k].second); ++n_evicted; }
            } else {
                void* p = nullptr;
                HIP_CHECK(hipMalloc(&p, want));
                slabs.push_back(p);
                to_zero.emplace_back(p, want);                       // rows are handed out as zeros
                slab_cur = (uint8_t*)p; slab_left = want; device_bytes += want;
            }
        }
        uint32_t* row;
        if (!free_rows.empty()) {
            row = free_rows.back(); free_rows.pop_back();
            to_zero.emplace_back(row, row_bytes);
        } else {
            row = (uint32_t*)slab_cur;
            slab_cur += row_bytes; slab_left -= row_bytes;
        }
        ++n_rows;
        return row;
    }
};

// ---- mask cache -----------------------------------------------------------------------------------------
struct PlaneInfo {
    int32_t rule, state, parent_rule, parent_state;         // the representative it is built for
    uint32_t* row;                                          // accepted row (uncertain at + W words, left early at + 2 W); null until built
    bool no_uncertain;
    PlaneKey key;                                           // identity in the pool
    uint32_t sid; int64_t waiter_sid;                       // start of the build: position, and the waiting parent state or -1
    uint64_t cost;                                          // estimate of the build work (tokens whose first byte the state reads)
    int32_t near_plane = -1, near_depth = 0;                // a plane with the same classes for every token of at most near_depth bytes
    int32_t fb_plane = -1;                                  // a plane with the same classes for every token whose first byte is in fb_same
    std::array<uint32_t, 8> fb_same{};
    int32_t site_plane = -1, site_list = -1;                // the same state under another site: same classes for every token outside that list
};
struct CacheImpl {
    bool follow = true;
    // builds this cache depends on that have not been finalised (its own, and those of other caches it took rows from);
    // the planes that got a row from them; what its own compile build reported; whether one of the builds failed
    std::vector<std::shared_ptr<BuildTicket>> tickets;
    std::vector<int32_t> fresh_planes;
    std::shared_ptr<BuildTicket> compile_ticket;
    bool failed = false;
    bool partial_hits = true;                               // derive planes from planes of the same structure under another follow language
    bool time_kernel = false;                               // record events around the classification kernel (they cost a few microseconds of device time each)
    std::vector<std::shared_ptr<BuildTicket>> jit_tickets;  // builds issued by fill calls whose device time has not been added up yet
    double host_lower_ms = 0;                               // EBNF -> tables and plan, of the compile call
    int64_t compile_built = 0;
    std::vector<uint32_t> site_off, site_tgt;               // per rule: states in which referencing rules continue
    int64_t n_built = 0, jit_calls = 0;                     // planes holding a row; build launches issued by fill
    double jit_device_ms = 0;
    std::shared_ptr<VocabImpl> vocab;
    std::shared_ptr<PoolImpl> pool;
    std::shared_ptr<GrammarImpl> gram;
    uint8_t* d_tables = nullptr;                            // one device block holding all packed tables
    ~CacheImpl();
    DevTables dt{};
    int32_t context_depth = 2;
    std::vector<PlaneInfo> planes;
    // for matchers that live on the device: plane look-up tables and the start state, made at first use
    struct OnDevice {
        std::mutex mu;
        bool ready = false;
        DevBuf<uint64_t> plain_row, pair_row, start_front;
        DevBuf<uint32_t> pair_off, pair_key, start_items, start_wait_off;
        DevBuf<uint2> start_wait;
        CacheDev cd{};
        uint32_t n_start_wait = 0;
    } on_device;
    std::vector<int32_t> plain_plane;                       // [sid] -> plane without context, or -1
    std::unordered_map<uint64_t, int32_t> pair_plane;       // (sid << 32 | parent continuation sid) -> plane
};

struct MatcherImpl {
    std::shared_ptr<CacheImpl> cache;           // null for host-only matchers
    std::shared_ptr<GrammarImpl> gram;
    std::shared_ptr<VocabImpl> vocab;
    EarleyChart chart;
    bool terminated = false;
    // what fill needs from this state, computed once per state (by the batched accept, else by the next fill)
    struct Prep {
        bool valid = false;
        int32_t status = XG2_OK;                             // an error found while preparing, reported by fill
        std::string error;
        ScanContext ctx;
        std::vector<std::pair<int32_t, bool>> planes;        // (plane index, only the accepted row counts)
    } prep;
    MatcherImpl(std::shared_ptr<GrammarImpl> g, std::shared_ptr<VocabImpl> v) : gram(std::move(g)), vocab(std::move(v)), chart(&gram->ft) {
        chart.start(gram->ft.root_start);
    }
};

// ---- fill workspace: pinned staging ring + device mirror ---------------------------------------------------
constexpr uint32_t kUnresolvedCap = 255;                    // (row, token) pairs a fill call can report as undecided
struct FillSlot {
    uint8_t* host = nullptr; uint8_t* dev = nullptr; size_t cap = 0;
    hipEvent_t done = nullptr; bool in_flight = false;
    uint32_t* res_host = nullptr;                           // pinned: {any, more than fit, pairs ...} written by the large-capacity re-check
};
struct MatcherImpl;
struct FillWorkspace {
    std::mutex mu;
    FillSlot slots[4];
    int next = 0;
    DevBuf<uint32_t> cand_words, work_list, row_count;
    hipEvent_t t_begin = nullptr, t_end = nullptr;          // around the device work of the latest fill
    const uint32_t* last_flags = nullptr;                   // device: overflow-list length and flag of the latest fill
    int32_t last_B = 0;                                     // rows of the latest fill
    const uint32_t* last_counts = nullptr;                  // device: their candidate-word counts
    hipStream_t last_stream = nullptr;
    bool timed = false;                                     // the latest fill recorded its events
    bool any = false;                                       // there has been a fill
    // the latest fill whose undecided pairs nobody has looked at yet: its slot and its matchers
    struct Pending { bool active = false; FillSlot* slot = nullptr; std::vector<MatcherImpl*> matchers; } pending;
    // waits for the device work of the latest fill
    void wait_last() {
        if (timed) HIP_CHECK(hipEventSynchronize(t_end));
        else HIP_CHECK(hipStreamSynchronize(last_stream));
    }
    void ensure_scratch(size_t words, size_t rows) {
        if (row_count.n < rows) row_count.alloc(rows * 2);
        if (!t_begin) { HIP_CHECK(hipEventCreate(&t_begin)); HIP_CHECK(hipEventCreate(&t_end)); }
        if (cand_words.n < words) { cand_words.alloc(words * 5 / 4); work_list.alloc(words * 5 / 4); }
    }
    FillSlot& acquire(size_t bytes) {
        FillSlot& s = slots[next];
        next = (next + 1) % 4;
        if (!s.done) HIP_CHECK(hipEventCreateWithFlags(&s.done, hipEventDisableTiming));
        if (!s.res_host) HIP_CHECK(hipHostMalloc((void**)&s.res_host, (2 + 2 * (size_t)kUnresolvedCap) * sizeof(uint32_t), hipHostMallocDefault));
        if (s.in_flight) { HIP_CHECK(hipEventSynchronize(s.done)); s.in_flight = false; }
        if (s.cap < bytes) {
            if (s.host) (void)hipHostFree(s.host);
            if (s.dev) (void)hipFree(s.dev);
            s.cap = std::max(bytes * 2, (size_t)1 << 20);
            HIP_CHECK(hipHostMalloc((void**)&s.host, s.cap, hipHostMallocDefault));
            HIP_CHECK(hipMalloc((void**)&s.dev, s.cap));
        }
        return s;
    }
};
FillWorkspace& fill_ws() { static FillWorkspace* w = new FillWorkspace(); return *w; }

// A fill call returns before its kernels run.  If the large-capacity re-check could not decide some (row, token) pair
// (item sets beyond even its lists), the mask has a 0 where a 1 may belong: the next call that touches matchers or masks
// fails with XG2_EOVERFLOW, once, unless xg2_fill_resolve_overflow has decided the pairs on the host in between.
// The caller holds no lock.
int32_t report_undecided_pairs() {
    FillWorkspace& W = fill_ws();
    std::lock_guard<std::mutex> lk(W.mu);
    if (!W.pending.active) return XG2_OK;
    if (hipEventSynchronize(W.pending.slot->done) != hipSuccess) return XG2_OK;
    W.pending.active = false;
    if (!W.pending.slot->res_host[0]) return XG2_OK;
    uint32_t n = 0;
    while (n < kUnresolvedCap && W.pending.slot->res_host[2 + 2 * n] != 0xFFFFFFFFu) ++n;
    return fail(XG2_EOVERFLOW, "the previous xg2_fill_next_token_bitmask call left " + std::to_string(n) + (W.pending.slot->res_host[1] ? "+" : "") +
                               " (row, token) pairs undecided: their Earley item sets exceed the large-capacity lists, and their mask bits are 0 "
                               "(xg2_fill_resolve_overflow decides them with the host parser)");
}

// A few host threads that stay around between calls (starting threads costs more than the work of a decode step).
// run(parts, job) calls job(0 .. parts - 1), the caller taking shares too, and returns when all are done; calls are
// serialised.  The pool is created at first use and lives until the process ends.
class HostWorkers {
    std::mutex call_mu, mu;
    std::condition_variable cv_work, cv_done;
    std::vector<std::thread> threads;
    const std::function<void(int32_t)>* job = nullptr;
    int32_t n_parts = 0, next = 0, pending = 0;
    void worker() {
        std::unique_lock<std::mutex> lk(mu);
        for (;;) {
            cv_work.wait(lk, [&] { return job && next < n_parts; });
            take(lk);
        }
    }
    void take(std::unique_lock<std::mutex>& lk) {               // runs parts until none is left; lk is held on entry and exit
        while (job && next < n_parts) {
            const int32_t part = next++;
            const std::function<void(int32_t)>* f = job;
            lk.unlock();
            (*f)(part);
            lk.lock();
            if (--pending == 0) { job = nullptr; cv_done.notify_all(); }
        }
    }
  public:
    explicit HostWorkers(int32_t n) { for (int32_t k = 0; k < n; ++k) threads.emplace_back([this] { worker(); }); for (auto& t : threads) t.detach(); }
    int32_t size() const { return (int32_t)threads.size(); }
    void run(int32_t parts, const std::function<void(int32_t)>& f) {
        if (parts <= 0) return;
        std::lock_guard<std::mutex> one_call(call_mu);
        std::unique_lock<std::mutex> lk(mu);
        job = &f; n_parts = parts; next = 0; pending = parts;
        cv_work.notify_all();
        take(lk);
        cv_done.wait(lk, [&] { return pending == 0; });
    }
};
HostWorkers& host_workers() {
    static HostWorkers* w = new HostWorkers(std::max<int32_t>(0, std::min<int32_t>((int32_t)std::thread::hardware_concurrency(), 8) - 1));
    return *w;
}

template <typename F>
int32_t guarded(F&& f) {
    try { return f(); }
    catch (const ParseError& e) { return fail(XG2_EPARSE, e.what()); }
    catch (const GrammarError& e) { return fail(XG2_EINVAL, e.what()); }
    catch (const HipError& e) { return fail(XG2_EHIP, e.what()); }
    catch (const std::length_error& e) { return fail(XG2_EOVERFLOW, e.what()); }
    catch (const std::bad_alloc&) { return fail(XG2_EOVERFLOW, "out of host memory"); }
    catch (const std::exception& e) { return fail(XG2_EINVAL, e.what()); }
}

std::shared_ptr<GrammarImpl> make_grammar(const char* ebnf, size_t len, const char* root) {
    if (!ebnf || !root) throw GrammarError("null grammar text or root rule");
    auto gi = std::make_shared<GrammarImpl>();
    gi->g = lower_grammar(std::string(ebnf, len), root);
    if ((uint32_t)gi->g.n_states + 1 > kSidMask) throw std::length_error("grammar has too many automaton states");
    gi->ft = flatten(gi->g);
    for (auto& r : gi->g.rules) gi->rule_names.push_back(r.name);
    return gi;
}

double ms_since(std::chrono::steady_clock::time_point t0) {
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
}

}  // namespace

struct xg2_vocab { std::shared_ptr<VocabImpl> p; };
struct xg2_grammar { std::shared_ptr<GrammarImpl> p; };
struct xg2_pool { std::shared_ptr<PoolImpl> p; };
struct xg2_mask_cache { std::shared_ptr<CacheImpl> p; };
struct xg2_matcher { std::unique_ptr<MatcherImpl> p; };

// Looks at a finished build.  The caller holds the pool's mutex.
void finalize_ticket(BuildTicket& T) {
    if (T.state) return;
    PoolImpl& pool = *T.pool;
    StagingSet& S = *T.staging;
    hipError_t e = hipEventSynchronize(S.ev[4]);
    bool failed = e != hipSuccess;
    if (!failed) {
        (void)hipEventElapsedTime(&T.device_ms, S.ev[0], S.ev[1]);
        if (T.timed_kernel) (void)hipEventElapsedTime(&T.kernel_ms, S.ev[2], S.ev[3]);
        T.slow = S.res[0];
        failed = S.res[1] != 0;                                     // item sets exceeded even the large-capacity lists
    }
    for (size_t k = 0; k < T.rows.size(); ++k) {
        pool.building.erase(T.rows[k]);
        if (failed) {
            // partial results: nobody may take the row from the pool any more (caches that did are failed through this
            // ticket); its memory is not handed out again while they may still hold it
            auto it = pool.rows.find(T.keys[k]);
            if (it != pool.rows.end() && it->second == T.rows[k]) pool.rows.erase(it);
            continue;
        }
        const uint32_t n_acc = S.res[2 + 2 * k], n_unc = S.res[3 + 2 * k];
        if (n_unc == 0) pool.no_uncertain.insert(T.rows[k]);
        if (T.keys[k][4] != 0) pool.by_structure.emplace(std::array<int64_t, 4>{T.keys[k][0], T.keys[k][1], T.keys[k][2], T.keys[k][3]}, T.rows[k]);
        T.n_accepted += n_acc; T.n_uncertain += n_unc;
    }
    T.state = failed ? 2 : 1;
    for (uint32_t* b : T.borrowed) pool.release(b);
    T.borrowed.clear();
    for (auto it = pool.pending.begin(); it != pool.pending.end(); ++it) if (it->get() == &T) { pool.pending.erase(it); break; }
    {
        std::lock_guard<std::mutex> ck(build_chain().mu);
        staging_pool().release(T.staging);
        T.staging = nullptr;
        if (build_chain().last.get() == &T) build_chain().last.reset();
    }
}

// Finalises every build the cache depends on; afterwards its planes know whether their uncertain rows are empty, and
// cache.failed says whether one of the builds overflowed.  Takes the pool's mutex.
void finalize_cache(CacheImpl& cache) {
    if (cache.tickets.empty() && cache.fresh_planes.empty()) return;
    std::lock_guard<std::mutex> lk(cache.pool->mu);
    for (auto& t : cache.tickets) { finalize_ticket(*t); if (t->state == 2) cache.failed = true; }
    cache.tickets.clear();
    for (int32_t k : cache.fresh_planes) {
        PlaneInfo& pi = cache.planes[(size_t)k];
        pi.no_uncertain = pi.row && cache.pool->no_uncertain.count(pi.row) != 0;
    }
    cache.fresh_planes.clear();
}
int32_t cache_failed() { return fail(XG2_EOVERFLOW, "mask cache build: Earley item sets exceeded the large-capacity limit"); }

CacheImpl::~CacheImpl() {
    if (pool) {
        // its own builds may still be writing: look at them first, so that the pool learns what became of the rows
        try { finalize_cache(*this); } catch (...) {}
        std::lock_guard<std::mutex> lk(pool->mu);
        for (const PlaneInfo& pi : planes) if (pi.row) pool->release(pi.row);
    }
    if (d_tables) (void)hipFree(d_tables);
}

// Enqueues the build of the planes `todo` of a cache that do not hold a row yet: rows the pool already has are taken
// from it, the others are allocated, planned (closed start set, live first-byte ranges, chunks) and classed on the
// device, on `stream`, after the build enqueued before this one.  with_tables: the packed grammar tables travel in the
// same upload and stay with the cache (first call only).  Does not wait: the planes have their rows when the call
// returns, the outcome is looked at by finalize_cache.  The caller holds the pool's mutex and the mutex of the
// large-capacity scratch.  *ticket_out = the build, or null if nothing had to be built.
int32_t build_planes(CacheImpl& cache, const std::vector<int32_t>& todo, hipStream_t stream, bool with_tables, SlowScratch S,
                     std::shared_ptr<BuildTicket>* ticket_out) {
    if (ticket_out) ticket_out->reset();
    auto t1 = std::chrono::steady_clock::now();
    PoolImpl& pool = *cache.pool;
    VocabImpl& V = *cache.vocab;
    const FlatTables& ft = cache.gram->ft;
    const size_t row_bytes = plane_words(V.W) * sizeof(uint32_t);      // accepted, uncertain, left early, list of uncertain tokens
    std::vector<int32_t> build;                                 // plane indices to class now
    std::vector<uint32_t*> build_rows;
    // Until the planes are known to be built, the pool must not offer their rows to anyone: whatever goes wrong
    // on the way (the pool is full, a HIP call fails, the item sets overflow), the rows this call has entered
    // are taken out of the pool again and their memory goes back to the free list.
    struct Rollback {
        PoolImpl& pool; CacheImpl& cache; const std::vector<int32_t>& build; const std::vector<uint32_t*>& rows; hipStream_t stream;
        bool armed = true;
        ~Rollback() {
            if (!armed) return;
            (void)hipStreamSynchronize(stream);                  // no kernel of this call writes to the rows any more
            for (size_t k = 0; k < build.size(); ++k) {
                auto it = pool.rows.find(cache.planes[(size_t)build[k]].key);
                if (it != pool.rows.end() && it->second == rows[k]) pool.rows.erase(it);
                pool.free_rows.push_back(rows[k]);
                --pool.n_rows;
            }
        }
    } rollback{pool, cache, build, build_rows, stream};
    struct ReleaseBorrowed {                                     // rows borrowed for a partial hit go back if the build is not enqueued
        PoolImpl& pool; std::vector<uint32_t*>* rows = nullptr; bool armed = true;
        ~ReleaseBorrowed() { if (armed && rows) for (uint32_t* r : *rows) pool.release(r); }
    } release_borrowed{pool};
    for (size_t i = 0; i < todo.size(); ++i) {
        const int32_t k = todo[i];
        PlaneInfo& pi = cache.planes[(size_t)k];
        if (pi.row) continue;
        auto have = pool.rows.find(pi.key);
        if (have != pool.rows.end()) {                           // another grammar built it, or is building it
            uint32_t* row = have->second;
            pi.row = row; pi.no_uncertain = pool.no_uncertain.count(row) != 0; pool.take(row, pi.key); ++cache.n_built;
            auto bt = pool.building.find(row);
            if (bt != pool.building.end()) {
                if (std::find(cache.tickets.begin(), cache.tickets.end(), bt->second) == cache.tickets.end()) cache.tickets.push_back(bt->second);
                cache.fresh_planes.push_back(k);
            }
            continue;
        }
        uint32_t* row = pool.alloc_row(row_bytes, todo.size() - i);
        build.push_back(k);
        build_rows.push_back(row);
        pool.rows.emplace(pi.key, row);
    }
    if (build.empty() && !with_tables) { rollback.armed = false; return XG2_OK; }
    // keep the number of builds nobody has looked at small: finished ones are finalised on the way, the oldest is waited for
    while (!pool.pending.empty() && (pool.pending.size() > 6 || hipEventQuery(pool.pending.front()->staging->ev[4]) == hipSuccess))
        finalize_ticket(*std::shared_ptr<BuildTicket>(pool.pending.front()));
    auto ticket = std::make_shared<BuildTicket>();
    ticket->pool = cache.pool;
    ticket->stream = stream;
    ticket->staging = staging_pool().acquire();
    StagingSet& SS = *ticket->staging;

    // plan: closed start set and live first-byte ranges of every plane to build
    std::vector<uint32_t> ctx_items, ctx_wait, ctx_wait_off;
    std::vector<uint4> plane_ctx, ranges;
    std::vector<CopyJob> copies, structure_copies;
    std::vector<FirstByteCopyJob> fb_copies;
    std::vector<uint64_t> derive_base(build.size(), 0);          // partial hits: address of the base plane's left-early row
    std::vector<uint32_t*> borrowed;
    release_borrowed.rows = &borrowed;
    int64_t executed = 0, executed_bytes = 0;
    EarleyChart chart(&ft);
    std::map<int32_t, size_t> building;                         // plane index -> position in build
    for (size_t k = 0; k < build.size(); ++k) building.emplace(build[k], k);
    for (size_t k = 0; k < build.size(); ++k) {
        const PlaneInfo& pi = cache.planes[(size_t)build[k]];
        // Partial cache hit (section 3.3): the pool holds a plane of the same structure built under another follow language.
        // Accepted tokens, and the tokens that leave the rule early and die, are the same; only which of the latter stay
        // uncertain depends on what may follow: those are run again, in follow mode, and nothing else is.
        if (cache.follow && cache.partial_hits && pi.key[4] != 0) {
            auto bs = pool.by_structure.find({pi.key[0], pi.key[1], pi.key[2], pi.key[3]});
            if (bs != pool.by_structure.end() && bs->second != build_rows[k]) {
                uint32_t* base = bs->second;
                pool.take(base, pi.key);                         // not to be evicted while this build reads it
                borrowed.push_back(base);
                structure_copies.push_back({build_rows[k], base, nullptr, 0});
                derive_base[k] = (uint64_t)(uintptr_t)(base + 2 * (size_t)V.W);
            }
        }
        const bool derived = derive_base[k] != 0;
        // short tokens from a plane that agrees on them, if that plane is there or is being built in this call
        uint32_t near_d = 0;
        if (!derived && pi.near_plane >= 0 && pi.near_depth >= 1 && V.near_depths >= 1) {
            const uint32_t* src = cache.planes[(size_t)pi.near_plane].row;
            if (!src) {
                auto pr = pool.rows.find(cache.planes[(size_t)pi.near_plane].key);
                auto bi = building.find(pi.near_plane);
                if (bi != building.end()) src = build_rows[bi->second];
                else if (pr != pool.rows.end() && pr->second) src = pr->second;
            }
            if (src) {
                near_d = std::min<uint32_t>((uint32_t)pi.near_depth, V.near_depths);
                copies.push_back({build_rows[k], src, V.d_short_mask.p + (size_t)(near_d - 1) * V.W, 0});
            }
        }
        // or the tokens with most first bytes from the plane of the rule's start state, under the same conditions
        bool by_first_byte = false;
        if (!derived && !near_d && pi.fb_plane >= 0) {
            const uint32_t* src = cache.planes[(size_t)pi.fb_plane].row;
            if (!src) {
                auto pr = pool.rows.find(cache.planes[(size_t)pi.fb_plane].key);
                auto bi = building.find(pi.fb_plane);
                if (bi != building.end()) src = build_rows[bi->second];
                else if (pr != pool.rows.end() && pr->second) src = pr->second;
            }
            if (src) {
                FirstByteCopyJob job{build_rows[k], src, {}};
                for (int w = 0; w < 8; ++w) job.bytes[w] = pi.fb_same[(size_t)w];
                fb_copies.push_back(job);
                by_first_byte = true;
            }
        }
        // or every token that cannot leave the plain states of the rule from the plane of the same state under another site
        const VocabImpl::ByteSetList* by_list = nullptr;
        if (!derived && !near_d && !by_first_byte && pi.site_plane >= 0) {
            const uint32_t* src = cache.planes[(size_t)pi.site_plane].row;
            if (!src) {
                auto pr = pool.rows.find(cache.planes[(size_t)pi.site_plane].key);
                auto bi = building.find(pi.site_plane);
                if (bi != building.end()) src = build_rows[bi->second];
                else if (pr != pool.rows.end() && pr->second) src = pr->second;
            }
            if (src) {
                by_list = &V.byte_lists[(size_t)pi.site_list];
                copies.push_back({build_rows[k], src, by_list->d_without->p, 0});
            }
        }
        if (pi.waiter_sid < 0) chart.start(pi.sid);
        else chart.start_pair(pi.sid, (uint32_t)pi.waiter_sid);
        const std::vector<ChartSet>& sets = chart.sets();
        auto loc = [](int32_t o) { return o < 0 ? kRootOrigin : (uint32_t)o; };
        bool live[257] = {false};
        const uint32_t item0 = (uint32_t)ctx_items.size();
        for (const ChartItem& it : sets.back().scan) {
            ctx_items.push_back(pack_item(ft.ref(it.sid), loc(it.origin)));
            const StateInfo& si = ft.state_info[it.sid];
            for (uint32_t e = 0; e < (si.counts & 0xFFFF); ++e) {
                const ByteEdge& be = ft.byte_edges[si.byte_off + e];
                for (uint32_t b = be.lohi & 0xFF; b <= ((be.lohi >> 8) & 0xFF); ++b) live[b] = true;
            }
        }
        plane_ctx.push_back(make_uint4(item0, (uint32_t)ctx_items.size() - item0, (uint32_t)ctx_wait_off.size(), (uint32_t)sets.size()));
        // a start set that is one item with byte edges only is walked as a plain automaton; the others need the
        // Earley steps from the first byte on and go first, so that the long workgroups do not end the launch
        const uint32_t heavy = (ctx_items.size() - item0 == 1 && (ctx_items[item0] & (kHasByte | kHasRef)) == kHasByte) ? 0u : 1u;
        for (const ChartSet& cs : sets) {
            ctx_wait_off.push_back((uint32_t)(ctx_wait.size() / 2));
            for (const ChartItem& it : cs.wait) chart.push_triples(it, loc(it.origin), ctx_wait);
        }
        ctx_wait_off.push_back((uint32_t)(ctx_wait.size() / 2));
        // A start set of at most two items that scan, none of them predicting, where the end of a waited-for instance
        // leads to one state of the outermost instance that does not predict either, is walked as a few automaton
        // threads; the two items and what each one's end leads to follow the plane's items.
        uint32_t threads = 0;
        if (heavy) {
            uint32_t desc[4] = {kNoThread, 0u, kNoThread, 0u};
            uint32_t nb = 0;
            bool ok = true;
            for (size_t q = item0; q < item0 + plane_ctx.back().y && ok; ++q) {
                const uint32_t it = ctx_items[q];
                if (!(it & kHasByte)) continue;
                if ((it & kHasRef) || nb == 2) { ok = false; break; }
                uint32_t lead = 0;
                const uint32_t origin = it >> kRefBits;
                if (origin != kRootOrigin) {
                    const uint32_t rule = ft.state_info[it & kSidMask].rule_final & 0x7FFFFFFFu;
                    const uint32_t w0 = ctx_wait_off[plane_ctx.back().z + origin], w1 = ctx_wait_off[plane_ctx.back().z + origin + 1];
                    uint32_t n_lead = 0;
                    for (uint32_t w = w0; w < w1; ++w)
                        if (ctx_wait[2 * (size_t)w] == rule) { ++n_lead; lead = ctx_wait[2 * (size_t)w + 1]; }
                    ok = n_lead == 1 && !(lead & kHasRef) && (lead >> kRefBits) == kRootOrigin;
                }
                desc[2 * nb] = it; desc[2 * nb + 1] = lead;
                ++nb;
            }
            if (ok && nb) {
                ctx_items.insert(ctx_items.end(), desc, desc + 4);
                threads = kChunkThreads;
            }
        }
        if (derived) {
            ranges.push_back(make_uint4((uint32_t)k, 0u, V.W, kChunkDerive | kChunkHeavy));
            continue;
        }
        if (by_first_byte) for (int b = 0; b < 256; ++b) if ((pi.fb_same[(size_t)b >> 5] >> (b & 31)) & 1u) live[b] = false;
        for (int b = 0; b < 256;) {
            if (!live[b]) { ++b; continue; }
            int e = b;
            while (live[e + 1]) ++e;
            uint32_t lo = V.fb_start[b], hi = V.fb_start[e + 1], listed = 0;
            if (near_d || by_list) {                                 // the same ranks, in the list of the tokens longer than near_d / with such bytes
                const uint32_t* first = V.long_rank.data() + (near_d ? V.long_off[near_d] : by_list->off);
                const uint32_t* last = V.long_rank.data() + (near_d ? V.long_off[near_d + 1] : by_list->off + by_list->n);
                lo = (uint32_t)(std::lower_bound(first, last, lo) - V.long_rank.data());
                hi = (uint32_t)(std::lower_bound(first, last, hi) - V.long_rank.data());
                listed = kChunkListed;
            }
            if (lo < hi) ranges.push_back(make_uint4((uint32_t)k, lo, hi, listed | threads | (heavy ? kChunkHeavy : 0u)));
            executed += hi - lo;
            executed_bytes += listed ? (int64_t)(V.long_bytes[hi] - V.long_bytes[lo]) : (int64_t)(V.s_off[hi] - V.s_off[lo]);
            b = e + 1;
        }
    }
    // The copies of derived planes and the per-plane summary go in one pass over the planes when no plane takes bits from
    // a plane that itself takes bits in this build (the separate kernels order such chains: masked copies, then
    // first-byte copies, then the summary).
    std::vector<FinishJob> finish(build_rows.size(), FinishJob{});
    bool finish_in_one = !build_rows.empty() && build_fusion().load();
    {
        std::map<const uint32_t*, size_t> at;
        for (size_t k = 0; k < build_rows.size(); ++k) at.emplace(build_rows[k], k);
        std::set<const uint32_t*> takes;
        for (const CopyJob& j : copies) takes.insert(j.dst);
        for (const FirstByteCopyJob& j : fb_copies) takes.insert(j.dst);
        for (const CopyJob& j : copies) {
            FinishJob& f = finish[at.at(j.dst)];
            if (f.m_src || takes.count(j.src)) finish_in_one = false;
            f.m_src = j.src; f.m_mask = j.mask;
        }
        for (const FirstByteCopyJob& j : fb_copies) {
            FinishJob& f = finish[at.at(j.dst)];
            if (f.f_src || takes.count(j.src)) finish_in_one = false;
            f.f_src = j.src;
            for (int w = 0; w < 8; ++w) f.f_bytes[w] = j.bytes[w];
        }
    }
    // The chunk records are written on the device (k_expand_chunks) from the ranges: per range {plane, first rank, end
    // rank, flags}, the index of its first chunk and what the walk needs of its plane.  Chunks of the heavy ranges come
    // first, then the others, each group in plane order; a long range is cut so that one thread writes at most 32 chunks.
    std::vector<uint4> range_a, range_b;
    std::vector<uint32_t> range_first;
    size_t n_chunks = 0;
    for (uint32_t pass_heavy : {kChunkHeavy, 0u})
        for (const uint4& r : ranges) {
            if ((r.w & kChunkHeavy) != pass_heavy) continue;
            const bool derive = r.w & kChunkDerive;
            const uint32_t step = derive ? kDeriveChunk : pass_heavy ? kHeavyChunk : kBuildChunk;
            const uint4& pc = plane_ctx[r.x];
            const uint64_t row = derive ? derive_base[r.x] : (uint64_t)(uintptr_t)build_rows[r.x];
            const uint4 second = derive ? make_uint4(0u, 0u, (uint32_t)row, (uint32_t)(row >> 32))
                                        : make_uint4(ctx_items[pc.x], pc.y, (uint32_t)row, (uint32_t)(row >> 32));
            for (uint32_t lo = r.y; lo < r.z; lo += 32 * step) {
                const uint32_t hi = std::min(r.z, lo + 32 * step);
                range_a.push_back(make_uint4(r.x, lo, hi, r.w));
                range_b.push_back(second);
                range_first.push_back((uint32_t)n_chunks);
                n_chunks += (hi - lo + step - 1) / step;
            }
        }
    if (n_chunks > 0xFFFFFFF0ull) throw std::length_error("mask cache build: too many chunks in one launch");

    // everything the device needs goes up in one copy: (the tables,) the plan, and a few zeroed words (overflow
    // counter and flag, bit counts per built plane).  With the tables the block stays with the cache.
    std::vector<uint32_t> zeros(8 + 2 * build_rows.size(), 0u);
    Packer tab;
    size_t o_state = 0, o_exp = 0, o_soff = 0, o_stgt = 0, o_trans = 0, o_cls = 0;
    if (with_tables) {
        o_state = tab.add(ft.dev_state); o_exp = tab.add(ft.exp_list); o_soff = tab.add(cache.site_off); o_stgt = tab.add(cache.site_tgt);
        o_trans = tab.add(ft.trans); o_cls = tab.add(ft.byte_class_words);
    }
    const size_t o_range_a = tab.add(range_a), o_range_b = tab.add(range_b), o_range_first = tab.add(range_first), o_pctx = tab.add(plane_ctx), o_items = tab.add(ctx_items), o_wait = tab.add(ctx_wait),
                 o_wait_off = tab.add(ctx_wait_off), o_rows = tab.add(build_rows), o_copies = tab.add(copies), o_structure_copies = tab.add(structure_copies), o_fb_copies = tab.add(fb_copies), o_finish = tab.add(finish), o_zero = tab.add(zeros);
    const size_t o_chunks = tab.reserve(n_chunks * 2 * sizeof(uint4));
    tab.stage(with_tables, SS);
    if (with_tables) cache.d_tables = tab.dev;                     // the cache owns the block from here on
    ticket->host_ms = ms_since(t1);

    SS.ensure_events();
    SS.ensure_res(2 + 2 * build_rows.size());
    const hipEvent_t ev0 = SS.ev[0], ev1 = SS.ev[1], evk0 = SS.ev[2], evk1 = SS.ev[3];
    {
        // after the build enqueued before this one, whatever its stream
        std::lock_guard<std::mutex> ck(build_chain().mu);
        std::shared_ptr<BuildTicket>& last = build_chain().last;
        if (last && last->state == 0 && last->staging && last->stream != stream) HIP_CHECK(hipStreamWaitEvent(stream, last->staging->ev[4], 0));
    }
    HIP_CHECK(hipEventRecord(ev0, stream));
    // The rows start as zeros (tokens skipped by their first byte are never written), the plan goes up and the chunk
    // records are written: one launch when the upload is small enough for a copy kernel and the pool has few ranges to
    // clear (a fresh slab, a few recycled rows), else one call each.
    bool staged = false;
    if (build_fusion().load() && tab.total <= kUploadByKernelMax && pool.to_zero.size() <= kStageZeroRanges) {
        StageZero Z{};
        bool ok = true;
        for (auto& z : pool.to_zero) {
            if (z.second % 4) { ok = false; break; }
            Z.p[Z.n] = static_cast<uint32_t*>(z.first); Z.words[Z.n] = z.second / 4; ++Z.n;
        }
        if (ok) {
            void* mapped = nullptr;
            HIP_CHECK(hipHostGetDevicePointer(&mapped, tab.host, 0));
            const uint8_t* hm = static_cast<const uint8_t*>(mapped);
            launch_stage(tab.dev, mapped, tab.total, Z, reinterpret_cast<const uint4*>(hm + o_range_a), reinterpret_cast<const uint4*>(hm + o_range_b),
                         reinterpret_cast<const uint32_t*>(hm + o_range_first), (uint32_t)range_a.size(), tab.at<uint4>(o_chunks), stream);
            pool.to_zero.clear();
            staged = true;
        }
    }
    if (!staged) {
        pool.flush_zero(stream);
        tab.copy(stream);
    }
    if (with_tables) {
        cache.dt.state = tab.at<const uint4>(o_state);
        cache.dt.exp_list = tab.at<const uint32_t>(o_exp);
        cache.dt.trans = tab.at<const uint32_t>(o_trans);
        cache.dt.byte_class_words = tab.at<const uint32_t>(o_cls);
        cache.dt.n_classes = ft.n_classes;
        cache.dt.sink = ft.sink;
        cache.dt.site_off = tab.at<const uint32_t>(o_soff);
        cache.dt.site_tgt = tab.at<const uint32_t>(o_stgt);
    }
    uint32_t* d_counts = tab.at<uint32_t>(o_zero) + 8;
    S.count = tab.at<uint32_t>(o_zero) + 4;                       // this call's own overflow counter and flag, zero on arrival
    BuildPlan P{};
    P.chunk = tab.at<const uint4>(o_chunks); P.n_chunks = (uint32_t)n_chunks;
    P.plane_ctx = tab.at<const uint4>(o_pctx);
    P.ctx_items = tab.at<const uint32_t>(o_items);
    P.ctx_wait = tab.at<const uint2>(o_wait); P.ctx_wait_off = tab.at<const uint32_t>(o_wait_off);
    P.plane_ptr = tab.at<uint32_t*>(o_rows);
    P.follow_filter = cache.follow ? 1u : 0u;
    uint32_t* const* d_rows_p = tab.at<uint32_t*>(o_rows);
    if (!staged)
        launch_expand_chunks(tab.at<const uint4>(o_range_a), tab.at<const uint4>(o_range_b), tab.at<const uint32_t>(o_range_first),
                             (uint32_t)range_a.size(), tab.at<uint4>(o_chunks), stream);
    ticket->timed_kernel = cache.time_kernel;
    if (cache.time_kernel) HIP_CHECK(hipEventRecord(evk0, stream));
    if (!build.empty()) launch_build(cache.dt, V.dv, P, S, stream);
    if (cache.time_kernel) HIP_CHECK(hipEventRecord(evk1, stream));
    if (!build.empty()) launch_build_slow(cache.dt, V.dv, P, S, stream);
    launch_copy_structure(tab.at<const CopyJob>(o_structure_copies), (uint32_t)structure_copies.size(), V.W, stream);
    if (finish_in_one) {
        launch_finish_planes(d_rows_p, tab.at<const FinishJob>(o_finish), (uint32_t)build_rows.size(), V.d_first_byte.p, V.W, d_counts, stream);
    } else {
        launch_copy_masked(tab.at<const CopyJob>(o_copies), (uint32_t)copies.size(), V.W, stream);
        launch_copy_first_byte(tab.at<const FirstByteCopyJob>(o_fb_copies), (uint32_t)fb_copies.size(), V.d_first_byte.p, V.W, stream);
        if (!build.empty()) launch_plane_summary(d_rows_p, (uint32_t)build_rows.size(), V.W, d_counts, stream);   // statistics, lists of uncertain tokens
    }
    HIP_CHECK(hipEventRecord(ev1, stream));                              // every plane is written, with its list of uncertain tokens
    HIP_CHECK(hipMemcpyAsync(SS.res, S.count, 2 * sizeof(uint32_t), hipMemcpyDeviceToHost, stream));
    if (!build_rows.empty()) HIP_CHECK(hipMemcpyAsync(SS.res + 2, d_counts, 2 * build_rows.size() * sizeof(uint32_t), hipMemcpyDeviceToHost, stream));
    HIP_CHECK(hipEventRecord(SS.ev[4], stream));
    HIP_CHECK(hipGetLastError());
    // from here on the build is under way: the planes have their rows, the ticket says what became of them
    rollback.armed = false;
    ticket->rows = build_rows;
    ticket->borrowed = borrowed;
    release_borrowed.armed = false;
    ticket->partial_hits = (int64_t)structure_copies.size();
    ticket->executed = executed; ticket->executed_bytes = executed_bytes;
    for (size_t k = 0; k < build.size(); ++k) {
        PlaneInfo& pi = cache.planes[(size_t)build[k]];
        pi.row = build_rows[k];
        pi.no_uncertain = false;                                    // not known yet
        pool.take(pi.row, pi.key);
        pool.building.emplace(pi.row, ticket);
        ticket->keys.push_back(pi.key);
        cache.fresh_planes.push_back(build[k]);
    }
    cache.n_built += (int64_t)build.size();
    cache.tickets.push_back(ticket);
    pool.pending.push_back(ticket);
    { std::lock_guard<std::mutex> ck(build_chain().mu); build_chain().last = ticket; }
    if (ticket_out) *ticket_out = ticket;
    return XG2_OK;
}

// Calls visit(plane index, accepted_only) for every plane the scannable frontier of a matcher needs: the plain plane
// of items of the root instance (or of every item at context depth 1), else one plane per waiting parent of the item.
template <class F>
int32_t for_frontier_planes(const MatcherImpl& M, F&& visit) {
    const Grammar& G = M.gram->g;
    const FlatTables& FT = M.gram->ft;
    for (const ChartItem& it : M.chart.last().scan) {
        if (G.sid_to_pos[it.sid] < 0) continue;                         // nothing to scan from this item
        if (it.origin < 0 || M.cache->context_depth == 1) {
            // the root instance: leaving the rule leaves the grammar, so uncertain tokens are never allowed
            int32_t plane = M.cache->plain_plane[it.sid];
            if (plane < 0) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: frontier item without a plane");
            visit(plane, it.origin < 0);
            continue;
        }
        const uint32_t rule = FT.state_info[it.sid].rule_final & 0x7FFFFFFFu;
        bool any_parent = false;
        for (const ChartItem& w : M.chart.sets()[(size_t)it.origin].wait) {
            const StateInfo& wi = FT.state_info[w.sid];
            for (uint32_t k = 0; k < (wi.counts >> 16); ++k) {
                const RefEdgeP& e = FT.ref_edges[wi.ref_off + k];
                if (e.rule != rule) continue;
                auto pp = M.cache->pair_plane.find(((uint64_t)it.sid << 32) | e.tgt);
                if (pp == M.cache->pair_plane.end()) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: frontier item without a plane");
                visit(pp->second, false);
                any_parent = true;
            }
        }
        if (!any_parent) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: frontier item without a referencing item");
    }
    return XG2_OK;
}

// The fill-side view of a matcher's current state: scan context and the planes of its frontier.
void prepare_matcher(MatcherImpl& M) {
    MatcherImpl::Prep& P = M.prep;
    if (P.valid || !M.cache) return;
    P.status = XG2_OK;
    P.planes.clear();
    if (!M.terminated) {
        if (!M.chart.context(P.ctx)) { P.status = XG2_EOVERFLOW; P.error = "xg2_fill_next_token_bitmask: parser context too deep"; }
        else {
            P.status = for_frontier_planes(M, [&](int32_t plane, bool accepted_only) {
                for (auto& pl : P.planes) if (pl.first == plane) { pl.second = pl.second && accepted_only; return; }
                P.planes.emplace_back(plane, accepted_only);
            });
            if (P.status != XG2_OK) P.error = g_error;
        }
    }
    P.valid = true;
}

// ---- matchers on the device -----------------------------------------------------------------------------------
struct BatchImpl {
    static constexpr uint32_t KI = kSlotItems, KH = kSlotSets, KW = kSlotWaits, KF = kSlotPlanes, kMaxCaches = 256;
    std::mutex mu;
    std::shared_ptr<VocabImpl> vocab;
    int32_t B = 0;
    BatchDev d{};
    DevBuf<FillRow> rows;
    DevBuf<uint64_t> front, slow_front;
    DevBuf<uint32_t> items, wait_off, slow_mem, flag_words;
    int flag_turn = 0;                                      // which half of flag_words the next fill counts in
    DevBuf<uint2> wait;
    DevBuf<uint8_t> slow_map;
    DevBuf<CacheDev> caches_dev;
    DevBuf<DevTables> tables_dev;
    DevBuf<int32_t> row_list;
    std::vector<std::shared_ptr<CacheImpl>> caches;
    std::vector<uint8_t> assigned;
    int32_t n_assigned = 0;
};

struct xg2_batch { std::unique_ptr<BatchImpl> p; };

// Plane look-up tables and start state of a fully built cache, on the device.
void ensure_cache_on_device(const std::shared_ptr<CacheImpl>& cp) {
    CacheImpl& C = *cp;
    std::lock_guard<std::mutex> lk(C.on_device.mu);
    if (C.on_device.ready) return;
    finalize_cache(C);
    if (C.failed) throw std::length_error("mask cache build: Earley item sets exceeded the large-capacity limit");
    if (C.n_built != (int64_t)C.planes.size())
        throw GrammarError("matchers on the device need a fully built mask cache (this one was compiled just in time)");
    CacheImpl::OnDevice& D = C.on_device;
    const size_t n_states = (size_t)C.gram->g.n_states;
    auto row_word = [&](int32_t plane, bool accepted_only) {
        const PlaneInfo& pi = C.planes[(size_t)plane];
        return (uint64_t)(uintptr_t)pi.row | ((accepted_only || pi.no_uncertain) ? 1u : 0u);
    };
    std::vector<uint64_t> plain(n_states, 0);
    for (size_t sid = 0; sid < n_states; ++sid) if (C.plain_plane[sid] >= 0) plain[sid] = row_word(C.plain_plane[sid], false);
    std::vector<std::array<uint64_t, 3>> pairs;                 // (state, state the referencing rule continues in, row)
    pairs.reserve(C.pair_plane.size());
    for (auto& kv : C.pair_plane) pairs.push_back({kv.first >> 32, kv.first & 0xFFFFFFFFull, row_word(kv.second, false)});
    std::sort(pairs.begin(), pairs.end());
    std::vector<uint32_t> pair_off(n_states + 1, 0), pair_key(std::max<size_t>(pairs.size(), 1), 0);
    std::vector<uint64_t> pair_row(std::max<size_t>(pairs.size(), 1), 0);
    for (size_t k = 0; k < pairs.size(); ++k) { ++pair_off[(size_t)pairs[k][0] + 1]; pair_key[k] = (uint32_t)pairs[k][1]; pair_row[k] = pairs[k][2]; }
    for (size_t sid = 0; sid < n_states; ++sid) pair_off[sid + 1] += pair_off[sid];
    // the start state, through the host parser
    MatcherImpl M(C.gram, C.vocab);
    M.cache = cp;
    prepare_matcher(M);
    if (M.prep.status != XG2_OK) throw GrammarError(M.prep.error);
    std::vector<uint32_t> s_items;
    for (uint32_t it : M.prep.ctx.items) if (it & kHasByte) s_items.push_back(it);
    std::vector<uint64_t> s_front;
    for (auto& pl : M.prep.planes) {
        const uint64_t w = row_word(pl.first, pl.second);
        bool seen = false;
        for (uint64_t& have : s_front) if ((have & ~(uint64_t)1) == (w & ~(uint64_t)1)) { have &= w | ~(uint64_t)1; seen = true; }
        if (!seen) s_front.push_back(w);
    }
    std::vector<uint2> s_wait(M.prep.ctx.wait.size() / 2);
    for (size_t k = 0; k < s_wait.size(); ++k) s_wait[k] = make_uint2(M.prep.ctx.wait[2 * k], M.prep.ctx.wait[2 * k + 1]);
    D.plain_row.upload(plain, nullptr); D.pair_off.upload(pair_off, nullptr); D.pair_key.upload(pair_key, nullptr); D.pair_row.upload(pair_row, nullptr);
    D.start_items.upload(s_items, nullptr); D.start_front.upload(s_front, nullptr); D.start_wait.upload(s_wait, nullptr);
    D.start_wait_off.upload(M.prep.ctx.wait_off, nullptr);
    HIP_CHECK(hipStreamSynchronize(nullptr));
    D.cd.T = C.dt;
    D.cd.plain_row = D.plain_row.p; D.cd.pair_off = D.pair_off.p; D.cd.pair_key = D.pair_key.p; D.cd.pair_row = D.pair_row.p;
    D.cd.context_depth = (uint32_t)C.context_depth;
    D.cd.start_n_items = (uint32_t)s_items.size(); D.cd.start_H = M.prep.ctx.H; D.cd.start_n_front = (uint32_t)s_front.size();
    D.cd.start_flags = M.chart.last().root_done ? 1u : 0u;
    D.cd.start_items = D.start_items.p; D.cd.start_wait = D.start_wait.p; D.cd.start_wait_off = D.start_wait_off.p; D.cd.start_front = D.start_front.p;
    D.n_start_wait = (uint32_t)s_wait.size();
    D.ready = true;
}

extern "C" {

const char* xg2_last_error(void) { return g_error.c_str(); }

int32_t xg2_vocab_create(const uint8_t* bytes, const uint64_t* offsets, int32_t V, int32_t eos_id,
                         const int32_t* special_ids, int32_t n_special, xg2_vocab** out) {
    return guarded([&]() -> int32_t {
        if (!offsets || !out || V <= 0 || eos_id < 0 || eos_id >= V || n_special < 0 || (n_special > 0 && !special_ids))
            return fail(XG2_EINVAL, "xg2_vocab_create: bad argument");
        for (int32_t i = 0; i < V; ++i) if (offsets[i + 1] < offsets[i]) return fail(XG2_EINVAL, "xg2_vocab_create: offsets not monotone");
        if (offsets[V] > offsets[0] && !bytes) return fail(XG2_EINVAL, "xg2_vocab_create: null bytes");
        if (offsets[V] - offsets[0] > 0xFFFFFFF0ull) return fail(XG2_EOVERFLOW, "xg2_vocab_create: vocabulary bytes exceed 4 GiB");
        auto v = std::make_shared<VocabImpl>();
        v->V = V; v->eos = eos_id; v->W = ((uint32_t)V + 31) / 32;
        v->offs.resize((size_t)V + 1);
        for (int32_t i = 0; i <= V; ++i) v->offs[(size_t)i] = offsets[i] - offsets[0];
        v->bytes.assign(bytes + offsets[0], bytes + offsets[V]);
        v->special.assign((size_t)V, 0);
        v->special[(size_t)eos_id] = 1;
        for (int32_t k = 0; k < n_special; ++k) {
            if (special_ids[k] < 0 || special_ids[k] >= V) return fail(XG2_EINVAL, "xg2_vocab_create: special id out of range");
            v->special[(size_t)special_ids[k]] = 1;
        }
        for (int32_t i = 0; i < V; ++i) if (v->len(i) == 0) v->special[(size_t)i] = 1;
        for (int32_t i = 0; i < V; ++i) if (!v->special[(size_t)i]) v->perm.push_back((uint32_t)i);
        std::sort(v->perm.begin(), v->perm.end(), [&](uint32_t a, uint32_t b) {
            // by first byte (whole ranges of it are skipped per plane), then by length (a wavefront's 64 lanes
            // run as long as its longest token), then by bytes (neighbours share prefixes)
            size_t la = v->len((int32_t)a), lb = v->len((int32_t)b);
            const uint8_t* ta = v->tok((int32_t)a);
            const uint8_t* tb = v->tok((int32_t)b);
            if (ta[0] != tb[0]) return ta[0] < tb[0];
            if (la != lb) return la < lb;
            int c = std::memcmp(ta, tb, la);
            if (c != 0) return c < 0;
            return a < b;
        });
        v->n_sorted = (uint32_t)v->perm.size();
        v->rank.assign((size_t)V, 0xFFFFFFFFu);
        v->s_off.push_back(0);
        for (uint32_t r = 0; r < v->n_sorted; ++r) {
            int32_t id = (int32_t)v->perm[r];
            v->rank[(size_t)id] = r;
            v->s_bytes.insert(v->s_bytes.end(), v->tok(id), v->tok(id) + v->len(id));
            v->s_off.push_back((uint32_t)v->s_bytes.size());
            v->max_len = std::max<uint32_t>(v->max_len, (uint32_t)v->len(id));
        }
        uint32_t r = 0;
        for (int b = 0; b <= 256; ++b) {
            while (r < v->n_sorted && (int)v->s_bytes[v->s_off[r]] < b) ++r;
            v->fb_start[b] = r;
        }
        *out = new xg2_vocab{v};
        return XG2_OK;
    });
}
void xg2_vocab_destroy(xg2_vocab* v) { delete v; }

int32_t xg2_grammar_create(const char* ebnf, size_t len, const char* root_rule, xg2_grammar** out) {
    return guarded([&]() -> int32_t {
        if (!out) return fail(XG2_EINVAL, "xg2_grammar_create: null out");
        *out = new xg2_grammar{make_grammar(ebnf, len, root_rule)};
        return XG2_OK;
    });
}
void xg2_grammar_destroy(xg2_grammar* g) { delete g; }

int32_t xg2_grammar_describe(const xg2_grammar* g, char* buf, size_t cap, size_t* needed) {
    return guarded([&]() -> int32_t {
        if (!g || !needed) return fail(XG2_EINVAL, "xg2_grammar_describe: bad argument");
        std::string s = describe_grammar(g->p->g);
        *needed = s.size() + 1;
        if (buf && cap) { size_t n = std::min(cap - 1, s.size()); std::memcpy(buf, s.data(), n); buf[n] = 0; }
        return XG2_OK;
    });
}
int32_t xg2_grammar_num_positions(const xg2_grammar* g, int32_t* out) {
    if (!g || !out) return fail(XG2_EINVAL, "xg2_grammar_num_positions: bad argument");
    *out = (int32_t)g->p->g.positions.size();
    return XG2_OK;
}

int32_t xg2_pool_create(size_t max_bytes, xg2_pool** out) {
    return guarded([&]() -> int32_t {
        if (!out) return fail(XG2_EINVAL, "xg2_pool_create: null out");
        auto p = std::make_shared<PoolImpl>();
        p->max_bytes = max_bytes;
        *out = new xg2_pool{p};
        return XG2_OK;
    });
}
void xg2_pool_destroy(xg2_pool* p) { delete p; }
int32_t xg2_pool_stats(const xg2_pool* p, int64_t* n_positions, int64_t* device_bytes) {
    if (!p) return fail(XG2_EINVAL, "xg2_pool_stats: null pool");
    std::lock_guard<std::mutex> lk(p->p->mu);
    if (n_positions) *n_positions = p->p->n_rows;
    if (device_bytes) *device_bytes = (int64_t)p->p->device_bytes;
    return XG2_OK;
}

int32_t xg2_compile_grammar(xg2_vocab* vocab, const char* ebnf, size_t len, const char* root_rule, const xg2_compile_opts* opts,
                            xg2_pool* pool_h, void* hip_stream, xg2_mask_cache** out, xg2_compile_stats* stats) {
    return guarded([&]() -> int32_t {
        if (!vocab || !out) return fail(XG2_EINVAL, "xg2_compile_grammar: bad argument");
        const int32_t depth = opts ? opts->context_depth : 2;
        const bool merge = opts ? opts->merge_equivalent != 0 : true;
        const bool follow = opts ? opts->follow_filter != 0 : true;
        const int32_t jit = (opts && opts->jit) ? std::max(opts->jit_prebuild, 0) : -1;   // -1: build every plane now
        const bool partial = opts ? opts->partial_hits != 0 : true;
        if (depth != 1 && depth != 2) return fail(XG2_EINVAL, "xg2_compile_grammar: context_depth must be 1 or 2");
        hipStream_t stream = (hipStream_t)hip_stream;
        auto t0 = std::chrono::steady_clock::now();
        auto cache = std::make_shared<CacheImpl>();
        cache->vocab = vocab->p;
        cache->context_depth = depth;
        cache->partial_hits = partial;
        cache->time_kernel = opts ? opts->time_kernel != 0 : false;
        cache->gram = make_grammar(ebnf, len, root_rule);
        const Grammar& g = cache->gram->g;
        const FlatTables& ft = cache->gram->ft;
        VocabImpl& V = *vocab->p;
        V.ensure_device();
        cache->pool = pool_h ? pool_h->p : std::make_shared<PoolImpl>();
        PoolImpl& pool = *cache->pool;
        std::lock_guard<std::mutex> pool_lock(pool.mu);
        if (!pool.vocab) pool.vocab = vocab->p;
        else if (pool.vocab.get() != vocab->p.get()) return fail(XG2_EINVAL, "xg2_compile_grammar: pool is bound to another vocabulary");
        std::lock_guard<std::mutex> slow_lock(build_slow().mu);
        build_slow().ensure();
        SlowScratch S = build_slow().s;
        const int R = (int)g.rules.size();

        // intern every rule in the pool, referenced rules first
        std::vector<int> entry((size_t)R, -1);
        std::vector<uint64_t> ref_id((size_t)R, 0);
        for (const auto& comp : g.hash_order) {
            const RuleFsm& first = g.rules[(size_t)comp[0]];
            if (!first.shareable) {
                for (int r : comp) entry[(size_t)r] = pool.intern(g.rules[(size_t)r].hash, "", false);
            } else if (first.ring.empty()) {
                int r = comp[0];
                entry[(size_t)r] = pool.intern(first.hash, serialise_rule(g, r, ref_id), true);
            } else {
                std::vector<uint64_t> ids = ref_id;
                for (int r : comp) ids[(size_t)r] = kInCycleRef;
                std::map<int, std::string> local;
                for (int r : comp) local[r] = serialise_rule(g, r, ids);
                for (int r : comp) {
                    std::string text = "C";
                    for (int v : g.rules[(size_t)r].ring) { text += local[v]; text.push_back('|'); }
                    entry[(size_t)r] = pool.intern(g.rules[(size_t)r].hash, text, true);
                }
            }
            for (int r : comp) ref_id[(size_t)r] = (uint64_t)entry[(size_t)r] + 1;
        }

        // states that tokens cannot tell apart share planes
        std::vector<std::vector<int32_t>> rep, classes;
        std::vector<NearClasses> near((size_t)R);
        if (merge || follow) {
            const int32_t class_budget = (int32_t)std::max<uint32_t>(V.max_len, 1);
            classes.resize((size_t)R);
            for (int r = 0; r < R; ++r) {
                const RuleFsm& f = g.rules[(size_t)r];
                const int n = f.n_states();
                std::vector<int32_t> by_canon((size_t)n);             // canonical number -> state
                for (int x = 0; x < n; ++x) by_canon[(size_t)f.canon_id[(size_t)x]] = x;
                auto key = std::make_pair(entry[(size_t)r], class_budget);
                auto hit = f.shareable ? pool.class_memo.find(key) : pool.class_memo.end();
                NearClasses& nr = near[(size_t)r];
                if (hit != pool.class_memo.end() && (int)hit->second.rep.size() == n) {
                    // an identical rule was analysed before (this grammar or an earlier one): translate through the canonical numbers
                    const PoolImpl::ClassMemo& cm = hit->second;
                    classes[(size_t)r].resize((size_t)n);
                    nr.base.resize((size_t)n); nr.depth.resize((size_t)n);
                    for (int x = 0; x < n; ++x) {
                        const size_t c = (size_t)f.canon_id[(size_t)x];
                        classes[(size_t)r][(size_t)x] = by_canon[(size_t)cm.rep[c]];
                        nr.base[(size_t)x] = cm.base[c] < 0 ? -1 : by_canon[(size_t)cm.base[c]];
                        nr.depth[(size_t)x] = cm.depth[c];
                    }
                    continue;
                }
                classes[(size_t)r] = bounded_classes_rule(g, r, class_budget, ref_id, &nr);
                if (f.shareable) {
                    PoolImpl::ClassMemo cm;
                    cm.rep.resize((size_t)n); cm.base.resize((size_t)n); cm.depth.resize((size_t)n);
                    for (int x = 0; x < n; ++x) {
                        const size_t c = (size_t)f.canon_id[(size_t)x];
                        cm.rep[c] = f.canon_id[(size_t)classes[(size_t)r][(size_t)x]];
                        cm.base[c] = nr.base[(size_t)x] < 0 ? -1 : f.canon_id[(size_t)nr.base[(size_t)x]];
                        cm.depth[c] = nr.depth[(size_t)x];
                    }
                    pool.class_memo.emplace(key, std::move(cm));
                }
            }
        }
        if (merge) rep = classes;
        else {
            rep.resize((size_t)R);
            for (int r = 0; r < R; ++r) { rep[(size_t)r].resize((size_t)g.rules[(size_t)r].n_states()); std::iota(rep[(size_t)r].begin(), rep[(size_t)r].end(), 0); }
        }
        FollowInfo follow_info;
        const int32_t budget = (int32_t)std::max<uint32_t>(V.max_len, 1);
        // follow signatures are numbers the pool hands out for exact descriptions of the bounded follow language (rules named
        // by their pool entries): equal numbers, equal structures
        const FollowInterner intern_follow = [&pool](const std::vector<uint64_t>& desc) -> uint64_t {
            auto it = pool.follow_nodes.find(desc);
            if (it != pool.follow_nodes.end()) return it->second;
            const uint64_t id = ((uint64_t)pool.follow_nodes.size() + 1) << 1;      // even: the key sets bit 0, and 0 stays "unfiltered"
            pool.follow_nodes.emplace(desc, id);
            return id;
        };
        const FollowMemo follow_memo = [&](int rule, int state, int d) -> uint64_t* {
            const RuleFsm& f = g.rules[(size_t)rule];
            if (!f.shareable) return nullptr;
            std::vector<uint64_t>& slots = pool.follow_unfold[entry[(size_t)rule]];
            const size_t n = (size_t)f.n_states();
            if (slots.size() != ((size_t)budget + 1) * n) slots.assign(((size_t)budget + 1) * n, 0);
            return &slots[(size_t)d * n + (size_t)f.canon_id[(size_t)state]];
        };
        if (follow) follow_info = follow_signatures(g, budget, &classes, &ref_id, &intern_follow, &follow_memo);
        // reference sites of every rule, one representative per class of the state the referencing rule continues in
        struct Site { int32_t q, waiter, x; };
        std::vector<std::vector<Site>> sites((size_t)R);            // all sites
        std::vector<std::map<std::pair<int, int>, Site>> site_rep((size_t)R);   // (q, class of x) -> representative
        if (depth == 2)
            for (int q = 0; q < R; ++q)
                for (int s = 0; s < g.rules[(size_t)q].n_states(); ++s)
                    for (auto& e : g.rules[(size_t)q].redges[(size_t)s]) {
                        Site st{q, s, e.tgt};
                        sites[(size_t)e.rule].push_back(st);
                        auto key = std::make_pair(q, (int)rep[(size_t)q][(size_t)e.tgt]);
                        auto it = site_rep[(size_t)e.rule].find(key);
                        const RuleFsm& fq = g.rules[(size_t)q];
                        if (it == site_rep[(size_t)e.rule].end()) site_rep[(size_t)e.rule].emplace(key, st);
                        else if (fq.canon_id[(size_t)e.tgt] < fq.canon_id[(size_t)it->second.x]) it->second = st;
                    }

        // planes of this grammar
        std::map<PlaneKey, int32_t> local_plane;
        auto make_key = [&](int rp, int sp_rep, int site_q, int site_x) -> PlaneKey {
            const RuleFsm& fp = g.rules[(size_t)rp];
            PlaneKey key{entry[(size_t)rp], fp.canon_id[(size_t)sp_rep], -1, -1, 0};
            if (site_q >= 0) { key[2] = entry[(size_t)site_q]; key[3] = g.rules[(size_t)site_q].canon_id[(size_t)site_x]; }
            if (follow) {
                // a token reaches what follows the outermost rule only after the shortest way out of the plane's rules, so
                // the plane depends on the follow language no deeper than the bytes that are left then: planes whose way out
                // is long are shared between grammars that differ only further on
                int64_t need = follow_info.min_suf[(size_t)rp][(size_t)sp_rep];
                if (site_q >= 0) need += follow_info.min_suf[(size_t)site_q][(size_t)site_x];
                const int64_t depth_left = std::max<int64_t>(0, (int64_t)budget - std::max<int64_t>(1, need));
                key[4] = (int64_t)(follow_info.sig[(size_t)(site_q >= 0 ? site_q : rp)][(size_t)depth_left] | 1);
            }
            return key;
        };
        auto plane_for = [&](int rp, int sp_rep, const Site* site) -> int32_t {
            const PlaneKey key = make_key(rp, sp_rep, site ? site->q : -1, site ? site->x : -1);
            auto lp = local_plane.find(key);
            if (lp != local_plane.end()) return lp->second;
            const uint32_t sid = (uint32_t)g.sid(rp, sp_rep);
            // cost estimate: tokens that start with a byte the state itself reads, weighted up when the start set
            // is more than a plain automaton state
            const StateInfo& si = ft.state_info[sid];
            uint64_t cost = 0;
            for (uint32_t e = 0; e < (si.counts & 0xFFFF); ++e) {
                const ByteEdge& be = ft.byte_edges[si.byte_off + e];
                cost += V.fb_start[((be.lohi >> 8) & 0xFF) + 1] - V.fb_start[be.lohi & 0xFF];
            }
            if ((si.counts >> 16) || (si.rule_final >> 31)) cost *= 4;
            int32_t idx = (int32_t)cache->planes.size();
            cache->planes.push_back({rp, sp_rep, site ? site->q : -1, site ? site->x : -1, nullptr, false, key, sid,
                                     site ? (int64_t)g.sid(site->q, site->waiter) : -1, cost});
            local_plane.emplace(key, idx);
            return idx;
        };
        cache->plain_plane.assign((size_t)g.n_states, -1);
        for (const Position& ps : g.positions) {
            int sp_rep = rep[(size_t)ps.rule][(size_t)ps.state];
            if (depth == 1 || ps.rule == g.root) cache->plain_plane[(size_t)ps.sid] = plane_for(ps.rule, sp_rep, nullptr);
            if (depth == 2)
                for (const Site& st : sites[(size_t)ps.rule]) {
                    const Site& sr = site_rep[(size_t)ps.rule].at(std::make_pair(st.q, (int)rep[(size_t)st.q][(size_t)st.x]));
                    cache->pair_plane[((uint64_t)(uint32_t)ps.sid << 32) | (uint32_t)g.sid(st.q, st.x)] = plane_for(ps.rule, sp_rep, &sr);
                }
        }

        // planes that coincide with another plane of the same rule and context on all short tokens (section 3.6: the states
        // near the end of a long repetition differ from the ones inside it only on tokens long enough to reach the bound)
        if (merge)
            for (PlaneInfo& pi : cache->planes) {
                const NearClasses& nr = near[(size_t)pi.rule];
                if (nr.base.empty() || nr.base[(size_t)pi.state] < 0) continue;
                auto lp = local_plane.find(make_key(pi.rule, nr.base[(size_t)pi.state], pi.parent_rule, pi.parent_state));
                if (lp == local_plane.end()) continue;
                pi.near_plane = lp->second;
                pi.near_depth = nr.depth[(size_t)pi.state];
            }

        // Planes of plain automaton states (byte edges only) that move like the start state of their rule on most first
        // bytes: the states of a dispatch automaton all fall back to free text on any byte that does not continue a tag.
        // After the first byte the two runs are in states no token can tell apart, so the classes of the tokens with such
        // a first byte are the start state's; only the tokens with the other first bytes are checked.
        if (merge) {
            std::vector<uint8_t> is_near_base(cache->planes.size(), 0);
            for (const PlaneInfo& pi : cache->planes) if (pi.near_plane >= 0) is_near_base[(size_t)pi.near_plane] = 1;
            auto plain = [&](const RuleFsm& f, int x) { return f.redges[(size_t)x].empty() && !f.bedges[(size_t)x].empty(); };
            struct FirstByteAlike { std::array<uint32_t, 8> same; bool worth; };
            std::vector<FirstByteAlike> fb_memo;
            std::vector<std::vector<int32_t>> fb_of((size_t)R);      // per rule and state: index into fb_memo, or -1
            for (size_t idx = 0; idx < cache->planes.size(); ++idx) {
                PlaneInfo& pi = cache->planes[idx];
                if (pi.near_plane >= 0 || is_near_base[idx]) continue;
                const RuleFsm& f = g.rules[(size_t)pi.rule];
                const int x = pi.state, b0 = rep[(size_t)pi.rule][0];
                // (a state that can end its rule brings the continuation of the referencing rule into its start set: the
                // same one for both states if both can end, none if neither can)
                if (x == b0 || !plain(f, x) || !plain(f, b0) || f.is_final[(size_t)x] != f.is_final[(size_t)b0]) continue;
                // the comparison depends on the state only, not on the site: done once per state
                std::vector<int32_t>& of = fb_of[(size_t)pi.rule];
                if (of.empty()) of.assign((size_t)f.n_states(), -1);
                if (of[(size_t)x] < 0) {
                    int32_t tx[256], ty[256];
                    std::fill(tx, tx + 256, -1); std::fill(ty, ty + 256, -1);
                    for (auto& e : f.bedges[(size_t)x]) for (int b = e.lo; b <= e.hi; ++b) tx[b] = rep[(size_t)pi.rule][(size_t)e.tgt];
                    for (auto& e : f.bedges[(size_t)b0]) for (int b = e.lo; b <= e.hi; ++b) ty[b] = rep[(size_t)pi.rule][(size_t)e.tgt];
                    uint64_t differ = 0, all = 0;
                    FirstByteAlike fa{};
                    for (int b = 0; b < 256; ++b) {
                        const uint64_t n_b = V.fb_start[b + 1] - V.fb_start[b];
                        if (tx[b] == ty[b]) fa.same[(size_t)b >> 5] |= 1u << (b & 31);
                        else if (tx[b] >= 0) differ += n_b;
                        if (tx[b] >= 0) all += n_b;
                    }
                    fa.worth = differ * 2 <= all;                    // else too little to gain
                    of[(size_t)x] = (int32_t)fb_memo.size();
                    fb_memo.push_back(fa);
                }
                const FirstByteAlike* memo = &fb_memo[(size_t)of[(size_t)x]];
                if (!memo->worth) continue;
                auto lp = local_plane.find(make_key(pi.rule, b0, pi.parent_rule, pi.parent_state));
                if (lp == local_plane.end() || cache->planes[(size_t)lp->second].near_plane >= 0) continue;
                pi.fb_plane = lp->second;
                pi.fb_same = memo->same;
            }
        }

        // The planes of one state under different referencing sites: as long as a token stays among the plain states of the
        // rule that cannot end it, the site plays no part.  Only the tokens that contain a byte on which some such state
        // (reachable from the plane's state) predicts or ends the rule are checked for every site; for the rest the plane of
        // the first site serves all.
        if (merge && depth == 2) {
            std::vector<uint8_t> is_base(cache->planes.size(), 0);
            for (const PlaneInfo& pi : cache->planes) {
                if (pi.near_plane >= 0) is_base[(size_t)pi.near_plane] = 1;
                if (pi.fb_plane >= 0) is_base[(size_t)pi.fb_plane] = 1;
            }
            std::map<std::pair<int32_t, int32_t>, std::vector<int32_t>> groups;      // (rule, state) -> planes with a site
            for (size_t idx = 0; idx < cache->planes.size(); ++idx) {
                const PlaneInfo& pi = cache->planes[idx];
                if (pi.parent_rule < 0 || pi.near_plane >= 0 || pi.fb_plane >= 0 || is_base[idx]) continue;
                const RuleFsm& f = g.rules[(size_t)pi.rule];
                if (!f.redges[(size_t)pi.state].empty() || f.is_final[(size_t)pi.state] || f.bedges[(size_t)pi.state].empty()) continue;
                groups[std::make_pair(pi.rule, pi.state)].push_back((int32_t)idx);
            }
            for (auto& kv : groups) {
                if (kv.second.size() < 2) continue;
                const RuleFsm& f = g.rules[(size_t)kv.first.first];
                // plain states that cannot end the rule, reachable from the state; bytes that lead out of them
                std::array<uint32_t, 8> out{};
                std::vector<uint8_t> seen((size_t)f.n_states(), 0);
                std::vector<int> stack{kv.first.second};
                seen[(size_t)kv.first.second] = 1;
                while (!stack.empty()) {
                    const int q = stack.back(); stack.pop_back();
                    for (auto& e : f.bedges[(size_t)q]) {
                        const bool inside = f.redges[(size_t)e.tgt].empty() && !f.is_final[(size_t)e.tgt];
                        if (!inside) { for (int b = e.lo; b <= e.hi; ++b) out[(size_t)b >> 5] |= 1u << (b & 31); }
                        else if (!seen[(size_t)e.tgt]) { seen[(size_t)e.tgt] = 1; stack.push_back(e.tgt); }
                    }
                }
                const int32_t list = V.list_of_tokens_with(out);
                if ((uint64_t)V.byte_lists[(size_t)list].n * 2 > cache->planes[(size_t)kv.second[0]].cost) continue;   // too little to gain
                for (size_t k = 1; k < kv.second.size(); ++k) {
                    PlaneInfo& pi = cache->planes[(size_t)kv.second[k]];
                    pi.site_plane = kv.second[0];
                    pi.site_list = list;
                }
            }
        }

        // per rule, the states referencing rules continue in: one per class of indistinguishable states
        cache->follow = follow;
        cache->site_off.assign(1, 0);
        if (follow) {
            std::vector<std::vector<uint32_t>> by_rule((size_t)R);
            for (int q = 0; q < R; ++q)
                for (int s = 0; s < g.rules[(size_t)q].n_states(); ++s)
                    for (auto& e : g.rules[(size_t)q].redges[(size_t)s])
                        by_rule[(size_t)e.rule].push_back(ft.ref((uint32_t)g.sid(q, classes[(size_t)q][(size_t)e.tgt])));
            for (auto& v : by_rule) {
                std::sort(v.begin(), v.end());
                v.erase(std::unique(v.begin(), v.end()), v.end());
                cache->site_tgt.insert(cache->site_tgt.end(), v.begin(), v.end());
                cache->site_off.push_back((uint32_t)cache->site_tgt.size());
            }
        } else cache->site_off.assign((size_t)R + 1, 0);

        // which planes to build now: all of them, or (section 3.5) the jit_prebuild most expensive ones
        std::vector<int32_t> todo((size_t)cache->planes.size());
        std::iota(todo.begin(), todo.end(), 0);
        if (jit >= 0 && (size_t)jit < todo.size()) {
            std::stable_sort(todo.begin(), todo.end(), [&](int32_t a, int32_t b) { return cache->planes[(size_t)a].cost > cache->planes[(size_t)b].cost; });
            todo.resize((size_t)jit);
            std::sort(todo.begin(), todo.end());
        }
        double host_ms_a = ms_since(t0);
        std::shared_ptr<BuildTicket> ticket;
        int32_t rc = build_planes(*cache, todo, stream, true, S, &ticket);
        if (rc != XG2_OK) return rc;
        cache->compile_ticket = ticket;
        cache->host_lower_ms = host_ms_a + (ticket ? ticket->host_ms : 0.0);
        cache->compile_built = ticket ? (int64_t)ticket->rows.size() : 0;
        if (stats) {                                            // what is known without waiting for the device
            std::memset(stats, 0, sizeof(*stats));
            stats->positions = (int64_t)g.positions.size();
            stats->unique = (int64_t)cache->planes.size();
            stats->built = cache->compile_built;
            stats->partial_hits = ticket ? ticket->partial_hits : 0;
            stats->checks = (cache->compile_built - stats->partial_hits) * (int64_t)V.n_sorted;
            stats->executed_checks = ticket ? ticket->executed : 0;
            stats->executed_token_bytes = ticket ? ticket->executed_bytes : 0;
            stats->host_lower_ms = cache->host_lower_ms;
        }
        *out = new xg2_mask_cache{cache};
        return XG2_OK;
    });
}
void xg2_mask_cache_destroy(xg2_mask_cache* c) { delete c; }

int32_t xg2_mask_cache_stats(xg2_mask_cache* c, xg2_compile_stats* stats) {
    return guarded([&]() -> int32_t {
        if (!c) return fail(XG2_EINVAL, "xg2_mask_cache_stats: null cache");
        CacheImpl& C = *c->p;
        finalize_cache(C);
        if (C.failed) return cache_failed();
        if (!stats) return XG2_OK;
        std::memset(stats, 0, sizeof(*stats));
        const BuildTicket* t = C.compile_ticket.get();
        stats->positions = (int64_t)C.gram->g.positions.size();
        stats->unique = (int64_t)C.planes.size();
        stats->built = C.compile_built;
        stats->partial_hits = t ? t->partial_hits : 0;
        stats->checks = (C.compile_built - stats->partial_hits) * (int64_t)C.vocab->n_sorted;
        stats->host_lower_ms = C.host_lower_ms;
        if (t) {
            stats->executed_checks = t->executed; stats->executed_token_bytes = t->executed_bytes;
            stats->slow_path = t->slow; stats->n_accepted = t->n_accepted; stats->n_uncertain = t->n_uncertain;
            stats->device_ms = t->device_ms; stats->kernel_ms = t->kernel_ms;
        }
        return XG2_OK;
    });
}

int32_t xg2_mask_cache_num_positions(const xg2_mask_cache* c, int32_t* out) {
    if (!c || !out) return fail(XG2_EINVAL, "xg2_mask_cache_num_positions: bad argument");
    *out = (int32_t)c->p->gram->g.positions.size();
    return XG2_OK;
}
int32_t xg2_mask_cache_jit_stats(const xg2_mask_cache* c, int32_t* n_built, int32_t* n_builds_in_fill, double* device_ms_in_fill) {
    if (!c) return fail(XG2_EINVAL, "xg2_mask_cache_jit_stats: null cache");
    CacheImpl& C = *const_cast<CacheImpl*>(c->p.get());
    try { finalize_cache(C); } catch (const std::exception& e) { return fail(XG2_EHIP, e.what()); }
    for (auto& t : C.jit_tickets) C.jit_device_ms += t->device_ms;
    C.jit_tickets.clear();
    if (n_built) *n_built = (int32_t)c->p->n_built;
    if (n_builds_in_fill) *n_builds_in_fill = (int32_t)c->p->jit_calls;
    if (device_ms_in_fill) *device_ms_in_fill = c->p->jit_device_ms;
    return XG2_OK;
}
int32_t xg2_mask_cache_num_planes(const xg2_mask_cache* c, int32_t* out) {
    if (!c || !out) return fail(XG2_EINVAL, "xg2_mask_cache_num_planes: bad argument");
    *out = (int32_t)c->p->planes.size();
    return XG2_OK;
}
int32_t xg2_mask_cache_plane_info(const xg2_mask_cache* c, int32_t k, const char** rule, int32_t* state,
                                  const char** parent_rule, int32_t* parent_state) {
    if (!c || k < 0 || (size_t)k >= c->p->planes.size()) return fail(XG2_EINVAL, "xg2_mask_cache_plane_info: bad argument");
    const PlaneInfo& pi = c->p->planes[(size_t)k];
    if (rule) *rule = c->p->gram->rule_names[(size_t)pi.rule].c_str();
    if (state) *state = pi.state;
    if (parent_rule) *parent_rule = pi.parent_rule >= 0 ? c->p->gram->rule_names[(size_t)pi.parent_rule].c_str() : nullptr;
    if (parent_state) *parent_state = pi.parent_state;
    return XG2_OK;
}
int32_t xg2_mask_cache_find_plane(const xg2_mask_cache* c, const char* rule, int32_t state, const char* parent_rule,
                                  int32_t parent_state, int32_t* k) {
    if (!c || !rule || !k) return fail(XG2_EINVAL, "xg2_mask_cache_find_plane: bad argument");
    const Grammar& g = c->p->gram->g;
    auto find_rule = [&](const char* name) { for (size_t r = 0; r < g.rules.size(); ++r) if (g.rules[r].name == name) return (int)r; return -1; };
    int rp = find_rule(rule);
    if (rp < 0 || state < 0 || state >= g.rules[(size_t)rp].n_states()) return fail(XG2_EINVAL, "xg2_mask_cache_find_plane: unknown rule or state");
    *k = -1;
    if (!parent_rule) { *k = c->p->plain_plane[(size_t)g.sid(rp, state)]; return XG2_OK; }
    int rq = find_rule(parent_rule);
    if (rq < 0 || parent_state < 0 || parent_state >= g.rules[(size_t)rq].n_states()) return fail(XG2_EINVAL, "xg2_mask_cache_find_plane: unknown parent rule or state");
    auto it = c->p->pair_plane.find(((uint64_t)(uint32_t)g.sid(rp, state) << 32) | (uint32_t)g.sid(rq, parent_state));
    if (it != c->p->pair_plane.end()) *k = it->second;
    return XG2_OK;
}
int32_t xg2_mask_cache_get_planes(const xg2_mask_cache* c, int32_t k, int32_t* accepted_host, int32_t* uncertain_host) {
    return guarded([&]() -> int32_t {
        if (!c || k < 0 || (size_t)k >= c->p->planes.size()) return fail(XG2_EINVAL, "xg2_mask_cache_get_planes: bad argument");
        const uint32_t W = c->p->vocab->W;
        finalize_cache(*const_cast<CacheImpl*>(c->p.get()));
        if (c->p->failed) return cache_failed();
        const uint32_t* row = c->p->planes[(size_t)k].row;
        if (!row) return fail(XG2_EINVAL, "xg2_mask_cache_get_planes: this plane has not been built yet (cache compiled just in time)");
        HIP_CHECK(hipDeviceSynchronize());
        if (accepted_host) HIP_CHECK(hipMemcpy(accepted_host, row, W * sizeof(uint32_t), hipMemcpyDeviceToHost));
        if (uncertain_host) HIP_CHECK(hipMemcpy(uncertain_host, row + W, W * sizeof(uint32_t), hipMemcpyDeviceToHost));
        return XG2_OK;
    });
}

int32_t xg2_matcher_create(const xg2_mask_cache* c, xg2_matcher** out) {
    return guarded([&]() -> int32_t {
        if (!c || !out) return fail(XG2_EINVAL, "xg2_matcher_create: bad argument");
        auto m = std::make_unique<MatcherImpl>(c->p->gram, c->p->vocab);
        m->cache = c->p;
        *out = new xg2_matcher{std::move(m)};
        return XG2_OK;
    });
}
int32_t xg2_matcher_create_host(const xg2_grammar* g, const xg2_vocab* v, xg2_matcher** out) {
    return guarded([&]() -> int32_t {
        if (!g || !v || !out) return fail(XG2_EINVAL, "xg2_matcher_create_host: bad argument");
        *out = new xg2_matcher{std::make_unique<MatcherImpl>(g->p, v->p)};
        return XG2_OK;
    });
}
void xg2_matcher_destroy(xg2_matcher* m) { delete m; }

static int32_t accept_one(xg2_matcher* m, int32_t token_id);
int32_t xg2_matcher_accept_token(xg2_matcher* m, int32_t token_id) {
    if (int32_t rc = report_undecided_pairs()) return rc;
    return accept_one(m, token_id);
}
static int32_t accept_one(xg2_matcher* m, int32_t token_id) {
    return guarded([&]() -> int32_t {
        if (!m) return fail(XG2_EINVAL, "xg2_matcher_accept_token: null matcher");
        MatcherImpl& M = *m->p;
        if (token_id < 0 || token_id >= M.vocab->V) return fail(XG2_EINVAL, "xg2_matcher_accept_token: token id out of range");
        if (M.terminated) return fail(XG2_EINVAL, "xg2_matcher_accept_token: matcher has terminated");
        if (token_id == M.vocab->eos) {
            if (!M.chart.last().root_done) return fail(XG2_EREJECTED, "end of sequence is not allowed here");
            M.terminated = true;
            M.prep.valid = false;
            return XG2_OK;
        }
        if (M.vocab->special[(size_t)token_id]) return fail(XG2_EREJECTED, "special or empty tokens are never allowed");
        if (!M.chart.advance(M.vocab->tok(token_id), M.vocab->len(token_id))) return fail(XG2_EREJECTED, "token is not allowed here");
        M.prep.valid = false;
        return XG2_OK;
    });
}
int32_t xg2_matcher_accept_tokens(xg2_matcher* const* matchers, const int32_t* token_ids, int32_t B, int32_t* status_host) {
    if (B < 0 || (B > 0 && (!matchers || !token_ids || !status_host))) return fail(XG2_EINVAL, "xg2_matcher_accept_tokens: bad argument");
    for (int32_t b = 0; b < B; ++b) if (!matchers[b]) return fail(XG2_EINVAL, "xg2_matcher_accept_tokens: null matcher");
    if (int32_t rc = report_undecided_pairs()) return rc;
    // matchers are independent: a few host threads each take a contiguous share (a handle listed twice would race)
    std::atomic<bool> failed{false};
    std::string what;
    std::mutex what_mu;
    const int32_t share = 32;                                   // matchers per part: small enough to balance, large enough to amortise the hand-over
    const int32_t parts = (B + share - 1) / share;
    const std::function<void(int32_t)> work = [&](int32_t part) {
        try {
            for (int32_t b = part * share; b < std::min(B, (part + 1) * share); ++b) {
                status_host[b] = token_ids[b] < 0 ? XG2_OK : accept_one(matchers[b], token_ids[b]);
                prepare_matcher(*matchers[b]->p);               // the next fill finds the state ready
            }
        } catch (const std::exception& e) {
            failed = true;
            std::lock_guard<std::mutex> lk(what_mu);
            what = e.what();
        }
    };
    if (parts <= 2) { for (int32_t p = 0; p < parts; ++p) work(p); }
    else host_workers().run(parts, work);
    if (failed) return fail(XG2_EINVAL, "xg2_matcher_accept_tokens: " + what);
    return XG2_OK;
}
int32_t xg2_matcher_reset(xg2_matcher* m) {
    if (!m) return fail(XG2_EINVAL, "xg2_matcher_reset: null matcher");
    m->p->chart.start(m->p->gram->ft.root_start);
    m->p->terminated = false;
    m->p->prep.valid = false;
    return XG2_OK;
}
int32_t xg2_matcher_is_terminated(const xg2_matcher* m, int32_t* out) {
    if (!m || !out) return fail(XG2_EINVAL, "xg2_matcher_is_terminated: bad argument");
    *out = m->p->terminated ? 1 : 0;
    return XG2_OK;
}
int32_t xg2_matcher_frontier(const xg2_matcher* m, int32_t* positions_host, int32_t cap, int32_t* n, int32_t* can_end) {
    if (!m || !n || cap < 0 || (cap > 0 && !positions_host)) return fail(XG2_EINVAL, "xg2_matcher_frontier: bad argument");
    const MatcherImpl& M = *m->p;
    std::vector<int32_t> pos;
    if (!M.terminated)
        for (const ChartItem& it : M.chart.last().scan) {
            int32_t p = M.gram->g.sid_to_pos[it.sid];
            if (p >= 0 && std::find(pos.begin(), pos.end(), p) == pos.end()) pos.push_back(p);
        }
    std::sort(pos.begin(), pos.end());
    *n = (int32_t)pos.size();
    for (int32_t k = 0; k < std::min<int32_t>(cap, *n); ++k) positions_host[k] = pos[(size_t)k];
    if (can_end) *can_end = (M.terminated || M.chart.last().root_done) ? 1 : 0;
    return XG2_OK;
}

}  // extern "C"

namespace {
// The body of both fill entry points.  no_alloc: every device buffer comes from the library's fixed scratch array, the
// per-row records are copied from ordinary host memory, nothing is allocated and nothing is built (a plane that is
// still missing is an error), no events are recorded.
int32_t fill_common(xg2_matcher* const* matchers, int32_t B, int32_t* bitmask_dev, int64_t row_stride_words,
                    void* hip_stream, bool no_alloc) {
    return guarded([&]() -> int32_t {
        if (B < 0 || (B > 0 && (!matchers || !bitmask_dev))) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: bad argument");
        if (B == 0) return XG2_OK;
        if (int32_t rc = report_undecided_pairs()) return rc;
        hipStream_t stream = (hipStream_t)hip_stream;
        for (int32_t b = 0; b < B; ++b) {
            if (!matchers[b]) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: null matcher");
            if (!matchers[b]->p->cache) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: host-only matcher has no mask cache");
            if (matchers[b]->p->vocab.get() != matchers[0]->p->vocab.get())
                return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: matchers use different vocabularies");
        }
        VocabImpl& V = *matchers[0]->p->vocab;
        if (row_stride_words < (int64_t)V.W) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: row stride smaller than ceil(V/32)");
        if (no_alloc) {
            if (!V.on_device) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask_noalloc: the vocabulary is not on the device");
            if ((size_t)B > kNoAllocMaxRows || (size_t)B * V.W > kNoAllocMaskWords)
                return fail(XG2_EOVERFLOW, "xg2_fill_next_token_bitmask_noalloc: batch beyond the fixed scratch (at most " + std::to_string(kNoAllocMaxRows) +
                                           " rows and " + std::to_string(kNoAllocMaskWords) + " mask words, rows x ceil(V/32), per call)");
        } else V.ensure_device();

        // caches compiled just in time (section 3.5): the planes this step's frontiers need and that hold no row yet
        // are built first, on the same stream
        {
            // matchers that moved since their last fill (and were not advanced by the batched accept call, which leaves them
            // ready) get their context slice and frontier planes first, on the host threads when there are many
            std::vector<MatcherImpl*> stale;
            for (int32_t b = 0; b < B; ++b) if (!matchers[b]->p->prep.valid) stale.push_back(matchers[b]->p.get());
            std::sort(stale.begin(), stale.end());
            stale.erase(std::unique(stale.begin(), stale.end()), stale.end());
            if (stale.size() >= 128) {
                const int32_t share = 32, parts = ((int32_t)stale.size() + share - 1) / share;
                std::atomic<bool> failed{false};
                const std::function<void(int32_t)> work = [&](int32_t part) {
                    try {
                        for (size_t k = (size_t)part * share; k < std::min(stale.size(), (size_t)(part + 1) * share); ++k) prepare_matcher(*stale[k]);
                    } catch (const std::exception&) { failed = true; }
                };
                host_workers().run(parts, work);
                if (failed) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask: preparing a matcher failed");
            }
            // builds enqueued by earlier calls (compile, or a fill that built just in time) are looked at now: by this
            // time they have finished, and a failed one must not pass
            {
                CacheImpl* seen = nullptr;
                for (int32_t b = 0; b < B; ++b) {
                    CacheImpl* C = matchers[b]->p->cache.get();
                    if (C == seen) continue;
                    seen = C;
                    if (!C->tickets.empty() || !C->fresh_planes.empty()) finalize_cache(*C);
                    if (C->failed) return cache_failed();
                }
            }
            std::map<CacheImpl*, std::vector<int32_t>> missing;
            for (int32_t b = 0; b < B; ++b) {
                MatcherImpl& M = *matchers[b]->p;
                prepare_matcher(M);
                if (M.prep.status != XG2_OK) return fail(M.prep.status, M.prep.error.c_str());
                if (M.terminated || M.cache->n_built == (int64_t)M.cache->planes.size()) continue;
                std::vector<int32_t>& v = missing[M.cache.get()];
                for (auto& pl : M.prep.planes) if (!M.cache->planes[(size_t)pl.first].row) v.push_back(pl.first);
            }
            for (auto& kv : missing) {
                std::vector<int32_t>& v = kv.second;
                std::sort(v.begin(), v.end());
                v.erase(std::unique(v.begin(), v.end()), v.end());
                if (v.empty()) continue;
                if (no_alloc) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask_noalloc: a plane of a cache compiled just in time is not built yet "
                                                      "(building allocates: use xg2_fill_next_token_bitmask for such caches)");
                CacheImpl& C = *kv.first;
                std::lock_guard<std::mutex> pool_lock(C.pool->mu);
                std::lock_guard<std::mutex> slow_lock(build_slow().mu);
                build_slow().ensure();
                // on the library's own stream, beside whatever the caller's stream is doing; the caller's stream waits for
                // it on the device, the host does not
                std::shared_ptr<BuildTicket> ticket;
                int32_t rc = build_planes(C, v, jit_stream(), false, build_slow().s, &ticket);
                if (rc != XG2_OK) return rc;
                if (ticket) {                                       // rows found in the pool cost no launch
                    ++C.jit_calls;
                    C.jit_tickets.push_back(ticket);
                    HIP_CHECK(hipStreamWaitEvent(stream, ticket->staging->ev[4], 0));
                }
            }
        }

        std::vector<FillRow> rows((size_t)B);
        std::vector<uint64_t> front;
        std::vector<uint32_t> items, wait, wait_off;
        std::vector<DevTables> tables;
        std::map<const CacheImpl*, uint32_t> table_idx;
        for (int32_t b = 0; b < B; ++b) {
            const MatcherImpl& M = *matchers[b]->p;
            FillRow& r = rows[(size_t)b];
            std::memset(&r, 0, sizeof(r));
            auto ti = table_idx.find(M.cache.get());
            if (ti == table_idx.end()) { ti = table_idx.emplace(M.cache.get(), (uint32_t)tables.size()).first; tables.push_back(M.cache->dt); }
            r.tables_idx = ti->second;
            r.front_off = (uint32_t)front.size();
            r.item_off = (uint32_t)items.size();
            r.wait_base = (uint32_t)(wait.size() / 2);
            r.waitoff_off = (uint32_t)wait_off.size();
            if (M.terminated) { r.flags = 2; continue; }
            r.flags = M.chart.last().root_done ? 1u : 0u;
            const ScanContext& ctx = M.prep.ctx;
            size_t f0 = front.size();
            for (auto& pl : M.prep.planes) {
                const PlaneInfo& pi = M.cache->planes[(size_t)pl.first];
                uint64_t row = (uint64_t)(uintptr_t)pi.row | ((pl.second || pi.no_uncertain) ? 1u : 0u);
                if (std::find(front.begin() + (long)f0, front.end(), row) == front.end()) front.push_back(row);
            }
            r.front_n = (uint32_t)(front.size() - f0);
            r.item_n = (uint32_t)ctx.items.size();
            r.H = ctx.H;
            items.insert(items.end(), ctx.items.begin(), ctx.items.end());
            wait.insert(wait.end(), ctx.wait.begin(), ctx.wait.end());
            wait_off.insert(wait_off.end(), ctx.wait_off.begin(), ctx.wait_off.end());
        }
        auto align = [](size_t x) { return (x + 255) & ~(size_t)255; };
        size_t o_rows = 0;
        size_t o_front = align(o_rows + rows.size() * sizeof(FillRow));
        size_t o_items = align(o_front + front.size() * sizeof(uint64_t));
        size_t o_wait = align(o_items + items.size() * sizeof(uint32_t));
        size_t o_woff = align(o_wait + wait.size() * sizeof(uint32_t));
        size_t o_tabs = align(o_woff + wait_off.size() * sizeof(uint32_t));
        size_t o_zero = align(o_tabs + tables.size() * sizeof(DevTables));      // overflow-list length and flag
        size_t total = align(o_zero + 4 * sizeof(uint32_t));

        {
            // on the device, after the latest build (the one this call issued, or one a compile call issued on another stream)
            std::lock_guard<std::mutex> ck(build_chain().mu);
            const std::shared_ptr<BuildTicket>& last = build_chain().last;
            if (last && last->state == 0 && last->staging && last->stream != stream) HIP_CHECK(hipStreamWaitEvent(stream, last->staging->ev[4], 0));
        }
        std::lock_guard<std::mutex> ws_lock(fill_ws().mu);
        std::lock_guard<std::mutex> slow_lock(slow().mu);
        auto pack = [&](uint8_t* host) {
            std::memcpy(host + o_rows, rows.data(), rows.size() * sizeof(FillRow));
            if (!front.empty()) std::memcpy(host + o_front, front.data(), front.size() * sizeof(uint64_t));
            if (!items.empty()) std::memcpy(host + o_items, items.data(), items.size() * sizeof(uint32_t));
            if (!wait.empty()) std::memcpy(host + o_wait, wait.data(), wait.size() * sizeof(uint32_t));
            if (!wait_off.empty()) std::memcpy(host + o_woff, wait_off.data(), wait_off.size() * sizeof(uint32_t));
            std::memcpy(host + o_tabs, tables.data(), tables.size() * sizeof(DevTables));
            std::memset(host + o_zero, 0, 4 * sizeof(uint32_t));
        };
        SlowScratch S{};
        FillBatch F{};
        uint8_t* dev = nullptr;
        FillSlot* slot = nullptr;
        if (no_alloc) {
            // everything lives in the fixed array: [staging | candidate words | work lists | row counts | overflow list | item lists]
            if (total > kNoAllocStagingBytes)
                return fail(XG2_EOVERFLOW, "xg2_fill_next_token_bitmask_noalloc: the matchers' parser contexts exceed the fixed staging area");
            NoAllocHost& NH = noalloc_host();
            if (!NH.ready) return fail(XG2_EINVAL, "xg2_fill_next_token_bitmask_noalloc: the library has not been set up on this device");
            void* base = nullptr;
            HIP_CHECK(noalloc_scratch(&base));                       // a table look-up after the first time on a device
            uint8_t* p = static_cast<uint8_t*>(base);
            dev = p; p += kNoAllocStagingBytes;
            F.cand_words = reinterpret_cast<uint32_t*>(p); p += kNoAllocMaskWords * 4;
            F.work_list = reinterpret_cast<uint32_t*>(p); p += kNoAllocMaskWords * 4;
            F.row_count = reinterpret_cast<uint32_t*>(p); p += kNoAllocMaxRows * 4;
            S.list = reinterpret_cast<uint32_t*>(p); S.list_cap = kNoAllocListCap; p += (size_t)kNoAllocListCap * 8;
            S.mem = reinterpret_cast<uint32_t*>(p); S.n_lanes = kNoAllocSlowLanes;
            S.k_cap = slow().k_cap; S.wm_cap = slow().wm_cap;
            const int k = NH.next;
            NH.next ^= 1;
            if (NH.in_flight[k]) { HIP_CHECK(hipEventSynchronize(NH.done[k])); NH.in_flight[k] = false; }   // the call before last has read it
            pack(NH.host[k]);
            upload_pinned(dev, NH.host[k], total, stream);
            HIP_CHECK(hipEventRecord(NH.done[k], stream));
            NH.in_flight[k] = true;
        } else {
            slow().ensure();
            S = slow().s;
            slot = &fill_ws().acquire(total);
            pack(slot->host);
            slot->res_host[0] = 0; slot->res_host[1] = 0;
            std::memset(slot->res_host + 2, 0xFF, 2 * (size_t)kUnresolvedCap * sizeof(uint32_t));
            void* res_dev = nullptr;
            HIP_CHECK(hipHostGetDevicePointer(&res_dev, slot->res_host, 0));
            S.unresolved = static_cast<uint32_t*>(res_dev); S.unresolved_cap = kUnresolvedCap;
            fill_ws().ensure_scratch((size_t)B * V.W, (size_t)B);
            HIP_CHECK(hipEventRecord(fill_ws().t_begin, stream));
            upload_pinned(slot->dev, slot->host, total, stream);
            dev = slot->dev;
            F.cand_words = fill_ws().cand_words.p; F.work_list = fill_ws().work_list.p;
            F.row_count = fill_ws().row_count.p;
        }
        F.rows = reinterpret_cast<const FillRow*>(dev + o_rows); F.B = (uint32_t)B;
        F.front_planes = reinterpret_cast<const uint64_t*>(dev + o_front);
        F.ctx_items = reinterpret_cast<const uint32_t*>(dev + o_items);
        F.ctx_wait = reinterpret_cast<const uint2*>(dev + o_wait);
        F.ctx_wait_off = reinterpret_cast<const uint32_t*>(dev + o_woff);
        F.tables = reinterpret_cast<const DevTables*>(dev + o_tabs);
        F.eos_id = (uint32_t)V.eos;
        S.count = reinterpret_cast<uint32_t*>(dev + o_zero);               // this call's overflow counter and flag, zero on arrival
        launch_fill(F, V.dv, bitmask_dev, row_stride_words, S, stream);
        launch_recheck_slow(F, V.dv, bitmask_dev, row_stride_words, S, stream);
        HIP_CHECK(hipGetLastError());
        fill_ws().last_flags = S.count;
        fill_ws().last_counts = F.row_count;
        fill_ws().last_B = B;
        fill_ws().last_stream = stream;
        fill_ws().timed = !no_alloc;
        fill_ws().any = true;
        if (!no_alloc) {
            HIP_CHECK(hipEventRecord(fill_ws().t_end, stream));
            HIP_CHECK(hipEventRecord(slot->done, stream));
            slot->in_flight = true;
            FillWorkspace::Pending& pd = fill_ws().pending;
            pd.active = true; pd.slot = slot;
            pd.matchers.resize((size_t)B);
            for (int32_t b = 0; b < B; ++b) pd.matchers[(size_t)b] = matchers[b]->p.get();
        }
        return XG2_OK;
    });
}
}  // namespace

extern "C" {

int32_t xg2_fill_next_token_bitmask(xg2_matcher* const* matchers, int32_t B, int32_t* bitmask_dev, int64_t row_stride_words,
                                    void* hip_stream) {
    return fill_common(matchers, B, bitmask_dev, row_stride_words, hip_stream, false);
}

int32_t xg2_fill_next_token_bitmask_noalloc(xg2_matcher* const* matchers, int32_t B, int32_t* bitmask_dev, int64_t row_stride_words,
                                            void* hip_stream) {
    return fill_common(matchers, B, bitmask_dev, row_stride_words, hip_stream, true);
}

int32_t xg2_fill_resolve_overflow(xg2_matcher* const* matchers, int32_t B, int32_t* bitmask_dev, int64_t row_stride_words, int32_t* n_decided) {
    return guarded([&]() -> int32_t {
        if (n_decided) *n_decided = 0;
        if (B < 0 || (B > 0 && (!matchers || !bitmask_dev))) return fail(XG2_EINVAL, "xg2_fill_resolve_overflow: bad argument");
        FillWorkspace& W = fill_ws();
        std::lock_guard<std::mutex> lk(W.mu);
        if (!W.pending.slot) return XG2_OK;
        FillSlot& slot = *W.pending.slot;
        HIP_CHECK(hipEventSynchronize(slot.done));
        W.pending.active = false;
        if (!slot.res_host[0]) return XG2_OK;
        if ((size_t)B != W.pending.matchers.size()) return fail(XG2_EINVAL, "xg2_fill_resolve_overflow: not the batch of the latest fill call");
        for (int32_t b = 0; b < B; ++b)
            if (!matchers[b] || matchers[b]->p.get() != W.pending.matchers[(size_t)b]) return fail(XG2_EINVAL, "xg2_fill_resolve_overflow: not the matchers of the latest fill call");
        if (slot.res_host[1]) return fail(XG2_EOVERFLOW, "xg2_fill_resolve_overflow: more undecided pairs than the list holds");
        int32_t n = 0;
        for (uint32_t k = 0; k < kUnresolvedCap && slot.res_host[2 + 2 * k] != 0xFFFFFFFFu; ++k) {
            const uint32_t b = slot.res_host[2 + 2 * k], id = slot.res_host[3 + 2 * k];
            if (b >= (uint32_t)B) return fail(XG2_EINVAL, "xg2_fill_resolve_overflow: corrupt list");
            MatcherImpl& M = *matchers[b]->p;
            if (id >= (uint32_t)M.vocab->V) return fail(XG2_EINVAL, "xg2_fill_resolve_overflow: corrupt list");
            EarleyChart probe = M.chart;                           // the host parser has no capacity limit
            if (!M.terminated && !M.vocab->special[id] && probe.advance(M.vocab->tok((int32_t)id), M.vocab->len((int32_t)id))) {
                uint32_t word = 0;
                uint32_t* at = reinterpret_cast<uint32_t*>(bitmask_dev) + (size_t)b * (size_t)row_stride_words + (id >> 5);
                HIP_CHECK(hipMemcpy(&word, at, sizeof(word), hipMemcpyDeviceToHost));
                word |= 1u << (id & 31);
                HIP_CHECK(hipMemcpy(at, &word, sizeof(word), hipMemcpyHostToDevice));
            }
            ++n;
        }
        slot.res_host[0] = 0;
        if (n_decided) *n_decided = n;
        return XG2_OK;
    });
}

int32_t xg2_debug_set_build_fusion(int32_t on) {
    build_fusion().store(on != 0);
    return XG2_OK;
}

int32_t xg2_debug_set_large_capacity(int32_t items, int32_t wait_entries) {
    for (SlowImpl* si : {&slow(), &build_slow()}) {
        std::lock_guard<std::mutex> slow_lock(si->mu);
        si->k_cap = items <= 0 ? kSlowK : std::min<uint32_t>((uint32_t)items, kSlowK);
        si->wm_cap = wait_entries <= 0 ? kSlowWM : std::min<uint32_t>((uint32_t)wait_entries, kSlowWM);
    }
    return XG2_OK;
}

int32_t xg2_fill_last_device_us(float* out) {
    return guarded([&]() -> int32_t {
        if (!out) return fail(XG2_EINVAL, "xg2_fill_last_device_us: null out");
        std::lock_guard<std::mutex> ws_lock(fill_ws().mu);
        if (!fill_ws().timed) return fail(XG2_EINVAL, "xg2_fill_last_device_us: the latest fill call recorded no events (none yet, or the one that allocates nothing)");
        HIP_CHECK(hipEventSynchronize(fill_ws().t_end));
        float ms = 0.f;
        HIP_CHECK(hipEventElapsedTime(&ms, fill_ws().t_begin, fill_ws().t_end));
        *out = ms * 1e3f;
        return XG2_OK;
    });
}

int32_t xg2_fill_last_status(int32_t* large_capacity_tokens, int32_t* overflowed) {
    return guarded([&]() -> int32_t {
        std::lock_guard<std::mutex> ws_lock(fill_ws().mu);
        if (!fill_ws().any) return fail(XG2_EINVAL, "xg2_fill_last_status: no fill call yet");
        fill_ws().wait_last();
        uint32_t words[2] = {0, 0};
        HIP_CHECK(hipMemcpy(words, fill_ws().last_flags, sizeof(words), hipMemcpyDeviceToHost));
        if (large_capacity_tokens) *large_capacity_tokens = (int32_t)words[0];
        if (overflowed) *overflowed = words[1] ? 1 : 0;
        return XG2_OK;
    });
}

int32_t xg2_fill_last_recheck_tokens(int32_t* tokens_host, int32_t cap, int32_t* n_rows) {
    return guarded([&]() -> int32_t {
        if (cap < 0 || (cap > 0 && !tokens_host)) return fail(XG2_EINVAL, "xg2_fill_last_recheck_tokens: bad argument");
        std::lock_guard<std::mutex> ws_lock(fill_ws().mu);
        if (!fill_ws().any) return fail(XG2_EINVAL, "xg2_fill_last_recheck_tokens: no fill call yet");
        fill_ws().wait_last();
        const int32_t n = std::min(cap, fill_ws().last_B);
        if (n > 0) HIP_CHECK(hipMemcpy(tokens_host, fill_ws().last_counts, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToHost));
        if (n_rows) *n_rows = fill_ws().last_B;
        return XG2_OK;
    });
}

int32_t xg2_apply_token_bitmask(void* logits_dev, int32_t dtype, int32_t B, int32_t V, int64_t row_stride_elems,
                                const int32_t* bitmask_dev, int64_t bm_row_stride_words, void* hip_stream) {
    return guarded([&]() -> int32_t {
        if (B < 0 || V < 0 || (dtype != XG2_F32 && dtype != XG2_BF16)) return fail(XG2_EINVAL, "xg2_apply_token_bitmask: bad argument");
        if (B == 0 || V == 0) return XG2_OK;
        if (!logits_dev || !bitmask_dev || row_stride_elems < V || bm_row_stride_words < (V + 31) / 32)
            return fail(XG2_EINVAL, "xg2_apply_token_bitmask: null buffer or stride smaller than the row");
        require_device();
        launch_apply(logits_dev, dtype, B, V, row_stride_elems, bitmask_dev, bm_row_stride_words, (hipStream_t)hip_stream);
        HIP_CHECK(hipGetLastError());
        return XG2_OK;
    });
}

// ---- matchers on the device ---------------------------------------------------------------------------------------

int32_t xg2_batch_create(xg2_vocab* vocab, int32_t B, xg2_batch** out) {
    return guarded([&]() -> int32_t {
        if (!vocab || !out || B <= 0 || B > (1 << 20)) return fail(XG2_EINVAL, "xg2_batch_create: bad argument");
        vocab->p->ensure_device();
        auto b = std::make_unique<BatchImpl>();
        b->vocab = vocab->p;
        b->B = B;
        const size_t n = (size_t)B;
        b->rows.alloc(n); b->front.alloc(n * BatchImpl::KF); b->slow_front.alloc(n * BatchImpl::KF);
        b->items.alloc(2 * n * BatchImpl::KI); b->wait.alloc(2 * n * BatchImpl::KW); b->wait_off.alloc(2 * n * (BatchImpl::KH + 1));
        b->slow_mem.alloc(n * kSlowSlots); b->slow_map.alloc(n * (BatchImpl::KH + kSlowMaxLen + 1));
        b->flag_words.alloc(8);
        b->caches_dev.alloc(BatchImpl::kMaxCaches); b->tables_dev.alloc(BatchImpl::kMaxCaches);
        b->row_list.alloc(n);
        HIP_CHECK(hipMemset(b->rows.p, 0, n * sizeof(FillRow)));
        HIP_CHECK(hipMemset(b->flag_words.p, 0, 8 * sizeof(uint32_t)));
        b->assigned.assign(n, 0);
        BatchDev& d = b->d;
        d.B = (uint32_t)B; d.KI = BatchImpl::KI; d.KH = BatchImpl::KH; d.KW = BatchImpl::KW; d.KF = BatchImpl::KF;
        d.rows = b->rows.p; d.front = b->front.p; d.items = b->items.p; d.wait = b->wait.p; d.wait_off = b->wait_off.p;
        d.caches = b->caches_dev.p; d.tables = b->tables_dev.p;
        d.slow_mem = b->slow_mem.p; d.slow_map = b->slow_map.p; d.slow_front = b->slow_front.p;
        *out = new xg2_batch{std::move(b)};
        return XG2_OK;
    });
}
void xg2_batch_destroy(xg2_batch* b) {
    if (b) (void)hipDeviceSynchronize();                        // kernels may still be reading the slots
    delete b;
}

int32_t xg2_batch_assign(xg2_batch* batch, const int32_t* rows_host, int32_t n, const xg2_mask_cache* cache, void* hip_stream) {
    return guarded([&]() -> int32_t {
        if (!batch || !cache || n < 0) return fail(XG2_EINVAL, "xg2_batch_assign: bad argument");
        BatchImpl& Bt = *batch->p;
        std::lock_guard<std::mutex> lk(Bt.mu);
        if (cache->p->vocab.get() != Bt.vocab.get()) return fail(XG2_EINVAL, "xg2_batch_assign: the cache was compiled for another vocabulary");
        if (!rows_host) n = Bt.B;
        if (n > Bt.B) return fail(XG2_EINVAL, "xg2_batch_assign: more rows than slots");
        for (int32_t k = 0; rows_host && k < n; ++k)
            if (rows_host[k] < 0 || rows_host[k] >= Bt.B) return fail(XG2_EINVAL, "xg2_batch_assign: row out of range");
        if (n == 0) return XG2_OK;
        hipStream_t stream = (hipStream_t)hip_stream;
        ensure_cache_on_device(cache->p);
        const CacheImpl::OnDevice& od = cache->p->on_device;
        if (od.cd.start_n_items > BatchImpl::KI || od.cd.start_H > BatchImpl::KH || od.n_start_wait > BatchImpl::KW || od.cd.start_n_front > BatchImpl::KF)
            return fail(XG2_EOVERFLOW, "xg2_batch_assign: the grammar's start state exceeds a matcher slot");
        size_t ci = 0;
        while (ci < Bt.caches.size() && Bt.caches[ci].get() != cache->p.get()) ++ci;
        if (ci == Bt.caches.size()) {
            if (ci >= BatchImpl::kMaxCaches) return fail(XG2_EOVERFLOW, "xg2_batch_assign: too many different caches in one batch");
            Bt.caches.push_back(cache->p);                      // kept alive while the batch lives
            HIP_CHECK(hipMemcpyAsync(Bt.caches_dev.p + ci, &od.cd, sizeof(CacheDev), hipMemcpyHostToDevice, stream));
            HIP_CHECK(hipMemcpyAsync(Bt.tables_dev.p + ci, &od.cd.T, sizeof(DevTables), hipMemcpyHostToDevice, stream));
        }
        if (rows_host) HIP_CHECK(hipMemcpyAsync(Bt.row_list.p, rows_host, (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice, stream));
        launch_batch_assign(Bt.d, rows_host ? Bt.row_list.p : nullptr, (uint32_t)n, (uint32_t)ci, stream);
        HIP_CHECK(hipGetLastError());
        HIP_CHECK(hipStreamSynchronize(stream));                // row_list and the host arrays may be reused by the next call
        for (int32_t k = 0; k < n; ++k) {
            uint8_t& a = Bt.assigned[(size_t)(rows_host ? rows_host[k] : k)];
            if (!a) { a = 1; ++Bt.n_assigned; }
        }
        return XG2_OK;
    });
}

int32_t xg2_batch_accept_tokens(xg2_batch* batch, const int32_t* token_ids_dev, int32_t* status_dev, void* hip_stream) {
    return guarded([&]() -> int32_t {
        if (!batch || !token_ids_dev) return fail(XG2_EINVAL, "xg2_batch_accept_tokens: bad argument");
        BatchImpl& Bt = *batch->p;
        std::lock_guard<std::mutex> lk(Bt.mu);
        if (Bt.n_assigned != Bt.B) return fail(XG2_EINVAL, "xg2_batch_accept_tokens: every slot needs a cache first (xg2_batch_assign)");
        launch_accept(Bt.d, Bt.vocab->dv, (uint32_t)Bt.vocab->eos, token_ids_dev, status_dev, (hipStream_t)hip_stream);
        HIP_CHECK(hipGetLastError());
        return XG2_OK;
    });
}

int32_t xg2_batch_fill_next_token_bitmask(xg2_batch* batch, int32_t* bitmask_dev, int64_t row_stride_words, void* hip_stream) {
    return guarded([&]() -> int32_t {
        if (!batch || !bitmask_dev) return fail(XG2_EINVAL, "xg2_batch_fill_next_token_bitmask: bad argument");
        BatchImpl& Bt = *batch->p;
        std::lock_guard<std::mutex> lk(Bt.mu);
        VocabImpl& V = *Bt.vocab;
        if (row_stride_words < (int64_t)V.W) return fail(XG2_EINVAL, "xg2_batch_fill_next_token_bitmask: row stride smaller than ceil(V/32)");
        if (Bt.n_assigned != Bt.B) return fail(XG2_EINVAL, "xg2_batch_fill_next_token_bitmask: every slot needs a cache first (xg2_batch_assign)");
        hipStream_t stream = (hipStream_t)hip_stream;
        std::lock_guard<std::mutex> ws_lock(fill_ws().mu);
        std::lock_guard<std::mutex> slow_lock(slow().mu);
        slow().ensure();
        SlowScratch S = slow().s;
        fill_ws().ensure_scratch((size_t)Bt.B * V.W, (size_t)Bt.B);
        FillBatch F{};
        F.rows = Bt.d.rows; F.B = (uint32_t)Bt.B;
        F.front_planes = Bt.d.front; F.ctx_items = Bt.d.items; F.ctx_wait = Bt.d.wait; F.ctx_wait_off = Bt.d.wait_off;
        F.tables = Bt.d.tables;
        F.eos_id = (uint32_t)V.eos;
        F.cand_words = fill_ws().cand_words.p; F.work_list = fill_ws().work_list.p; F.row_count = fill_ws().row_count.p;
        // nothing is uploaded: two sets of counter words take turns, each call's last kernel clears the set of the next call
        S.count = Bt.flag_words.p + 4 * Bt.flag_turn;
        Bt.flag_turn ^= 1;
        F.zero_words = Bt.flag_words.p + 4 * Bt.flag_turn;
        S.mark_rows = Bt.d.rows;                                // an undecided pair makes its slot unusable: the next accept says so
        HIP_CHECK(hipEventRecord(fill_ws().t_begin, stream));
        launch_fill(F, V.dv, bitmask_dev, row_stride_words, S, stream);
        launch_recheck_slow(F, V.dv, bitmask_dev, row_stride_words, S, stream);
        HIP_CHECK(hipGetLastError());
        HIP_CHECK(hipEventRecord(fill_ws().t_end, stream));
        fill_ws().last_flags = S.count; fill_ws().last_counts = F.row_count; fill_ws().last_B = Bt.B; fill_ws().last_stream = stream;
        fill_ws().timed = true; fill_ws().any = true;
        return XG2_OK;
    });
}

int32_t xg2_batch_row_info(xg2_batch* batch, int32_t row, int32_t* info_host) {
    return guarded([&]() -> int32_t {
        if (!batch || !info_host || row < 0 || row >= batch->p->B) return fail(XG2_EINVAL, "xg2_batch_row_info: bad argument");
        BatchImpl& Bt = *batch->p;
        std::lock_guard<std::mutex> lk(Bt.mu);
        HIP_CHECK(hipDeviceSynchronize());
        FillRow r;
        HIP_CHECK(hipMemcpy(&r, Bt.rows.p + row, sizeof(r), hipMemcpyDeviceToHost));
        uint32_t n_wait = 0;
        HIP_CHECK(hipMemcpy(&n_wait, Bt.wait_off.p + r.waitoff_off + r.H, sizeof(uint32_t), hipMemcpyDeviceToHost));
        info_host[0] = (r.flags & 1u) ? 1 : 0; info_host[1] = (r.flags & 2u) ? 1 : 0; info_host[2] = (int32_t)r.pad[1];
        info_host[3] = (int32_t)r.H; info_host[4] = (int32_t)r.item_n; info_host[5] = (int32_t)n_wait; info_host[6] = (int32_t)r.front_n;
        info_host[7] = Bt.assigned[(size_t)row] ? (int32_t)r.tables_idx : -1;
        return XG2_OK;
    });
}

}  // extern "C"
