/*
 * xg2mask -- token-mask cache for grammar-constrained decoding on AMD MI355X (gfx950).
 *
 * C ABI of the library (libxg2mask.so).  The calls follow the statement of the problem in
 * XGrammar-2 (arXiv 2601.04426):
 *
 *   compile_grammar(ebnf, vocab) -> mask_cache          section 3.4 (Earley-based adaptive token
 *                                                       mask cache), section 3.3 (cross-grammar cache)
 *   fill_next_token_bitmask(matchers[B], bitmask[B, ceil(V/32)])
 *                                                       section 3.4 last paragraph and the appendix
 *                                                       "XGrammar's Adaptive Token Mask cache
 *                                                       Generation Algorithm" (runtime combination)
 *   apply_token_bitmask(logits[B, V], bitmask)          section 2.1 (invalid tokens get -infinity)
 *
 * Conventions
 *   - Every call returns an int32 status: XG2_OK or a negative XG2_E* code; the text of the last
 *     error of the calling thread is returned by xg2_last_error().
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory of the
 *     current device.  The library never frees or keeps a caller's device buffer.
 *   - Handles are created and destroyed by the library.  A mask cache keeps its vocabulary and
 *     grammar alive; a matcher keeps its grammar (and cache) alive.
 *   - Bit v%32 (least significant bit = 0) of int32 word v/32 stands for token v; 1 = allowed;
 *     bits at or beyond V in the last word are 0.
 *   - Device work is enqueued on the HIP stream given by the caller (a hipStream_t passed as
 *     void*, NULL = the default stream); compile, fill, accept and apply all return as soon as their
 *     work is enqueued.  Cache builds follow one another on the device whatever their streams (the
 *     library orders them with events), and a fill waits on the device for the builds enqueued before
 *     it, so a build may run on one stream while fill and apply of other caches run on another.  Fill
 *     calls share one scratch: keep them on one stream (or order their streams).  apply has no state.
 *   - There is no CPU fallback: without a usable HIP device every call that needs one fails
 *     with XG2_EHIP.
 */
#ifndef XG2MASK_H
#define XG2MASK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define XG2_OK          0
#define XG2_EINVAL     (-1)   /* bad argument, ill-formed vocabulary, unproductive grammar, ...   */
#define XG2_EPARSE     (-2)   /* EBNF syntax error (line number in xg2_last_error())              */
#define XG2_EREJECTED  (-3)   /* accept_token: token not allowed here; matcher state unchanged    */
#define XG2_EOVERFLOW  (-4)   /* an internal capacity was exceeded; nothing partial is returned   */
#define XG2_EHIP       (-5)   /* HIP runtime error or no device                                   */

typedef struct xg2_vocab xg2_vocab;
typedef struct xg2_grammar xg2_grammar;
typedef struct xg2_pool xg2_pool;
typedef struct xg2_mask_cache xg2_mask_cache;
typedef struct xg2_matcher xg2_matcher;

/* Options of xg2_compile_grammar (NULL = defaults).
 * context_depth 1: one plane pair per scannable position (rule, state), the cache of section 3.4 as it stands.
 * context_depth 2 (default): a position of a referenced rule is cached once per distinct state the
 *   referencing rule continues in, i.e. with one level of the reference structure built into the
 *   plane (the context expansion that section 2.2 and section 3.3 recall); far fewer tokens stay
 *   uncertain.  Positions of the root rule have no referencing rule and keep a plain plane.
 * merge_equivalent (default 1): states that no string as long as the longest token can tell apart
 *   share one plane (section 3.6: states inside a repetition differ minimally).  States that no
 *   string of at most d bytes (3 <= d <= 32) can tell apart have equal planes on the tokens of at
 *   most d bytes: such a plane is checked for its longer tokens only and takes the others from the
 *   plane it agrees with.  Likewise a plain automaton state that moves like its rule's start state
 *   on most first bytes (the states of a dispatch automaton) is checked only for the tokens with
 *   the other first bytes, and the planes of one state under several referencing sites share the
 *   tokens that cannot leave the rule.  The planes are the same with or without the option.
 * follow_filter (default 1): a token that leaves the plane's (outermost) rule before its last byte
 *   stays uncertain only if the rest of the token is a viable prefix of what can follow that rule
 *   at some reference site of the grammar; otherwise it is rejected at build time (sections 2.2 and
 *   3.3: the reference structure / lookahead is used to reject context-dependent tokens).  Planes
 *   built with the filter are shared between grammars only where the follow sets agree.
 * jit (default 0): 1 = just-in-time compilation (section 3.5): xg2_compile_grammar builds only the
 *   jit_prebuild planes with the largest estimated cost; every other plane is built by the first
 *   xg2_fill_next_token_bitmask call whose matchers reach it (looked up in the pool first), on that
 *   call's stream, before the masks are filled.  The masks are the same either way.
 * partial_hits (default 1; with follow_filter and a pool): a plane whose structure (rule, state, referencing state)
 *   the pool already holds under another follow language is not built from scratch (section 3.3, partial cache
 *   hit): its accepted tokens are copied, and only the tokens that leave the rule early and die -- every plane
 *   keeps them in a third row -- are run again, against this grammar's follow language.  Same planes either way. */
typedef struct xg2_compile_opts {
    int32_t context_depth;
    int32_t merge_equivalent;
    int32_t follow_filter;
    int32_t jit;
    int32_t jit_prebuild;
    int32_t partial_hits;
    int32_t time_kernel;      /* measurement aid: also time the classification kernel alone (xg2_compile_stats.kernel_ms); the two
                                 extra events sit between the kernels of the build and lengthen device_ms by a few microseconds */
} xg2_compile_opts;

/* Counters filled by xg2_compile_grammar. */
typedef struct xg2_compile_stats {
    int64_t positions;        /* scannable (rule, state) positions of the grammar                 */
    int64_t unique;           /* distinct planes this grammar uses (after dedupe and merging)     */
    int64_t built;            /* planes computed by this call (pool misses)                       */
    int64_t partial_hits;     /* of those: derived from a plane of the same structure (section 3.3) */
    int64_t checks;           /* (built - partial_hits) * (number of checkable tokens): logical (plane, token) pairs */
    int64_t executed_checks;  /* (plane, token) pairs a lane actually stepped through (not the
                                 tokens skipped by their first byte or taken from another plane)  */
    int64_t executed_token_bytes; /* summed token lengths over the executed pairs                     */
    int64_t slow_path;        /* pairs finished by the large-capacity kernel                      */
    int64_t n_accepted;       /* set bits over the built accepted planes                          */
    int64_t n_uncertain;      /* set bits over the built uncertain planes                         */
    double  host_lower_ms;    /* EBNF -> tables and work plan on the host                         */
    double  device_ms;        /* first clear / table upload -> last plane written and summarised (HIP events) */
    double  kernel_ms;        /* the classification kernel alone (HIP events around its launch); 0 unless time_kernel was set */
} xg2_compile_stats;

const char* xg2_last_error(void);

/* ---- vocabulary -------------------------------------------------------------------------------
 * bytes/offsets: host CSR in token-id order, token i = bytes[offsets[i] .. offsets[i+1]).  The
 * library copies it, sorts the tokens by bytes and (at first use on a device) lays the sorted
 * CSR out in device memory.  eos_id is the end-of-sequence token; special_ids (host, may be
 * NULL) are never allowed by a mask, and neither are zero-length tokens.                        */
int32_t xg2_vocab_create(const uint8_t* bytes, const uint64_t* offsets, int32_t V, int32_t eos_id,
                         const int32_t* special_ids, int32_t n_special, xg2_vocab** out);
void    xg2_vocab_destroy(xg2_vocab*);

/* ---- grammar (host only; no device needed) ----------------------------------------------------
 * Lowers EBNF text (section 2.1; TagDispatch of section 3.2; repetition X{m,n} of section 3.6)
 * to one canonical minimal byte-level automaton per rule (section 3.3) and hashes the rules
 * (Algorithm 1; Algorithm 2 for simple reference cycles).  ebnf need not be NUL-terminated.     */
int32_t xg2_grammar_create(const char* ebnf, size_t len, const char* root_rule, xg2_grammar** out);
void    xg2_grammar_destroy(xg2_grammar*);
/* JSON description of the lowered automata (rules, states, byte ranges, rule edges, hashes,
 * positions).  Writes at most cap bytes incl. the NUL; *needed receives the full size.          */
int32_t xg2_grammar_describe(const xg2_grammar*, char* buf, size_t cap, size_t* needed);
int32_t xg2_grammar_num_positions(const xg2_grammar*, int32_t* out);

/* ---- cross-grammar pool (section 3.3) ---------------------------------------------------------
 * Planes of structurally identical rule positions are built once and shared by every grammar
 * compiled with the same pool and vocabulary.  max_bytes bounds the device memory of the pool
 * (0 = unbounded).  When it is reached, planes that no live mask cache uses are given up, least
 * recently used first, and built again if a later grammar needs them; if every plane is in use,
 * compile (or a just-in-time fill) fails with XG2_EOVERFLOW.                                     */
int32_t xg2_pool_create(size_t max_bytes, xg2_pool** out);
void    xg2_pool_destroy(xg2_pool*);
int32_t xg2_pool_stats(const xg2_pool*, int64_t* n_positions, int64_t* device_bytes);

/* ---- compile_grammar(ebnf, vocab) -> mask_cache ------------------------------------------------
 * Builds, on the device, the accepted and uncertain bit planes [W = ceil(V/32) int32 words each]
 * of every plane of the grammar that the pool (nullable) does not hold yet.  A plane belongs to a
 * position (rule, state), or to a position plus the state (parent rule, parent state) in which the
 * referencing rule continues once the position's rule instance ends:
 *   accepted  = tokens that are a prefix of a string of Suf(position) [. Suf(parent)],
 *   uncertain = the other tokens with a proper non-empty prefix that is a whole such string
 *               (and, with follow_filter, a rest that some reference site can continue).
 * opts and stats may be NULL.  The call returns once the build is enqueued on hip_stream; stats then
 * holds what the host knows (positions, planes, checks, executed checks, host time) and zeros for what
 * the device reports (xg2_mask_cache_stats waits and gives everything).                          */
int32_t xg2_compile_grammar(xg2_vocab* vocab, const char* ebnf, size_t len, const char* root_rule,
                            const xg2_compile_opts* opts, xg2_pool* pool, void* hip_stream,
                            xg2_mask_cache** out, xg2_compile_stats* stats);
void    xg2_mask_cache_destroy(xg2_mask_cache*);
/* xg2_compile_grammar returns when the build is enqueued; this call waits for it and gives the full statistics.  It is
 * also where a failed build is reported: XG2_EOVERFLOW if item sets exceeded even the large-capacity lists (so do
 * xg2_mask_cache_get_planes, xg2_batch_assign and fill calls on such a cache; nothing partial is ever served).          */
int32_t xg2_mask_cache_stats(xg2_mask_cache*, xg2_compile_stats* stats);
int32_t xg2_mask_cache_num_positions(const xg2_mask_cache*, int32_t* out);
int32_t xg2_mask_cache_num_planes(const xg2_mask_cache*, int32_t* out);
/* Just-in-time caches: planes that hold a row by now, build launches issued by fill calls so far and
 * their summed device time in milliseconds (each argument may be NULL).                          */
int32_t xg2_mask_cache_jit_stats(const xg2_mask_cache*, int32_t* n_built, int32_t* n_builds_in_fill, double* device_ms_in_fill);
/* The representative the planes of index k were built for.  Names stay valid while the cache lives;
 * *parent_rule is NULL (and *parent_state -1) for a plane without context.                        */
int32_t xg2_mask_cache_plane_info(const xg2_mask_cache*, int32_t k, const char** rule, int32_t* state,
                                  const char** parent_rule, int32_t* parent_state);
/* Index of the plane used for (rule, state) [inside (parent_rule, parent_state); parent_rule NULL =
 * no context]; *k = -1 if the cache holds no plane for that combination.                          */
int32_t xg2_mask_cache_find_plane(const xg2_mask_cache*, const char* rule, int32_t state,
                                  const char* parent_rule, int32_t parent_state, int32_t* k);
/* Copies plane k to host arrays of W int32 words each (synchronises).  XG2_EINVAL if the plane has
 * not been built yet (just-in-time cache).                                                        */
int32_t xg2_mask_cache_get_planes(const xg2_mask_cache*, int32_t k, int32_t* accepted_host, int32_t* uncertain_host);

/* ---- matchers (one per sequence) ---------------------------------------------------------------
 * A matcher follows the output with an Earley parser (section 3.4, appendix on Earley parsing).
 * xg2_matcher_create_host makes a matcher that can accept tokens and report its frontier but
 * cannot be passed to fill (no cache).                                                          */
int32_t xg2_matcher_create(const xg2_mask_cache*, xg2_matcher** out);
int32_t xg2_matcher_create_host(const xg2_grammar*, const xg2_vocab*, xg2_matcher** out);
void    xg2_matcher_destroy(xg2_matcher*);
int32_t xg2_matcher_accept_token(xg2_matcher*, int32_t token_id);
/* One token for each of B matchers (the sampled tokens of a decoding step; section 3.4: the parser traces
 * the output).  token_ids[b] < 0 skips matcher b.  status_host[b] receives what xg2_matcher_accept_token
 * would have returned for matcher b; the call itself fails only on bad arguments.  The matchers must be
 * distinct; several host threads share the work (a small pool that the library starts at the first
 * such call and keeps until the process ends).                                                     */
int32_t xg2_matcher_accept_tokens(xg2_matcher* const* matchers, const int32_t* token_ids, int32_t B, int32_t* status_host);
int32_t xg2_matcher_reset(xg2_matcher*);
int32_t xg2_matcher_is_terminated(const xg2_matcher*, int32_t* out);
/* Position indices (into the grammar's position list) of the scannable items of the current
 * closed Earley set (at most cap are written, *n receives the count) and whether the root rule
 * can end here.                                                                                 */
int32_t xg2_matcher_frontier(const xg2_matcher*, int32_t* positions_host, int32_t cap, int32_t* n,
                             int32_t* can_end);

/* ---- fill_next_token_bitmask(matchers[B], bitmask[B, ceil(V/32)] int32) ------------------------
 * For every matcher b: bitmask[b] = union of the accepted planes of its frontier (each scannable
 * item, with its referencing item at context depth 2), plus every token that is uncertain
 * somewhere in the frontier and passes a re-check against the matcher's full Earley context, plus
 * the end-of-sequence bit if the root rule can end.  A terminated
 * matcher gets a row allowing only end-of-sequence.  matchers: host array of B handles that
 * share one vocabulary (their caches may differ).  bitmask_dev: device, B rows of
 * row_stride_words int32 (row_stride_words >= W).                                               */
int32_t xg2_fill_next_token_bitmask(xg2_matcher* const* matchers, int32_t B, int32_t* bitmask_dev,
                                    int64_t row_stride_words, void* hip_stream);

/* The same masks for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  This call allocates and frees nothing (no hipMalloc, no hipFree, no pinned memory, no
 * event): its device scratch (staging of the per-row records, candidate words, work lists, the large-capacity item lists)
 * is one fixed array of 13 MiB per GPU that the library holds until the process ends, and its two pinned host buffers are
 * made when the first vocabulary is laid out on the device.  Limits per call: B <= 4096 rows, B * ceil(V/32) <= 2^20 mask
 * words, 1 MiB of per-row records (frontier planes and parser contexts); beyond them the call fails with XG2_EOVERFLOW and
 * enqueues nothing.  Every plane the frontiers need must have been built (XG2_EINVAL otherwise: a cache compiled just in time
 * builds, and therefore allocates, inside xg2_fill_next_token_bitmask only).  All calls on one GPU share the one array,
 * which keeps the previous call's contents (what must start at zero is cleared by the call itself): calls whose device work
 * overlaps on one GPU race, so keep them on one stream or order them with events.  Arguments, bitmask layout and errors are
 * otherwise those of xg2_fill_next_token_bitmask; xg2_fill_last_status and xg2_fill_last_recheck_tokens work after it (they
 * wait for the stream), xg2_fill_last_device_us does not (no events are recorded).                                          */
int32_t xg2_fill_next_token_bitmask_noalloc(xg2_matcher* const* matchers, int32_t B, int32_t* bitmask_dev,
                                            int64_t row_stride_words, void* hip_stream);

/* Measurement aid: device time in microseconds of the work the latest fill call of this process enqueued
 * (context upload, plane union, re-check), from HIP events on its stream.  Waits for that work.   */
int32_t xg2_fill_last_device_us(float* out);

/* What became of the re-checks of the latest fill call of this process (waits for its device work): how
 * many (row, token) pairs needed the large-capacity kernel, and whether one of them exceeded even its
 * item lists (256 items, 1024 wait entries, tokens of 1024 bytes) -- such a token's bit is left 0 although
 * the token might be allowed.  fill itself returns before the device work runs and cannot report this.   */
int32_t xg2_fill_last_status(int32_t* large_capacity_tokens, int32_t* overflowed);

/* A fill call returns before its kernels run, so it cannot itself report that the large-capacity re-check left a (row,
 * token) pair undecided.  It is reported by the next call instead: the next xg2_fill_next_token_bitmask,
 * xg2_matcher_accept_token or xg2_matcher_accept_tokens call of the process fails with XG2_EOVERFLOW, once, and changes
 * nothing (for matchers on the device: the slot is marked and its next accept answers XG2_EOVERFLOW).  To get the exact
 * mask instead, call xg2_fill_resolve_overflow after the fill, with the same matchers and bitmask, before the mask is
 * used: it waits for the fill, decides every listed pair with the host parser (which has no capacity limit), sets the bits
 * of the allowed ones in bitmask_dev and clears the pending error.  *n_decided (nullable) = pairs looked at (0 almost
 * always).  Not for xg2_fill_next_token_bitmask_noalloc (use xg2_fill_last_status there) nor for xg2_batch_*.          */
int32_t xg2_fill_resolve_overflow(xg2_matcher* const* matchers, int32_t B, int32_t* bitmask_dev, int64_t row_stride_words,
                                  int32_t* n_decided);

/* Test aid: on = 0 makes the builds that follow use one launch per step (clearing of rows, upload, chunk records; copy
 * kernels of derived planes, per-plane summary) also where the library would otherwise do them in one launch each; on = 1
 * (the default) restores that.  The planes are the same either way.                                                    */
int32_t xg2_debug_set_build_fusion(int32_t on);

/* Test aid: lowers the capacities of the large-capacity item lists (256 items, 1024 wait entries; 0 = back to these) for
 * the build and fill calls that follow, so that the handling of their overflow can be exercised with small grammars.   */
int32_t xg2_debug_set_large_capacity(int32_t items, int32_t wait_entries);

/* Measurement and test aid: for each row of the latest fill call of this process (waits for its device work), the
 * number of candidate tokens, i.e. tokens that are uncertain in a plane of the row's frontier and therefore went through
 * the full-context re-check (section 3.4, runtime part).  tokens_host: host array; at most cap entries are written;
 * *n_rows (nullable) receives the batch size.                                                                        */
int32_t xg2_fill_last_recheck_tokens(int32_t* tokens_host, int32_t cap, int32_t* n_rows);

/* ---- matchers that live on the device (section 3.4 and the appendix on Earley parsing: the parser that traces the
 * output, one per sequence) ------------------------------------------------------------------------------------------
 * A batch holds B matcher slots in device memory: per slot the scannable items of the current closed Earley set, what the
 * waiting items of every older set still reachable wait for, and the planes of the scannable frontier.  A decoding step
 * then needs nothing from the host: xg2_batch_accept_tokens runs the sampled tokens (a device array, e.g. the sampler's
 * output) through the Earley recogniser, one lane per slot, and leaves each slot's next state in place;
 * xg2_batch_fill_next_token_bitmask reads the slots directly.  Both only enqueue kernels on the caller's stream.
 * Capacities of a slot: 64 scannable items, 240 reachable sets, 512 wait entries, 32 frontier planes (a grammar whose
 * parse needs more, e.g. deeply right-recursive rules, makes the slot fail with XG2_EOVERFLOW until it is reassigned: use
 * host matchers for it).  Caches compiled just in time are not accepted (XG2_EINVAL): every plane must exist.            */
typedef struct xg2_batch xg2_batch;
int32_t xg2_batch_create(xg2_vocab* vocab, int32_t B, xg2_batch** out);
void    xg2_batch_destroy(xg2_batch*);
/* Slots rows_host[0 .. n) (host array; NULL = all B slots) start a new sequence of `cache`, which the batch keeps alive; at
 * most 256 different caches per batch.  Waits for the assignment to finish.                                              */
int32_t xg2_batch_assign(xg2_batch*, const int32_t* rows_host, int32_t n, const xg2_mask_cache* cache, void* hip_stream);
/* token_ids_dev: device, B int32: the token slot b accepts; -1 = none for this slot; -2 = slot b starts a new sequence of its
 * cache.  status_dev (device, B int32, may be NULL) receives per slot what xg2_matcher_accept_token would return: XG2_OK,
 * XG2_EREJECTED (state unchanged), XG2_EINVAL (terminated, or id out of range), XG2_EOVERFLOW (slot capacity exceeded; sticky
 * until the slot is reset or reassigned).  Accepting the end-of-sequence token where the root rule can end terminates the slot.  */
int32_t xg2_batch_accept_tokens(xg2_batch*, const int32_t* token_ids_dev, int32_t* status_dev, void* hip_stream);
/* The masks of xg2_fill_next_token_bitmask for the B slots, row b for slot b; nothing is uploaded.                        */
int32_t xg2_batch_fill_next_token_bitmask(xg2_batch*, int32_t* bitmask_dev, int64_t row_stride_words, void* hip_stream);
/* Test aid (synchronises): info_host[8] = {root can end, terminated, sticky error, reachable sets, scannable items, wait
 * entries, frontier planes, index of the slot's cache in the batch or -1}.                                               */
int32_t xg2_batch_row_info(xg2_batch*, int32_t row, int32_t* info_host);

/* ---- apply_token_bitmask(logits[B, V], bitmask) -------------------------------------------------
 * In place: logits[b, v] = -infinity where bit v of bitmask row b is 0; other elements keep
 * their bit pattern.  dtype: XG2_F32 or XG2_BF16.  logits_dev: device, B rows of
 * row_stride_elems elements.  bitmask_dev: device, B rows of bm_row_stride_words int32.         */
#define XG2_F32  0
#define XG2_BF16 1
int32_t xg2_apply_token_bitmask(void* logits_dev, int32_t dtype, int32_t B, int32_t V, int64_t row_stride_elems,
                                const int32_t* bitmask_dev, int64_t bm_row_stride_words, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XG2MASK_H */
