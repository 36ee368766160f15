/*
 * CPU ORACLE -- test infrastructure only.  Nothing in the product path may call this.
 *
 * A textbook Earley recogniser (Earley 1970; the predict / scan / complete operations the
 * paper recalls in its appendix "Earley's Parsing Algorithm") over a byte-level context-free
 * grammar given as plain BNF productions.  Terminals are sets of byte values.  Empty
 * productions are handled the standard way (Aycock & Horspool 2002): when a nullable
 * nonterminal is predicted, the predicting item is also advanced over it.
 *
 * With it, written straight from the definitions:
 *   - viable-prefix test: history.token is a prefix of a sentence  <=> the item set after its
 *     last byte is non-empty (the grammar must be reduced: every nonterminal productive);
 *   - token classes of a cache position (paper section 3.4 and the appendix on the adaptive
 *     token mask cache): accepted = token is a viable prefix of the position's suffix language,
 *     uncertain = not accepted and some proper non-empty prefix of the token is a complete
 *     sentence of that language, rejected = neither.
 *
 * No sorting of the vocabulary, no tries, no bit tricks, no table sharing with the GPU
 * library: one independent parse per token.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct { int32_t prod, dot, origin; } Item;
typedef struct { Item* it; int32_t n, cap; } Set;

typedef struct {
    int32_t n_nt, n_prod, n_tset;
    int32_t* lhs;        /* [n_prod]                                   */
    int32_t* off;        /* [n_prod+1] into syms                       */
    int32_t* syms;       /* >=0: terminal-set index, <0: ~nonterminal  */
    uint32_t* tsets;     /* [n_tset][8] 256-bit byte sets              */
    int32_t* nt_off;     /* [n_nt+1] productions grouped by lhs        */
    int32_t* nt_prods;
    uint8_t* nullable;   /* [n_nt]                                     */
} Grammar;

static void set_init(Set* s) { s->it = NULL; s->n = 0; s->cap = 0; }
static void set_free(Set* s) { free(s->it); s->it = NULL; s->n = s->cap = 0; }

static int set_add(Set* s, int32_t prod, int32_t dot, int32_t origin) {
    for (int32_t i = 0; i < s->n; ++i)
        if (s->it[i].prod == prod && s->it[i].dot == dot && s->it[i].origin == origin) return 0;
    if (s->n == s->cap) {
        s->cap = s->cap ? s->cap * 2 : 16;
        s->it = (Item*)realloc(s->it, sizeof(Item) * (size_t)s->cap);
    }
    s->it[s->n].prod = prod; s->it[s->n].dot = dot; s->it[s->n].origin = origin;
    s->n++;
    return 1;
}

void* eo_grammar_new(int32_t n_nt, int32_t n_prod, const int32_t* lhs, const int32_t* off,
                     const int32_t* syms, int32_t n_tset, const uint32_t* tsets) {
    Grammar* g = (Grammar*)calloc(1, sizeof(Grammar));
    g->n_nt = n_nt; g->n_prod = n_prod; g->n_tset = n_tset;
    g->lhs = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_prod + 1));
    g->off = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_prod + 2));
    memcpy(g->lhs, lhs, sizeof(int32_t) * (size_t)n_prod);
    memcpy(g->off, off, sizeof(int32_t) * (size_t)(n_prod + 1));
    int32_t nsym = off[n_prod];
    g->syms = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nsym + 1));
    memcpy(g->syms, syms, sizeof(int32_t) * (size_t)nsym);
    g->tsets = (uint32_t*)malloc(sizeof(uint32_t) * 8 * (size_t)(n_tset + 1));
    memcpy(g->tsets, tsets, sizeof(uint32_t) * 8 * (size_t)n_tset);
    g->nt_off = (int32_t*)calloc((size_t)n_nt + 1, sizeof(int32_t));
    g->nt_prods = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_prod + 1));
    for (int32_t p = 0; p < n_prod; ++p) g->nt_off[lhs[p] + 1]++;
    for (int32_t a = 0; a < n_nt; ++a) g->nt_off[a + 1] += g->nt_off[a];
    int32_t* fill = (int32_t*)calloc((size_t)n_nt, sizeof(int32_t));
    for (int32_t p = 0; p < n_prod; ++p) g->nt_prods[g->nt_off[lhs[p]] + fill[lhs[p]]++] = p;
    free(fill);
    /* nullable nonterminals: least fixed point */
    g->nullable = (uint8_t*)calloc((size_t)n_nt, 1);
    for (int changed = 1; changed;) {
        changed = 0;
        for (int32_t p = 0; p < n_prod; ++p) {
            if (g->nullable[lhs[p]]) continue;
            int ok = 1;
            for (int32_t k = off[p]; k < off[p + 1]; ++k)
                if (syms[k] >= 0 || !g->nullable[~syms[k]]) { ok = 0; break; }
            if (ok) { g->nullable[lhs[p]] = 1; changed = 1; }
        }
    }
    return g;
}

void eo_grammar_free(void* h) {
    Grammar* g = (Grammar*)h;
    if (!g) return;
    free(g->lhs); free(g->off); free(g->syms); free(g->tsets);
    free(g->nt_off); free(g->nt_prods); free(g->nullable); free(g);
}

int32_t eo_is_nullable(void* h, int32_t nt) { return ((Grammar*)h)->nullable[nt]; }

/* productive nonterminals (derive at least one terminal string): out[n_nt] */
void eo_productive(void* h, uint8_t* out) {
    Grammar* g = (Grammar*)h;
    memset(out, 0, (size_t)g->n_nt);
    for (int changed = 1; changed;) {
        changed = 0;
        for (int32_t p = 0; p < g->n_prod; ++p) {
            if (out[g->lhs[p]]) continue;
            int ok = 1;
            for (int32_t k = g->off[p]; k < g->off[p + 1]; ++k) {
                int32_t s = g->syms[k];
                if (s >= 0) {
                    int any = 0;
                    for (int w = 0; w < 8; ++w) any |= g->tsets[s * 8 + w] != 0;
                    if (!any) { ok = 0; break; }
                } else if (!out[~s]) { ok = 0; break; }
            }
            if (ok) { out[g->lhs[p]] = 1; changed = 1; }
        }
    }
}

/* The augmented start production  S' -> start  (or  S' -> start start2 ) has index g->n_prod. */
typedef struct { const Grammar* g; int32_t start, start2; } Ctx;

static inline int32_t rhs_len(const Ctx* c, int32_t prod) {
    return prod == c->g->n_prod ? (c->start2 >= 0 ? 2 : 1) : c->g->off[prod + 1] - c->g->off[prod];
}
static inline int32_t rhs_sym(const Ctx* c, int32_t prod, int32_t dot) {
    return prod == c->g->n_prod ? (dot == 0 ? ~c->start : ~c->start2) : c->g->syms[c->g->off[prod] + dot];
}
static inline int32_t prod_lhs(const Ctx* c, int32_t prod) {
    return prod == c->g->n_prod ? -1 : c->g->lhs[prod];
}

/* predictor + completer until nothing new; sets[j] is the set being closed */
static void closure(const Ctx* c, Set* sets, int32_t j) {
    const Grammar* g = c->g;
    Set* cur = &sets[j];
    for (int32_t i = 0; i < cur->n; ++i) {
        Item it = cur->it[i];
        if (it.dot == rhs_len(c, it.prod)) {                    /* completer */
            int32_t A = prod_lhs(c, it.prod);
            if (A < 0) continue;                                /* S' complete */
            Set* o = &sets[it.origin];
            for (int32_t k = 0; k < o->n; ++k) {                /* o may be cur and may grow */
                Item w = o->it[k];
                if (w.dot < rhs_len(c, w.prod) && rhs_sym(c, w.prod, w.dot) == ~A)
                    set_add(cur, w.prod, w.dot + 1, w.origin);
            }
        } else {
            int32_t s = rhs_sym(c, it.prod, it.dot);
            if (s < 0) {                                        /* predictor */
                int32_t B = ~s;
                for (int32_t k = g->nt_off[B]; k < g->nt_off[B + 1]; ++k)
                    set_add(cur, g->nt_prods[k], 0, j);
                if (g->nullable[B]) set_add(cur, it.prod, it.dot + 1, it.origin);
            }
        }
    }
}

/* scanner: sets[j] --byte--> sets[j+1] (cleared first), then closure */
static void step(const Ctx* c, Set* sets, int32_t j, uint8_t byte) {
    const Grammar* g = c->g;
    Set* cur = &sets[j];
    Set* nxt = &sets[j + 1];
    nxt->n = 0;
    for (int32_t i = 0; i < cur->n; ++i) {
        Item it = cur->it[i];
        if (it.dot == rhs_len(c, it.prod)) continue;
        int32_t s = rhs_sym(c, it.prod, it.dot);
        if (s >= 0 && ((g->tsets[s * 8 + (byte >> 5)] >> (byte & 31)) & 1u))
            set_add(nxt, it.prod, it.dot + 1, it.origin);
    }
    closure(c, sets, j + 1);
}

static int start_complete(const Ctx* c, const Set* s) {
    for (int32_t i = 0; i < s->n; ++i)
        if (s->it[i].prod == c->g->n_prod && s->it[i].dot == rhs_len(c, c->g->n_prod) && s->it[i].origin == 0) return 1;
    return 0;
}

/*
 * Parse `hist` (hlen bytes) from nonterminal `start` (followed by nonterminal `start2` unless that is
 * negative: the language is then the concatenation); then for every token t of the vocabulary
 * (CSR: blob + offs[V+1]) decide
 *     viable[t]  = 1  iff  the item set after hist.bytes(t) is non-empty
 *     early[t]   = 1  iff  for some i, 1 <= i < len(t), hist.t[0:i] is a complete sentence
 * If follow >= 0, early[t] additionally requires that the rest of the token, t[i:], is a viable prefix
 * of the language of nonterminal `follow` (what may come after the start symbols in some context).
 * Zero-length tokens get 0 / 0.  Returns -1 if hist itself is not a viable prefix, else
 * 1 if hist is a complete sentence, else 0.
 * Optionally exports the items of the closed set after hist: last_items[3*k] = prod, dot, origin
 * (at most last_cap items; *last_n receives the true count).
 */
static int viable_from(const Grammar* g, int32_t nt, const uint8_t* text, int64_t n, Set* scratch) {
    Ctx c; c.g = g; c.start = nt; c.start2 = -1;
    scratch[0].n = 0;
    set_add(&scratch[0], g->n_prod, 0, 0);
    closure(&c, scratch, 0);
    for (int64_t j = 0; j < n; ++j) {
        step(&c, scratch, (int32_t)j, text[j]);
        if (scratch[j + 1].n == 0) return 0;
    }
    return 1;
}

int32_t eo_scan_vocab(void* h, int32_t start, int32_t start2, int32_t follow, const uint8_t* hist, int64_t hlen,
                      const uint8_t* blob, const int64_t* offs, int32_t V,
                      uint8_t* viable, uint8_t* early,
                      int32_t* last_items, int32_t last_cap, int32_t* last_n, int32_t n_threads) {
    Grammar* g = (Grammar*)h;
    Ctx c; c.g = g; c.start = start; c.start2 = start2;
    int64_t max_tok = 0;
    for (int32_t t = 0; t < V; ++t) if (offs[t + 1] - offs[t] > max_tok) max_tok = offs[t + 1] - offs[t];
    Set* base = (Set*)malloc(sizeof(Set) * (size_t)(hlen + 1));
    for (int64_t j = 0; j <= hlen; ++j) set_init(&base[j]);
    set_add(&base[0], g->n_prod, 0, 0);
    closure(&c, base, 0);
    int dead = 0;
    for (int64_t j = 0; j < hlen; ++j) {
        step(&c, base, (int32_t)j, hist[j]);
        if (base[j + 1].n == 0) { dead = 1; break; }
    }
    int32_t ret = -1;
    if (!dead) {
        ret = start_complete(&c, &base[hlen]);
        if (last_n) {
            *last_n = base[hlen].n;
            for (int32_t k = 0; k < base[hlen].n && k < last_cap; ++k) {
                last_items[3 * k] = base[hlen].it[k].prod;
                last_items[3 * k + 1] = base[hlen].it[k].dot;
                last_items[3 * k + 2] = base[hlen].it[k].origin;
            }
        }
        if (viable) {
#ifdef _OPENMP
            if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel
#endif
            {
                Set* sets = (Set*)malloc(sizeof(Set) * (size_t)(hlen + max_tok + 2));
                for (int64_t j = 0; j <= hlen; ++j) sets[j] = base[j];       /* shared, read-only */
                for (int64_t j = hlen + 1; j <= hlen + max_tok + 1; ++j) set_init(&sets[j]);
                Set* fsets = (Set*)malloc(sizeof(Set) * (size_t)(max_tok + 2));
                for (int64_t j = 0; j <= max_tok + 1; ++j) set_init(&fsets[j]);
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 256)
#endif
                for (int32_t t = 0; t < V; ++t) {
                    int64_t n = offs[t + 1] - offs[t];
                    const uint8_t* b = blob + offs[t];
                    uint8_t ok = 0, ear = 0;
                    if (n > 0) {
                        ok = 1;
                        for (int64_t i = 0; i < n; ++i) {
                            step(&c, sets, (int32_t)(hlen + i), b[i]);
                            if (sets[hlen + i + 1].n == 0) { ok = 0; break; }
                            if (i + 1 < n && start_complete(&c, &sets[hlen + i + 1])) {
                                if (follow < 0) ear = 1;
                                else if (!ear && viable_from(g, follow, b + i + 1, n - i - 1, fsets)) ear = 1;
                            }
                        }
                    }
                    viable[t] = ok;
                    if (early) early[t] = ear;
                }
                for (int64_t j = hlen + 1; j <= hlen + max_tok + 1; ++j) set_free(&sets[j]);
                for (int64_t j = 0; j <= max_tok + 1; ++j) set_free(&fsets[j]);
                free(fsets);
                free(sets);
            }
        }
    }
    for (int64_t j = 0; j <= hlen; ++j) set_free(&base[j]);
    free(base);
    return ret;
}

/* Does `text` belong to L(start)?  (sentence test, used by the pins) */
int32_t eo_accepts(void* h, int32_t start, const uint8_t* text, int64_t n) {
    return eo_scan_vocab(h, start, -1, -1, text, n, NULL, NULL, 0, NULL, NULL, NULL, 0, NULL, 1) == 1;
}

/* In-place token-bitmask application, plain loops (paper section 2.1: logits of tokens that do
 * not conform get -infinity).  bit v%32 of word v/32 set = token allowed. */
void eo_apply_f32(uint32_t* logits_bits, int64_t B, int64_t V, int64_t stride,
                  const int32_t* bitmask, int64_t bm_stride) {
    for (int64_t b = 0; b < B; ++b)
        for (int64_t v = 0; v < V; ++v)
            if (!((((uint32_t)bitmask[b * bm_stride + v / 32]) >> (v % 32)) & 1u))
                logits_bits[b * stride + v] = 0xFF800000u;
}
void eo_apply_bf16(uint16_t* logits_bits, int64_t B, int64_t V, int64_t stride,
                   const int32_t* bitmask, int64_t bm_stride) {
    for (int64_t b = 0; b < B; ++b)
        for (int64_t v = 0; v < V; ++v)
            if (!((((uint32_t)bitmask[b * bm_stride + v / 32]) >> (v % 32)) & 1u))
                logits_bits[b * stride + v] = 0xFF80u;
}
