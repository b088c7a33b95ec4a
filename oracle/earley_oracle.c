/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.  Nothing in the product library may
 * include, link or call this file; only the tests, the smoke check and the
 * benchmark's CPU-baseline leg use it.
 *
 * A plain textbook Earley recognizer (paper Section 3.2: items (X -> a . b, j),
 * state sets S[0..n], the Predict / Scan / Complete operations, every set holding
 * an item at most once) over a context-free grammar whose terminals
 * are single-byte classes.  There is no trie, no automaton, no cache and no
 * pruning here.  The per-step vocabulary check (Section 3.3 / 4.1: every token of
 * the vocabulary is tested at every decoding step, invalid logits become -inf)
 * is written out literally: copy the chart, feed the token's bytes one at a
 * time, and call the token allowed iff no byte leaves an empty state set.
 *
 * Rules that derive the empty string are handled natively with the
 * Aycock-Horspool rule (when a nullable nonterminal is predicted, the predicting
 * item is also advanced over it), which is the standard way to make the textbook
 * closure loop complete in the presence of empty rules.
 *
 * Pins: tests/test_oracle_pins.py (worked examples of Sections 1 and 3.2, brute
 * force enumeration, CYK, regular special case, JSON library cross-check).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int n_nt, start, n_rules;
    int *lhs;      /* [n_rules+1]; the last rule is the added start rule S' -> S, lhs = n_nt */
    int *rhs_off;  /* [n_rules+2] */
    int *rhs_sym;  /* >= 0 nonterminal, < 0 byte class ~sym */
    int n_classes;
    uint8_t *class_bits; /* [n_classes][32]: bit c of the class = byte c matches */
    uint8_t *nullable;   /* [n_nt+1] */
} orc_grammar;

typedef struct { int rule, dot, origin; } orc_item;

typedef struct {
    const orc_grammar *g;
    orc_item *items; long n_items, cap_items;
    long *set_off;   /* set k = items[set_off[k] .. set_off[k+1]) */
    long n_sets, cap_sets;
} orc_state;

static int rule_len(const orc_grammar *g, int r) { return g->rhs_off[r + 1] - g->rhs_off[r]; }
static int class_has(const orc_grammar *g, int cls, uint8_t byte)
{
    return (g->class_bits[(size_t)cls * 32 + (byte >> 3)] >> (byte & 7)) & 1;
}

orc_grammar *orc_grammar_new(int n_nt, int start, int n_rules, const int *lhs, const int *rhs_off,
                             const int *rhs_sym, int n_classes, const uint8_t *class_bits)
{
    orc_grammar *g = calloc(1, sizeof *g);
    int n_sym = rhs_off[n_rules];
    g->n_nt = n_nt; g->start = start; g->n_rules = n_rules; g->n_classes = n_classes;
    g->lhs = malloc(sizeof(int) * (n_rules + 1));
    g->rhs_off = malloc(sizeof(int) * (n_rules + 2));
    g->rhs_sym = malloc(sizeof(int) * (n_sym + 1));
    memcpy(g->lhs, lhs, sizeof(int) * n_rules);
    memcpy(g->rhs_off, rhs_off, sizeof(int) * (n_rules + 1));
    memcpy(g->rhs_sym, rhs_sym, sizeof(int) * n_sym);
    g->lhs[n_rules] = n_nt;               /* S' -> S */
    g->rhs_sym[n_sym] = start;
    g->rhs_off[n_rules + 1] = n_sym + 1;
    g->class_bits = malloc((size_t)n_classes * 32 + 1);
    memcpy(g->class_bits, class_bits, (size_t)n_classes * 32);
    /* nullable nonterminals: least fixed point of "some rule has only nullable symbols" */
    g->nullable = calloc(n_nt + 1, 1);
    for (int changed = 1; changed;) {
        changed = 0;
        for (int r = 0; r <= n_rules; r++) {
            if (g->nullable[g->lhs[r]]) continue;
            int all = 1;
            for (int k = g->rhs_off[r]; k < g->rhs_off[r + 1]; k++)
                if (g->rhs_sym[k] < 0 || !g->nullable[g->rhs_sym[k]]) { all = 0; break; }
            if (all) { g->nullable[g->lhs[r]] = 1; changed = 1; }
        }
    }
    return g;
}

void orc_grammar_free(orc_grammar *g)
{
    if (!g) return;
    free(g->lhs); free(g->rhs_off); free(g->rhs_sym); free(g->class_bits); free(g->nullable); free(g);
}

int orc_is_nullable(const orc_grammar *g, int nt) { return g->nullable[nt]; }

/* ---- chart ------------------------------------------------------------------------- */
static void push_set(orc_state *s)
{
    if (s->n_sets + 2 > s->cap_sets) {
        s->cap_sets = s->cap_sets * 2 + 16;
        s->set_off = realloc(s->set_off, sizeof(long) * s->cap_sets);
    }
    s->n_sets++;
    s->set_off[s->n_sets] = s->n_items;
}

/* add an item to the last set unless it is already there (unique states only) */
static void add_item(orc_state *s, int rule, int dot, int origin)
{
    long b = s->set_off[s->n_sets - 1];
    for (long i = b; i < s->n_items; i++)
        if (s->items[i].rule == rule && s->items[i].dot == dot && s->items[i].origin == origin) return;
    if (s->n_items == s->cap_items) {
        s->cap_items = s->cap_items * 2 + 64;
        s->items = realloc(s->items, sizeof(orc_item) * s->cap_items);
    }
    s->items[s->n_items].rule = rule; s->items[s->n_items].dot = dot; s->items[s->n_items].origin = origin;
    s->n_items++;
    s->set_off[s->n_sets] = s->n_items;
}

/* Predict and Complete until the last set stops growing */
static void closure(orc_state *s)
{
    const orc_grammar *g = s->g;
    int k = (int)s->n_sets - 1;
    for (long i = s->set_off[k]; i < s->n_items; i++) {
        orc_item it = s->items[i];
        if (it.dot == rule_len(g, it.rule)) {
            /* Complete: advance every item of S[origin] whose postdot symbol is this lhs */
            int X = g->lhs[it.rule];
            long e = (it.origin == k) ? s->n_items : s->set_off[it.origin + 1];
            for (long j = s->set_off[it.origin]; j < e; j++) {
                orc_item q = s->items[j];
                if (q.dot < rule_len(g, q.rule) && g->rhs_sym[g->rhs_off[q.rule] + q.dot] == X) {
                    add_item(s, q.rule, q.dot + 1, q.origin);
                    if (it.origin == k) e = s->n_items;
                }
            }
        } else {
            int Y = g->rhs_sym[g->rhs_off[it.rule] + it.dot];
            if (Y >= 0) {
                /* Predict: all rules of Y start here; a nullable Y may also be skipped */
                for (int r = 0; r < g->n_rules; r++)
                    if (g->lhs[r] == Y) add_item(s, r, 0, k);
                if (g->nullable[Y]) add_item(s, it.rule, it.dot + 1, it.origin);
            }
        }
    }
}

orc_state *orc_state_new(const orc_grammar *g)
{
    orc_state *s = calloc(1, sizeof *s);
    s->g = g;
    s->cap_sets = 16; s->set_off = malloc(sizeof(long) * s->cap_sets); s->set_off[0] = 0;
    push_set(s);
    add_item(s, g->n_rules, 0, 0);   /* (S' -> . S, 0) */
    closure(s);
    return s;
}

orc_state *orc_state_clone(const orc_state *o)
{
    orc_state *s = malloc(sizeof *s);
    *s = *o;
    s->cap_items = o->n_items + 256; s->cap_sets = o->n_sets + 32;
    s->items = malloc(sizeof(orc_item) * s->cap_items);
    s->set_off = malloc(sizeof(long) * s->cap_sets);
    memcpy(s->items, o->items, sizeof(orc_item) * o->n_items);
    memcpy(s->set_off, o->set_off, sizeof(long) * (o->n_sets + 1));
    return s;
}

void orc_state_free(orc_state *s) { if (s) { free(s->items); free(s->set_off); free(s); } }

/* Scan byte c from the last set into a new set, then close it.  Returns 1 if the new set is
 * non-empty (the prefix is still viable); otherwise removes the empty set and returns 0. */
int orc_feed(orc_state *s, uint8_t c)
{
    const orc_grammar *g = s->g;
    int k = (int)s->n_sets - 1;
    long b = s->set_off[k], e = s->set_off[k + 1];
    push_set(s);
    for (long i = b; i < e; i++) {
        orc_item it = s->items[i];
        if (it.dot < rule_len(g, it.rule)) {
            int a = g->rhs_sym[g->rhs_off[it.rule] + it.dot];
            if (a < 0 && class_has(g, ~a, c)) add_item(s, it.rule, it.dot + 1, it.origin);
        }
    }
    if (s->n_items == s->set_off[k + 1]) { s->n_sets--; return 0; }
    closure(s);
    return 1;
}

/* Drop the last n sets (Earley never changes earlier sets, so this undoes n feeds). */
static void truncate_sets(orc_state *s, long n_sets) { s->n_sets = n_sets; s->n_items = s->set_off[n_sets]; }

/* Would these bytes keep the prefix viable?  The state is left unchanged. */
int orc_check(orc_state *s, const uint8_t *bytes, long n)
{
    long keep = s->n_sets;
    int ok = n > 0;
    for (long i = 0; i < n && ok; i++) ok = orc_feed(s, bytes[i]);
    truncate_sets(s, keep);
    return ok;
}

/* Feed all bytes or none. */
int orc_feed_bytes(orc_state *s, const uint8_t *bytes, long n)
{
    long keep = s->n_sets;
    for (long i = 0; i < n; i++)
        if (!orc_feed(s, bytes[i])) { truncate_sets(s, keep); return 0; }
    return 1;
}

/* prefix in L(G)  <=>  (S' -> S ., 0) is in the last set */
int orc_accepting(const orc_state *s)
{
    long k = s->n_sets - 1;
    for (long i = s->set_off[k]; i < s->set_off[k + 1]; i++)
        if (s->items[i].rule == s->g->n_rules && s->items[i].dot == 1 && s->items[i].origin == 0) return 1;
    return 0;
}

long orc_n_sets(const orc_state *s) { return s->n_sets; }
long orc_n_items(const orc_state *s) { return s->n_items; }
long orc_set_size(const orc_state *s, long k) { return s->set_off[k + 1] - s->set_off[k]; }
void orc_set_items(const orc_state *s, long k, int *out /* [size][3] rule,dot,origin */)
{
    for (long i = s->set_off[k], j = 0; i < s->set_off[k + 1]; i++, j++) {
        out[3 * j] = s->items[i].rule; out[3 * j + 1] = s->items[i].dot; out[3 * j + 2] = s->items[i].origin;
    }
}

/* The vocabulary mask of one state: bit (v & 31) of word (v >> 5) is 1 iff token v is
 * allowed.  Tokens are checked independently; each thread works on its own copy of the
 * chart.  Returns the number of threads used.  Zero-length tokens are never allowed. */
int orc_mask(const orc_state *s, long V, const int64_t *off, const uint8_t *bytes, uint32_t *out, int n_threads)
{
    long W = (V + 31) / 32;
    int used = 1;
    memset(out, 0, sizeof(uint32_t) * W);
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
        orc_state *c = orc_state_clone(s);
        #pragma omp for schedule(dynamic, 8)
        for (long w = 0; w < W; w++) {
            uint32_t word = 0;
            for (long v = w * 32; v < V && v < w * 32 + 32; v++)
                if (orc_check(c, bytes + off[v], off[v + 1] - off[v])) word |= 1u << (v & 31);
            out[w] = word;
        }
        orc_state_free(c);
    }
#else
    (void)n_threads;
    orc_state *c = orc_state_clone(s);
    for (long v = 0; v < V; v++)
        if (orc_check(c, bytes + off[v], off[v + 1] - off[v])) out[v >> 5] |= 1u << (v & 31);
    orc_state_free(c);
#endif
    return used;
}

/* Masking of logits (Section 3.3): a disallowed position becomes -inf, an allowed one is
 * copied bit for bit.  elem_size 4 = IEEE binary32 (-inf = 0xFF800000), 2 = bfloat16 (0xFF80). */
void orc_apply_mask(const void *logits, void *out, int elem_size, long B, long V, long row_stride,
                    const uint32_t *mask /* [B][ceil(V/32)] */)
{
    long W = (V + 31) / 32;
    for (long b = 0; b < B; b++)
        for (long v = 0; v < V; v++) {
            int bit = (mask[b * W + (v >> 5)] >> (v & 31)) & 1;
            if (elem_size == 4) {
                uint32_t x = ((const uint32_t *)logits)[b * row_stride + v];
                ((uint32_t *)out)[b * row_stride + v] = bit ? x : 0xFF800000u;
            } else {
                uint16_t x = ((const uint16_t *)logits)[b * row_stride + v];
                ((uint16_t *)out)[b * row_stride + v] = bit ? x : (uint16_t)0xFF80u;
            }
        }
}
