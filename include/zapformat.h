/*
 * zapformat -- per-decode-step vocabulary mask for grammar-constrained decoding on MI355X.
 *
 * The operations follow the paper's statement of the problem:
 *   - a context-free grammar A -> alpha (Section 3.1) whose terminals are byte strings or
 *     byte-level regular expressions matched by finite-state machines (Section 4.1);
 *   - an Earley recognizer state per query, updated after every decoded token with
 *     Scan / Complete / Compact / Predict (Sections 3.2 and 4.2, ZapFormat pruning);
 *   - at every decoding step, a validity verdict for EVERY vocabulary token, applied to the
 *     logits by writing -inf over the invalid ones (Sections 3.3 and 4.1).
 *
 * All functions return ZF_OK (0) or a negative error code; nothing aborts or throws across
 * this boundary.  Handles are opaque, owned by the library and released only by *_destroy.
 * "host" / "device" in a comment says where a pointer must live.  The library needs a HIP
 * device for zf_compute_mask / zf_apply_mask; there is no CPU substitute for them.
 */
#ifndef ZAPFORMAT_H
#define ZAPFORMAT_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum {
    ZF_OK = 0,
    ZF_ERR_INVALID_ARG = -1, /* null pointer, bad size, bad dtype, state of another engine */
    ZF_ERR_GRAMMAR = -2,     /* bad symbol id, bad regex, terminal with empty language or that
                                matches the empty string, start symbol derives nothing */
    ZF_ERR_REJECTED = -3,    /* token / bytes not allowed in this state; the state is unchanged */
    ZF_ERR_RANGE = -4,       /* token id outside [0, V) */
    ZF_ERR_DEVICE = -5,      /* HIP call failed, or the engine was compiled without a device */
    ZF_ERR_OOM = -6,
    ZF_ERR_OVERFLOW = -7     /* an Earley set outgrew even the device fallback arena; the mask
                                written by this call is not valid */
};

const char *zf_strerror(int code); /* static string */
const char *zf_last_error(void);   /* thread-local detail of the last failure on this thread */

typedef struct zf_engine zf_engine; /* immutable after zf_compile; may be shared by many states */
typedef struct zf_state zf_state;   /* one query: the (pruned) Earley chart of its prefix */

/* A grammar (Section 3.1).  All arrays are host memory, owned by the caller, copied by
 * zf_compile.  Nonterminals are 0..n_nonterminals-1.  rhs_sym >= 0 is a nonterminal id,
 * rhs_sym < 0 is terminal ~rhs_sym.  An empty right-hand side is an epsilon rule. */
typedef struct {
    int32_t n_nonterminals, start;
    int32_t n_rules;
    const int32_t *rule_lhs; /* [n_rules] */
    const int32_t *rhs_off;  /* [n_rules+1] CSR offsets into rhs_sym */
    const int32_t *rhs_sym;
    int32_t n_terminals;
    const uint8_t *term_kind; /* [n_terminals] 0 = literal bytes, 1 = byte-regex source */
    const int64_t *term_off;  /* [n_terminals+1] CSR offsets into term_data */
    const uint8_t *term_data;
} zf_grammar_desc;

/* The vocabulary: token v is bytes[off[v] .. off[v+1]).  Host memory.  Tokens are arbitrary
 * byte strings (they may split multi-byte characters, Section 2); duplicates are legal and get
 * equal verdicts; a zero-length token is never allowed. */
typedef struct {
    int32_t V;
    const int64_t *off;
    const uint8_t *bytes;
} zf_vocab_desc;

typedef struct {
    int32_t pruning;       /* 1 = ZapFormat Compact phase on (Section 4.2), 0 = keep every item */
    int32_t lane_item_cap; /* Earley item budget (LDS) of one walking wavefront of the mask kernel,
                              0 = automatic (96, more when the current sets are large); what does not fit goes to the exact fallback pass */
    int32_t device;        /* HIP device ordinal, or -1 = host tables only (no mask calls) */
    int32_t chunk_strings; /* vocabulary strings walked by one lane: 8, 16 or 32; 0 = default */
    int32_t fallback_item_cap; /* item budget of a fallback wavefront (global memory), 0 = default
                                  (65536); tests set it low to provoke ZF_ERR_OVERFLOW */
    int32_t state_cache_entries; /* state cache (Section 5.2): finished mask rows kept on the device,
                                  keyed by the row's pruned chart; 0 = default (2048 rows), -1 = off */
    int32_t disable_token_mask_cache; /* 1 = every token goes through the parser walk (Section 4.3
                                  optimisation off); masks are identical either way */
    int32_t walk_mode;     /* which mask kernel checks the tokens the token-mask cache leaves undecided (masks are identical):
                              0 = per-block automaton (a block builds the row's automaton of Earley sets over byte classes
                              lazily in LDS, from the row's uploaded chart; one lane per token string),
                              1 = trie walk (one wavefront per chunk of the vocabulary trie),
                              2 = persistent automaton (one automaton for all rows and steps, kept in device memory: Earley sets
                              named by content; a call uploads the bytes fed since the last call, not the charts, and a transition
                              is computed once per engine; needs pruning = 1, else mode 0 runs in its place).  A call the
                              persistent automaton has no room for is answered by mode 0 when it is a waiting call.  With mode 2
                              and pruning = 1 zf_advance, too, goes through such an automaton, kept on the host (a look-up per
                              byte once a transition is known; results are those of the plain advance) -- with or without a device. */
    int32_t precompute_states; /* walk_mode 2: how much of the persistent automaton is built before the first decode step.  When the
                              engine is compiled, and again whenever zf_engine_clear_state_cache empties it, the automaton is
                              explored breadth first from the state of the empty prefix, one byte of every byte class at a time,
                              and the mask at every state found is computed once (a mask call computes every transition its
                              walk of the vocabulary meets), until no new state turns up, this many states have been visited,
                              a second has passed, or the store is a quarter full.  A grammar without recursion has a finite automaton and gets
                              it whole, the way engines for regular constraints build theirs at compile time (a decode loop then
                              computes no transition at all); of a recursive grammar the states nearest the start are built.  Masks are the same with or without.
                              0 = default (65536 states), -1 = off */
} zf_options;

typedef struct {
    int64_t n_sets, n_items;   /* chart as it stands (after Compact when pruning is on) */
    int64_t items_created;     /* every item ever added by Scan/Complete since the last reset */
    int64_t bytes_fed;
    int32_t accepting;
} zf_stats;

typedef struct {
    int32_t V, W;                 /* W = ceil(V/32) mask words per row */
    int32_t n_nonterminals, n_rules, n_positions;
    int32_t n_dfa_states, n_byte_classes;
    int32_t n_trie_nodes, n_strings; /* distinct non-empty token strings */
    int32_t lane_item_cap, device;
    int32_t table_lds_mode;       /* grammar tables the mask kernels keep in LDS: 0 = all, 1 = the small ones, 2 = none;
                                     -1 when the engine has no device */
} zf_engine_info;

typedef struct {               /* facts about the last zf_compute_mask, for reporting only */
    int64_t overflow_chunks;   /* trie chunks handed to the fallback pass in the last call */
    int64_t walk_chunks;       /* work the token-mask cache left to the parser kernel: undecided strings (mask
                                  automaton) or trie chunks that hold such strings (trie walk) */
    int64_t chart_bytes;       /* bytes uploaded for the last call */
    int32_t cache_hits, cache_misses; /* rows of the last call served from / added to the state cache */
    float main_ms, fallback_ms, permute_ms; /* durations from HIP events on the call's stream, 0 unless
                                               zf_engine_set_profiling is on: main_ms the mask kernel;
                                               permute_ms the closing kernel (fallback pass for what the
                                               mask kernel listed + permutation into token order, and the
                                               state cache's gather); fallback_ms always 0 (that pass has
                                               no kernel of its own) */
    int32_t parser_steps;      /* Earley byte steps the mask-automaton kernel took in the last call (all blocks) */
    int32_t cache_rows;        /* token-mask-cache bitset rows merged in the last call (sum over its rows) */
} zf_mask_report;

/* compile(grammar rules, vocab byte strings): clean the grammar (useless rules, nullable
 * symbols: Section 4.5), build one byte-level DFA per terminal (Section 4.1), flatten the
 * vocabulary into a prefix trie, upload the immutable tables.  *out is set on success only. */
int zf_compile(const zf_grammar_desc *g, const zf_vocab_desc *v, const zf_options *opt, zf_engine **out);
void zf_engine_destroy(zf_engine *e);
int zf_engine_get_info(const zf_engine *e, zf_engine_info *out);

int zf_state_new(zf_engine *e, zf_state **out); /* chart of the empty prefix */
int zf_state_clone(const zf_state *s, zf_state **out);
int zf_state_reset(zf_state *s);
void zf_state_destroy(zf_state *s);

/* advance(state, token_id): feed the token's bytes through Scan -> Complete -> Compact ->
 * Predict (Sections 3.2, 4.2).  All or nothing: on ZF_ERR_REJECTED the state is unchanged.
 * States of one engine may be advanced from several threads at once (one thread per state). */
int zf_advance(zf_state *s, int32_t token_id);
int zf_advance_bytes(zf_state *s, const uint8_t *bytes /* host */, int64_t n);
/* One decode step of a whole batch (the generation loop of Section 3.3 applied to every row):
 * row b is advanced by token_ids[b], or reset to the empty prefix when token_ids[b] < 0.
 * states and token_ids are host arrays of n entries; status (host, n entries, may be null)
 * receives each row's return code.  Every row is processed; the return value is the first
 * code that is not ZF_OK (zf_last_error then holds the text of the first failing row).  A
 * rejected row is left unchanged, as with zf_advance; a null state fails the whole call with
 * ZF_ERR_INVALID_ARG before any row is touched.  A state named twice is fed twice, in order.
 * Rows are independent, so when the batch is expensive to feed (wide Earley sets of an ambiguous
 * grammar) its rows are dealt to worker threads that the library starts on first need and keeps
 * (at most 15; a forked child process feeds its rows on the calling thread); small batches
 * never leave the caller's thread.  The call returns when every row is done. */
int zf_advance_batch(zf_state *const *states, const int32_t *token_ids, int32_t n, int32_t *status);
int zf_is_accepting(const zf_state *s, int32_t *out); /* is the prefix a sentence of the grammar? */
int zf_state_stats(const zf_state *s, zf_stats *out);
/* Copy the chart out for inspection: items as int32 triples (dotted position, origin set, DFA
 * state), set_off[n_sets+1].  Pass null buffers to query sizes through zf_state_stats. */
int zf_state_chart(const zf_state *s, int32_t *items /* host [n_items][3] */, int64_t *set_off /* host */);
/* Describe a dotted position: lhs nonterminal id (original numbering), rule index (original),
 * dot.  For tests that compare charts with the paper's worked examples. */
int zf_position_info(const zf_engine *e, int32_t position, int32_t *lhs, int32_t *rule, int32_t *dot);

/* compute_mask(states[batch]): for every row and every token v, bit (v & 31) of word (v >> 5)
 * of d_mask[row] becomes 1 iff the token's bytes, fed one at a time, never empty the Earley
 * set (Section 4.1: all tokens are checked at every step).  d_mask: device, [batch][W]
 * uint32, fully overwritten, padding bits zero.  The states' charts are snapshotted before
 * the call returns.  The work is enqueued on hip_stream (a hipStream_t, null = default
 * stream); the call waits for its own kernels so that ZF_ERR_OVERFLOW can be reported. */
int zf_compute_mask(zf_engine *e, zf_state *const *states /* host array */, int32_t batch,
                    uint32_t *d_mask, void *hip_stream);
/* The same, without waiting: the kernels (the fallback pass is part of the last one) are only enqueued on
 * hip_stream, so that the caller's next launches (zf_apply_mask, the sampler) queue up right
 * behind them.  ZF_ERR_OVERFLOW, if any, is reported by zf_mask_wait.  At most 4 calls may be in
 * flight between two zf_mask_wait calls; calls on one engine must all use the same stream and must
 * not overlap from several host threads.
 *   zf_mask_wait returns once the status of the calls in flight is final (a block of their last kernel writes
 * it to pinned host memory, which the call polls; when the fallback pass had work, whose waits can fail, it is
 * the block that finishes last; bounded: after two seconds the stream is synchronised instead).  It does NOT
 * wait for work the caller queued behind them (zf_apply_mask, a sampler), and the mask tensor is to be
 * consumed in stream order: queue its readers on hip_stream, or synchronise the stream before reading it
 * from the host or from another stream (zf_compute_mask, the waiting call, does synchronise).  With no call
 * in flight zf_mask_wait synchronises hip_stream. */
int zf_compute_mask_async(zf_engine *e, zf_state *const *states /* host array */, int32_t batch,
                          uint32_t *d_mask, void *hip_stream);
int zf_mask_wait(zf_engine *e, void *hip_stream);
/* compute_mask followed by apply_mask on the same rows (Sections 4.1 and 3.3: the verdicts of a step are there to mask that
 * step's logits), enqueued together: the result in d_mask and d_out is exactly what zf_compute_mask_async followed by
 * zf_apply_mask(e, d_logits, d_out, dtype, batch, row_stride_elems, d_mask, hip_stream) gives, and zf_mask_wait reports as
 * for that pair.  With the persistent automaton as the mask kernel and the state cache off, one kernel does both (a wavefront
 * masks the logits of the tokens whose mask words it has just written), provided the pointers, the row stride and V are
 * multiples of 16 bytes' worth of logits; in every other case the call enqueues the two kernels one after the other.  d_out may
 * equal d_logits; dtype 0 = fp32, 1 = bf16. */
int zf_compute_mask_apply_async(zf_engine *e, zf_state *const *states /* host array */, int32_t batch, uint32_t *d_mask,
                                const void *d_logits, void *d_out, int32_t dtype, int64_t row_stride_elems, void *hip_stream);
/* zf_compute_mask for callers that cannot allocate device memory: tight serving loops, harnesses
 * that forbid hipMalloc, code that runs while a HIP graph is being captured on another stream.  Same
 * arguments, same result, same waiting behaviour as zf_compute_mask, but the call allocates nothing
 * (no hipMalloc, hipHostMalloc, hipFree): every per-call device buffer (counters, rank-ordered verdict
 * words, fallback list and arenas, the trie walk's queue and chart copy) is a slice of one static
 * device array of 16 MiB that each GPU the library runs on holds until the process ends, and the
 * packed charts must fit the 256 KiB of pinned staging memory every engine owns from zf_compile on.
 * The state cache is passed by.  A call that does not fit -- batch x vocabulary beyond the array,
 * charts beyond the staging room -- returns ZF_ERR_INVALID_ARG with the sizes in zf_last_error, and so
 * does a call made while asynchronous mask calls are in flight.  The fallback pass has 32 wavefronts
 * with arenas of 16,384 items here, and its list holds what the other buffers leave of the array
 * (ZF_ERR_OVERFLOW beyond either, as always: the mask is then not valid).  All calls on one GPU,
 * from any engine, share the array: calls that overlap on one GPU (other streams, other threads)
 * race; one call after the other is fine, whatever their sizes. */
int zf_compute_mask_noalloc(zf_engine *e, zf_state *const *states /* host array */, int32_t batch,
                            uint32_t *d_mask, void *hip_stream);
int zf_last_mask_report(const zf_engine *e, zf_mask_report *out);
/* Forget every cached mask row and empty the persistent automata on the device and on the host: everything is
 * parsed again the next time it is needed (benchmarks call it to start cold).  Results do not change.  With
 * zf_options.precompute_states on, and no asynchronous mask call in flight, the automata are then explored from the
 * empty prefix again as when the engine was compiled (mask calls on the null stream, which this call waits for):
 * the engine is back to what it knew after zf_compile, not to nothing. */
int zf_engine_clear_state_cache(zf_engine *e);
/* on != 0: zf_compute_mask brackets each of its kernels with HIP events (a few microseconds
 * of extra host time per call) and zf_last_mask_report returns their durations. */
int zf_engine_set_profiling(zf_engine *e, int32_t on);

/* apply_mask(logits): out[b][v] = bit(b, v) ? logits[b][v] (bit copy) : -inf (Section 3.3).
 * d_logits / d_out: device, [batch][row_stride_elems] with V valid elements per row; d_out may
 * equal d_logits.  dtype: 0 = fp32, 1 = bf16.  Asynchronous on hip_stream. */
int zf_apply_mask(zf_engine *e, const void *d_logits, void *d_out, int32_t dtype, int32_t batch,
                  int64_t row_stride_elems, const uint32_t *d_mask, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
