/*
 * zapformat, test-only declarations: host-side diagnostics of the compiled tables.  Nothing here is
 * part of the product interface (include/zapformat.h); zf_compute_mask never calls any of it.  The
 * functions exist so that the host logic -- grammar tables, trie, token-mask cache, the automata
 * the mask kernels build -- can be tested without a GPU.
 */
#ifndef ZAPFORMAT_DEBUG_H
#define ZAPFORMAT_DEBUG_H
#include "zapformat.h"
#ifdef __cplusplus
extern "C" {
#endif

/* Diagnostic: the same verdicts computed on the host from the compiled tables (trie, DFAs,
 * chart).  Never used by zf_compute_mask; exists so the host logic can be tested without a GPU. */
int zf_debug_host_mask(zf_engine *e, const zf_state *s, uint32_t *mask /* host [W] */);
/* Same, plus counters of the walk in stats[0..4] (host): byte steps taken, steps that left a
 * live set, largest item count of one trie path, largest single set, chunks whose path
 * outgrows lane_item_cap (an estimate of what the fallback pass receives). */
int zf_debug_host_mask_stats(zf_engine *e, const zf_state *s, uint32_t *mask /* host [W] */, int64_t *stats);
/* Diagnostic: host walk that first merges the context-independent token-mask cache (Section
 * 4.3) of the current set's items and sends only the undecided strings through the parser, as
 * the kernel does.  stats[0..4] (host, may be null): byte steps, undecided strings, cache rows,
 * byte steps the chunk-wise kernel adds by replaying the path above each chunk, chunks walked. */
int zf_debug_host_mask_cached(zf_engine *e, const zf_state *s, uint32_t *mask /* host [W] */, int64_t *stats);
/* Diagnostic: host twin of the mask-automaton kernel.  The Earley sets met while checking one
 * row's tokens are the states of a deterministic automaton over byte classes; a transition is
 * computed by one Earley byte step (Section 3.2) the first time a token needs it and looked up
 * afterwards, sets are interned by content (the state-cache idea of Section 5.2 inside one
 * mask).  stats[0..4] (host, may be null): automaton states created, Earley byte steps taken,
 * transition look-ups, undecided strings, largest set. */
int zf_debug_host_mask_automaton(zf_engine *e, const zf_state *s, uint32_t *mask /* host [W] */, int64_t *stats);

/* Host twin of the persistent automaton (the mask kernels' cross-step store, Sections 4.4 / 5.2): every
 * Earley set is named by its content, items carrying the name of the set their rule started in, so the
 * sets of all rows and steps are the states of one automaton over byte classes.  A twin lives beside an
 * engine and keeps what it has computed.  State 0 names the empty prefix on input.
 *   zf_debug_twin_advance: walk n bytes from *state (Section 4.1: the update after a decoded token);
 *     ZF_ERR_REJECTED and *state unchanged if they cannot extend the prefix; *accepting = the prefix is a sentence.
 *   zf_debug_twin_mask: the vocabulary mask of a state; stats[0..4] (host, may be null): states in the
 *     store, Earley byte steps this call took, transition look-ups, undecided strings, items in the store. */
typedef struct zf_twin zf_twin;
int zf_debug_twin_new(zf_engine *e, zf_twin **out);
void zf_debug_twin_destroy(zf_twin *t);
int zf_debug_twin_advance(zf_twin *t, uint32_t *state, const uint8_t *bytes /* host */, int64_t n, int32_t *accepting);
int zf_debug_twin_mask(zf_twin *t, uint32_t state, uint32_t *mask /* host [W] */, int64_t *stats);

#ifdef __cplusplus
}
#endif
#endif
