// Mask kernel over the persistent automaton (zf_options.walk_mode = 2): mask_store_kernel, with the
// kernels that set the store up and bring a row's chart into it.
//
// Every Earley set is named by its content: its items, each with the NAME of the set its rule started
// in (not a position in some row's chart).  Named that way the sets of all rows and of all decode
// steps are the states of ONE deterministic automaton over byte classes, kept in device memory for
// the life of the engine:
//   - feeding the token that was just decoded (Section 4.1: the update after every decoding step) is
//     a walk of its bytes through the automaton from the row's current state: the host sends the
//     bytes, not the chart;
//   - the per-step token check walks every undecided vocabulary string through the same table;
//   - a transition is computed by one wavefront-cooperative Earley byte step (Scan + Complete with
//     tabulated Predict, Section 3.2) the first time any row, token or step needs it, and is a
//     look-up for everybody ever after (the reuse across steps that Sections 4.4 and 5.2 aim at).
// A state refers only to the sets its items started in, transitively, which is exactly what
// ZapFormat's reachability closure keeps of a chart (Section 4.2.3); completed items are dropped
// when a set is closed (Figure 3, first rule).  Nothing is ever removed from the store: when it
// fills up the host clears it and the rows come back in from their host charts (import_kernel).
//
// Concurrency.  A transition entry goes NONE -> BUSY -> final value, once; whoever swaps NONE for
// BUSY computes it; everybody else polls (the owner is a running wavefront that waits for nothing,
// so the wait ends; it is bounded all the same).  A new state is written completely (items, dead
// transitions, header) and released at device scope before any entry or hash-table slot names it.
// Table entries are read with device-scope atomic loads (they bypass the per-CU cache); a
// wavefront makes an acquire fence before it reads items it learnt of through such a load.
#include "zf_kernel_common.h"
#include "zf_aut_step.h"

namespace zf {
namespace {

static const uint32_t STORE_ROOT = 1;                  // the state of the empty prefix
static const uint32_t UNPUBLISHED = 0xFFFFFFFFu;
static const int LC_BITS = STORE_LC_BITS;               // block-local cache of table entries
static const uint32_t LC_ENTRIES = 1u << LC_BITS;
static const unsigned long long LC_EMPTY = 0xFFFFFFFF00000000ull;

__device__ __forceinline__ uint32_t g_load(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void g_store_release(uint32_t *p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ bool t_final(uint32_t t) { return t != AT_NONE && t != AT_BUSY; }
// A table entry changes NONE -> BUSY -> final value and never again, so a copy read through the caches is either
// right or "not there yet": look-ups read through the caches first and ask device memory (an atomic load, or the
// compare-and-swap that claims the entry) only when the cached answer is not final.

// Hundreds of wavefronts of a row can wait for the same entry: they ask less and less often, so that their polls do not
// slow the memory channel the owner works through (at most 64 x 64 cycles between two polls: 1.7 us).
__device__ __forceinline__ void poll_pause(uint32_t spins) {
    if (spins < 2) __builtin_amdgcn_s_sleep(8);
    else if (spins < 6) __builtin_amdgcn_s_sleep(24);
    else __builtin_amdgcn_s_sleep(64);
}

struct Staging { uint32_t *ctl; uint8_t *smem; const uint8_t *blob; uint32_t n16; uint8_t *rep; const uint8_t *rep_src; uint32_t ncls; bool wide_sets; };   // what ensure_tables needs; wide_sets: the rows' charts hold sets of many items
// The grammar tables are needed only by a wavefront that computes a transition, which is rare once the automaton has
// grown: the first such wavefront of a block copies them into LDS (ctl[4]: 0 = not there, 1 = being copied, 2 = there).
__device__ __forceinline__ bool ensure_tables(const Staging &g, uint32_t lane) {
    uint32_t *ctl = g.ctl;
    uint8_t *smem = g.smem;
    const uint8_t *blob = g.blob;
    const uint32_t n16 = g.n16;
    uint32_t st = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&ctl[4]));
    if (st == 0) {
        uint32_t old = 0;
        if (lane == 0) old = atomicCAS(&ctl[4], 0u, 1u);
        old = (uint32_t)__builtin_amdgcn_readfirstlane((int)old);
        if (old == 0) {
            const uint4 *src = reinterpret_cast<const uint4 *>(blob);
            uint4 *dst = reinterpret_cast<uint4 *>(smem);
            for (uint32_t k0 = 0; k0 < n16; k0 += 64 * 8) {   // eight 16-byte loads in flight per lane
                uint4 x[8];
#pragma unroll
                for (int u = 0; u < 8; u++) { const uint32_t k = k0 + (uint32_t)u * 64 + lane; x[u] = k < n16 ? src[k] : make_uint4(0, 0, 0, 0); }
#pragma unroll
                for (int u = 0; u < 8; u++) { const uint32_t k = k0 + (uint32_t)u * 64 + lane; if (k < n16) dst[k] = x[u]; }
            }
            for (uint32_t k = lane; k < g.ncls; k += 64) g.rep[k] = g.rep_src[k];   // one byte of every class
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) lds_store(&ctl[4], 2u);
            return true;
        }
        st = old;
    }
    for (uint32_t spins = 0; st != 2 && spins < (uint32_t)AUT_SPIN_LIMIT; spins++) {   // the copying wavefront waits for nothing
        __builtin_amdgcn_s_sleep(2);
        st = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&ctl[4]));
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return st == 2;
}

struct StoreSets {             // resolves the name of a set to its items (device memory)
    const StoreView &G;
    uint32_t *errors;
    __device__ __forceinline__ uint2 item(uint64_t h, uint32_t i) const { return reinterpret_cast<const uint2 *>((uintptr_t)h)[i]; }
    __device__ __forceinline__ void view(uint32_t ref, uint64_t &p, uint32_t &n) const {   // the handle is the address of the set's first item
        uint2 h = make_uint2(0, 0);
        if (ref < G.cap_states) h = G.hdr[ref];
        // a name that leads nowhere cannot come from a correct store: read nothing, and fail the call loudly
        if (ref >= G.cap_states || h.y > G.cap_items || h.x > G.cap_items - h.y) { h = make_uint2(0, 0); atomicAdd(errors, 1u); }
        p = (uint64_t)(uintptr_t)(G.arena + h.x);
        n = h.y;
    }
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
struct Scratch { uint32_t *w, *o, *h; uint32_t cap; };   // one wavefront's set under construction (+ hash table of the wide step)

// true when state `id` holds exactly the `kept` items in the scratch
__device__ __forceinline__ bool same_content(const StoreView &G, uint32_t id, const Scratch &sc, uint32_t kept, uint32_t lane) {
    if (id == 0 || id >= G.cap_states) return false;
    const uint2 hj = G.hdr[id];
    if (hj.y != kept || hj.x > G.cap_items - kept) return false;
    unsigned long long diff = 0;
    for (uint32_t i0 = 0; i0 < kept; i0 += 64) {
        bool ne = false;
        if (i0 + lane < kept) { const uint2 x = G.arena[hj.x + i0 + lane]; ne = x.x != lds_load(&sc.w[i0 + lane]) || x.y != lds_load(&sc.o[i0 + lane]); }
        diff |= __ballot(ne);
    }
    return diff == 0;
}

// The transition of state s on class cl: one Earley byte step, then the state that holds the
// resulting set -- found by content in the store's hash table, or made.  Uniform over the wavefront.
// Returns a state id, AT_DEAD, AT_SINK or AT_FAIL (no room in the scratch or in the store).
__device__ __forceinline__ uint32_t store_transition(const TV &T, const StoreView &G, const Scratch &sc, const Staging &stg, uint32_t *errors,
                                                     uint32_t s, uint32_t cl, uint32_t lane) {
    if (!ensure_tables(stg, lane)) return AT_FAIL;
    const uint8_t *rep = stg.rep;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");      // s and every set it refers to were released before the entry that led here
    const StoreSets S{G, errors};
    uint32_t nnew = 0, kept = 0;
    uint64_t src_p;
    uint32_t src_n;
    S.view(s, src_p, src_n);
    const uint32_t byte = rep[cl];
    // the narrow step takes sets of up to 64 items; where the charts hold wide sets (an ambiguous grammar) a source set of more
    // than a few items rarely leaves a narrow one, and the narrow step's one-candidate-at-a-time Complete would be wasted
    const bool wide_first = src_n > 64u || (stg.wide_sets && src_n > (uint32_t)AUT_NARROW_SET_MAX);
    int st = wide_first ? (int)AUT_WIDE : aut_step_narrow<true>(T, S, sc.w, sc.o, sc.cap, s, byte, cl, lane, nnew, kept);
    if (st == AUT_WIDE) st = aut_step_wide(T, S, sc.w, sc.o, sc.h, sc.cap, s, byte, cl, lane, nnew, kept);
    if (st != AUT_OK) return AT_FAIL;
    if (nnew == 0) return AT_DEAD;
    if (kept == 0) return AT_SINK;
    // signature of the content (never 0: 0 marks a free slot of the hash table)
    uint32_t h = 0x811C9DC5u;
    for (uint32_t i0 = 0; i0 < kept; i0 += 64) {
        uint32_t x = 0;
        if (i0 + lane < kept) { x = (lds_load(&sc.w[i0 + lane]) * 0x9E3779B1u) ^ (lds_load(&sc.o[i0 + lane]) * 0x85EBCA77u); x ^= x >> 15; x *= (2u * (i0 + lane) + 1u) * 0x2C1B3C6Du; }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d);
        h = (h ^ x) * 0x01000193u;
    }
    h = (uint32_t)__builtin_amdgcn_readfirstlane((int)(h ^ kept)) | 1u;
    uint32_t slot = (h * 0x9E3779B1u) & G.intern_mask;
    for (uint32_t probes = 0; probes <= G.intern_mask; probes++) {
        const unsigned long long e = __hip_atomic_load(&G.intern[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (e == 0) break;
        if ((uint32_t)(e >> 32) == h) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // the state was released before its slot was written
            if (same_content(G, (uint32_t)e, sc, kept, lane)) return (uint32_t)e;
        }
        slot = (slot + 1) & G.intern_mask;
    }
    uint32_t id = 0, at = 0;
    if (lane == 0) { id = atomicAdd(&G.ctl[0], 1u); at = atomicAdd(&G.ctl[1], kept); }
    id = (uint32_t)__builtin_amdgcn_readfirstlane((int)id);
    at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
    if (id >= G.cap_states || at > G.cap_items - kept) { if (lane == 0) atomicAdd(&G.ctl[2], 1u); return AT_FAIL; }   // the store is full
    for (uint32_t i0 = 0; i0 < kept; i0 += 64)
        if (i0 + lane < kept) G.arena[at + i0 + lane] = make_uint2(lds_load(&sc.w[i0 + lane]), lds_load(&sc.o[i0 + lane]));
    uint32_t *row = G.trans + (size_t)id * T.ncls;
    aut_mark_dead<true>(T, T.ncls, rep, [&](uint32_t i) { return lds_load(&sc.w[i]); }, kept, lane, [&](uint32_t c) { row[c] = AT_DEAD; });
    if (lane == 0) G.hdr[id] = make_uint2(at, kept);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");      // items, dead entries and header before anything that names the state
    for (uint32_t probes = 0; probes <= G.intern_mask; probes++) {
        unsigned long long old = 0;
        if (lane == 0) old = atomicCAS(&G.intern[slot], 0ull, ((unsigned long long)h << 32) | id);
        old = ((unsigned long long)(uint32_t)__builtin_amdgcn_readfirstlane((int)(old >> 32)) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)old);
        if (old == 0) return id;
        if ((uint32_t)(old >> 32) == h) {                    // somebody made the same set meanwhile: theirs is the name
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            if (same_content(G, (uint32_t)old, sc, kept, lane)) return (uint32_t)old;
        }
        slot = (slot + 1) & G.intern_mask;
    }
    return id;                                               // the table has twice as many slots as states: not reached
}

// Look the transition (s, cl) up for the whole wavefront (uniform arguments), computing it if nobody has.
__device__ __forceinline__ uint32_t store_lookup_uniform(const TV &T, const StoreView &G, const Scratch &sc, const Staging &stg, uint32_t *errors,
                                                         uint32_t *steps, uint32_t s, uint32_t cl, uint32_t lane) {
    uint32_t *entry = G.trans + (size_t)s * T.ncls + cl;
    // the read through the caches answers at once when the entry is final; else the claim itself (a compare-and-swap,
    // which returns what device memory holds) is the fresh read
    uint32_t t = (uint32_t)__builtin_amdgcn_readfirstlane((int)__hip_atomic_load(entry, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT));
    if (t_final(t)) return t;
    if (lane == 0) t = atomicCAS(entry, (uint32_t)AT_NONE, (uint32_t)AT_BUSY);
    t = (uint32_t)__builtin_amdgcn_readfirstlane((int)t);
    if (t == AT_NONE) {
        const uint32_t r = store_transition(T, G, sc, stg, errors, s, cl, lane);
        ++*steps;
        if (lane == 0) g_store_release(entry, r);            // everything the transition wrote, then the entry
        return r;
    }
    for (uint32_t spins = 0; !t_final(t) && spins < (uint32_t)AUT_SPIN_LIMIT; spins++) {   // the owner is a running wavefront that waits for nothing
        poll_pause(spins);
        t = (uint32_t)__builtin_amdgcn_readfirstlane((int)g_load(entry));
    }
    return t_final(t) ? t : (uint32_t)AT_FAIL;
}

// Grid (blocks of all rows), blocks of STORE_WAVES wavefronts.  The kernel works in TOKEN order and writes the caller's mask
// rows itself: nothing has to be permuted afterwards.  The wavefronts of a block work on their own; what they share is
// the block's LDS cache of table entries and (once somebody needs them) the staged grammar tables.  A wavefront
//  (a) takes its row's record -- start state, pending bytes, token-mask-cache row numbers -- from the kernel's argument
//      block (calls of up to STORE_MINI_ROWS rows), else from the call's upload with one 128-byte load;
//  (b) requests the token-mask cache words (Section 4.3) of its segment of STORE_SEG_WORDS mask words, and while they are
//      on their way walks the row's pending bytes (the tokens fed since the row's state was last known) from that state to
//      the row's current state, then warms the LDS cache with the current state's table row;
//  (c) takes the undecided tokens of the segment, 64 at a time, one lane per token, through the transition table: first the
//      LDS cache, then device memory, and an Earley byte step for what nobody has computed yet;
//  (d) stores the segment's words of the row's mask (the next segment's cache words are requested before (c)).
// No block-wide barrier between the first one and the hand-over of the call's status at the end.
template <int MODE>
__global__ __launch_bounds__(STORE_BLOCK) void mask_store_kernel(MaskArgs a, StoreMiniRows mini) {
    extern __shared__ __align__(16) uint8_t smem[];
    __shared__ uint32_t block_undecided;                     // tokens the block's wavefronts walked through the table (for the report)
    const DeviceTables &D = a.tab;
    const StoreView &G = a.store;
    const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const uint32_t W = (uint32_t)D.W, ncls = (uint32_t)D.n_cls;
    if (tid == 0) block_undecided = 0;
    // LDS: the cache of table entries and the staging flag come first, at offsets that do not depend on the kernel's arguments:
    // they are cleared while the arguments are still on their way
    unsigned long long *lc = reinterpret_cast<unsigned long long *>(smem);
    uint32_t *ctl = reinterpret_cast<uint32_t *>(smem + LC_ENTRIES * 8);   // [4] state of the staged tables
    uint8_t *const tables_at = smem + LC_ENTRIES * 8 + 32;
    for (uint32_t k = tid; k < LC_ENTRIES; k += STORE_BLOCK) lc[k] = LC_EMPTY;
    if (tid == 0) ctl[4] = 0;
    __syncthreads();
    // Grid (blocks of the row that has most, rows): the row's record -- with the number of blocks the row really has -- is
    // the first thing read, from the kernel's argument block when the call has few enough rows (one read; a block beyond its
    // row's count leaves at once).
    const uint32_t use_mini = (uint32_t)a.store_mini, uniform_parts = (uint32_t)a.store_uniform_parts;
    // Which row the block belongs to is known only once the rows' first blocks have been read, and the row's record only
    // after that: so lane l asks for the first block AND the twelve words of the record of row l, all at once, and the
    // wavefront picks its row's out of the lanes (one trip to the argument block instead of two, one after the other).
    static_assert(STORE_MINI_ROWS == 64 && sizeof(StoreRowMini) == 48, "one short record per lane");
    uint32_t rw[12];
    {
        const uint32_t *mp = reinterpret_cast<const uint32_t *>(&mini);
#pragma unroll
        for (int k = 0; k < 12; k++) rw[k] = mp[lane * 12u + (uint32_t)k];
    }
    const uint32_t fbv = a.store_first_block[lane], fbv2 = a.store_first_block[lane + 1u];
    const uint32_t n_before = (uint32_t)__popcll(__ballot(blockIdx.x >= fbv));   // rows that start at or before this block (0xFFFF beyond the call's rows)
    const uint32_t row = uniform_parts ? blockIdx.x / (uniform_parts ? uniform_parts : 1u) : n_before - 1u;
    const uint32_t frow = row < (uint32_t)STORE_MINI_ROWS ? row : 0u;
    StoreRowMini m;
    {
        uint32_t *mw = reinterpret_cast<uint32_t *>(&m);
#pragma unroll
        for (int k = 0; k < 12; k++) mw[k] = (uint32_t)__builtin_amdgcn_readlane((int)rw[k], (int)frow);
    }
    const uint32_t fb0 = (uint32_t)__builtin_amdgcn_readlane((int)fbv, (int)frow), fb1 = (uint32_t)__builtin_amdgcn_readlane((int)fbv2, (int)frow);
    const uint32_t part = uniform_parts ? blockIdx.x - row * uniform_parts : blockIdx.x - fb0;
    const uint32_t parts = uniform_parts ? uniform_parts : fb1 - fb0;
    // mask words a wavefront takes per pass: the host picks fewer for rows most of whose tokens are undecided, so that a pass
    // holds about one batch of 64 tokens and the row can be dealt to more wavefronts
    const uint32_t sw = use_mini ? ((m.meta >> 24) & 63u) + 1u : (uint32_t)STORE_SEG_WORDS;
    // lanes per copy of the segment: the wavefront holds the segment's words 64 / slots times over, and each copy ORs its
    // share of the row's cache rows (16 words: four copies; up to 64 words -- rows few of whose tokens are undecided: one)
    const uint32_t slots_log2 = sw <= 16u ? 4u : (sw <= 32u ? 5u : 6u), slots = 1u << slots_log2, n_grp = 64u >> slots_log2;
    const uint32_t n_seg = (W + sw - 1) / sw;
    const uint32_t unit = part * STORE_WAVES + wave, n_units = parts * STORE_WAVES;   // a unit = one wavefront of one of the row's blocks
    uint32_t steps = 0;
    if (part < parts && (part * STORE_WAVES < n_seg || part == 0)) {   // uniform over the block (the row's first block reports the row's state even when there is no mask word)
    // the row's record in the layout of StoreRow: lane k holds word k
    uint32_t rec = 0;
    const bool spilled = !use_mini || ((m.meta >> 16) & STORE_ROW_SPILL) != 0;
    {
        const uint32_t *mw = reinterpret_cast<const uint32_t *>(&m);
        rec = lane == 0u ? m.start : rec;
        rec = lane == 1u ? (m.meta & 0xFFu) : rec;
        rec = lane == 3u ? ((m.meta >> 8) & 0xFFu) : rec;
        rec = lane == 5u ? (m.meta >> 16) : rec;
#pragma unroll
        for (int k = 0; k < STORE_MINI_ENT; k++) rec = lane == (uint32_t)(STORE_ROW_ENT_AT + k) ? ((mw[6 + k / 2] >> (16 * (k & 1))) & 0xFFFFu) : rec;
#pragma unroll
        for (int k = 0; k < STORE_MINI_PEND / 4; k++) rec = lane == (uint32_t)(STORE_ROW_PEND_AT + k) ? mw[2 + k] : rec;
    }
    if (spilled) rec = lane < sizeof(StoreRow) / 4 ? reinterpret_cast<const uint32_t *>(a.store_rows + row)[lane] : 0u;
    TV T;
    uint32_t off = table_view<MODE>(D, tables_at, T);
    const uint32_t n16 = off / 16;
    uint8_t *l_rep = tables_at + off; off += 256;
    uint32_t *vbuf = reinterpret_cast<uint32_t *>(tables_at + off) + wave * 64; off += STORE_WAVES * 64 * 4;   // per wavefront: verdicts of the pass's words
    const Staging stg{ctl, tables_at, D.table_blob, n16, l_rep, D.cls_rep, ncls, a.aut_wide != 0};
    Scratch sc;
    sc.cap = (uint32_t)a.aut_scratch;
    sc.w = reinterpret_cast<uint32_t *>(tables_at + off) + (size_t)wave * (2 * sc.cap + aut_hash_places(sc.cap));
    sc.o = sc.w + sc.cap;
    sc.h = sc.o + sc.cap;
    if (unit < n_seg || unit == 0) {
    auto field = [&](uint32_t k) { return (uint32_t)__builtin_amdgcn_readlane((int)rec, (int)k); };
    const uint32_t flags = field(5), n_pending = field(1), pend_off = field(2), n_ent = field(3), ent_off = field(4);
    uint32_t start = field(0);
    if (flags & STORE_ROW_IMPORTED) start = a.store_import_root[row];
    const bool use_cache = (flags & STORE_ROW_CACHE) != 0;
    const bool ent_inline = n_ent <= (uint32_t)STORE_ROW_ENT, pend_inline = n_pending <= (uint32_t)(spilled ? STORE_ROW_PEND : STORE_MINI_PEND);
    // the row number of cache row k0 + (the lane's group): the groups' numbers are read out of the record one by one (lane
    // reads with a uniform index: no trip through LDS, which a shuffle would be) and each lane keeps its group's
    auto entry = [&](uint32_t k0, uint32_t k) -> uint32_t {
        uint32_t inl = 0;
        for (uint32_t j = 0; j < n_grp; j++) {
            const uint32_t kj = k0 + j < (uint32_t)STORE_ROW_ENT ? k0 + j : 0u;
            const uint32_t ej = (uint32_t)__builtin_amdgcn_readlane((int)rec, (int)(STORE_ROW_ENT_AT + kj));
            inl = (lane >> slots_log2) == j ? ej : inl;
        }
        return ent_inline ? inl : a.entries[ent_off + k];
    };
    auto pending = [&](uint32_t k) -> uint32_t {
        return pend_inline ? (field(STORE_ROW_PEND_AT + (k >> 2)) >> ((k & 3u) * 8u)) & 0xFFu : (uint32_t)a.store_pending[pend_off + k];
    };
    uint32_t root = AT_FAIL, undecided = 0;
    uint32_t *errors = &a.counters[2];
    uint32_t *out_row = a.out_mask + (size_t)(a.dst_row ? a.dst_row[row] : row) * W;
    const uint32_t slot16 = lane & (slots - 1u), grp = lane >> slots_log2;    // lane = (word of the segment, which copy)
    // the token-mask cache words of segment g: every quarter of the wavefront ORs a quarter of the row's cache rows
    auto request = [&](uint32_t g, uint32_t &v, uint32_t &c) {
        const uint32_t w = slot16 < sw ? g * sw + slot16 : 0xFFFFFFFFu;
        v = 0; c = use_cache ? 0u : 0xFFFFFFFFu;
        if (use_cache && g < n_seg)
            for (uint32_t k0 = 0; k0 < n_ent; k0 += n_grp) { // uniform trip count: the row numbers come by shuffle
                const uint32_t k = k0 + grp;
                const uint32_t er = entry(k0, k < n_ent ? k : 0u);
                if (k < n_ent && w < W) { const size_t r = (size_t)er * W + w; v |= D.ci_valid_tok[r]; c |= D.ci_cd_tok[r]; }
            }
    };
    // the first look-up of the pending walk is requested ahead of the cache words: loads come back in the order they were issued
    uint32_t hop0 = AT_NONE;
    const bool start_ok = start != 0 && start < G.cap_states;
    if (n_pending && start_ok && pending(0) < ncls) hop0 = __hip_atomic_load(&G.trans[start * ncls + pending(0)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    uint32_t v = 0, c = 0;
    request(unit, v, c);
    // The logits of a segment (when the call masks them too): 16-byte pieces, the first two of every lane requested one pass
    // ahead (those of the first segment here), so that they wait in registers when the segment's verdicts are in.
    const uint32_t tp = a.apply_dtype ? 8u : 4u, esz = a.apply_dtype ? 2u : 4u;   // tokens per 16-byte piece, bytes per logit
    auto logits_of = [&](uint32_t g, uint32_t &pieces, size_t &at) {
        const uint32_t tok0 = g * sw * 32u;
        const uint32_t n_tok = a.apply_out && g < n_seg && tok0 < (uint32_t)D.V ? (sw * 32u < (uint32_t)D.V - tok0 ? sw * 32u : (uint32_t)D.V - tok0) : 0u;
        pieces = n_tok / tp;
        at = ((size_t)row * (size_t)a.apply_stride + tok0) * esz;
    };
    auto logits_ahead = [&](uint32_t g, u32x4 (&pre)[2]) {
        uint32_t pieces;
        size_t at;
        logits_of(g, pieces, at);
        const u32x4 *src = reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint8_t *>(a.apply_logits) + at);
#pragma unroll
        for (int u = 0; u < 2; u++) { pre[u] = u32x4{0, 0, 0, 0}; if ((uint32_t)u * 64u + lane < pieces) pre[u] = __builtin_nontemporal_load(src + (uint32_t)u * 64u + lane); }
    };
    u32x4 l_pre[2];
    logits_ahead(unit, l_pre);
    auto find_root = [&]() {
        // ---- the row's current state: walk the bytes fed since `start` was its state (the loads above are in flight) ----
        uint32_t s = start;
        bool bad = s == 0 || (s >= G.cap_states && s != AT_SINK);
        for (uint32_t k = 0; k < n_pending && !bad; k++) {
            const uint32_t cl = pending(k);
            if (s == AT_SINK || cl >= ncls) { bad = true; break; }
            uint32_t t = k == 0 ? (uint32_t)__builtin_amdgcn_readfirstlane((int)hop0) : (uint32_t)AT_NONE;
            if (!t_final(t)) t = store_lookup_uniform(T, G, sc, stg, errors, &steps, s, cl, lane);
            if (t == AT_DEAD || t == AT_FAIL) { bad = true; break; }   // the host accepted these bytes: a dead end here is an error
            s = t;
        }
        if (bad) { s = AT_FAIL; if (lane == 0 && unit == 0) atomicAdd(errors, 1u); }
        // The host reads this word once it has seen the call's status.  It is written through to device memory here (no fence:
        // a release would write the whole L2 back, and every wavefront of the chip would wait behind that), long before this
        // block draws its ticket; the block that hands the status over reads it back and passes it on.
        if (unit == 0 && lane == 0) __hip_atomic_store(&a.store_row_dev[row], s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        root = s;
        if (root < AT_FAIL) {
            // Warm the block's cache with the current state's row of the table, and with the rows of the states one byte
            // away (every wavefront of the block takes its share of them): a row is read by neighbouring lanes, once per
            // block.  Left to the walk below, thousands of wavefronts would ask for the same few lines at the same
            // moment, lane by lane, and queue up at the one memory channel that holds them (8 us and more).
            auto warm_row = [&](uint32_t st) {
                for (uint32_t c0 = 0; c0 < ncls; c0 += 64) {
                    const uint32_t cl = c0 + lane;
                    uint32_t t = AT_NONE;
                    const uint32_t key = st * ncls + cl;
                    if (cl < ncls) t = __hip_atomic_load(&G.trans[key], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                    if (cl < ncls && t_final(t) && t != AT_FAIL)
                        __hip_atomic_store(&lc[(key * 0x9E3779B1u) >> (32 - LC_BITS)], ((unsigned long long)key << 32) | t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    // the states this row leads to, each once: the wavefront's share of them is warmed in turn
                    if (st == root) {
                        unsigned long long todo = __ballot(cl < ncls && t < AT_FAIL && t != root);
                        constexpr int SHARE = (STORE_WARM_ROWS + STORE_WAVES - 1) / STORE_WAVES;
                        uint32_t mine[SHARE], n_mine = 0, n_done = 0;
#pragma unroll
                        for (int k = 0; k < SHARE; k++) mine[k] = 0;
                        while (todo && n_done < (uint32_t)STORE_WARM_ROWS) {
                            const int l = __ffsll((long long)todo) - 1;
                            const uint32_t nx = (uint32_t)__builtin_amdgcn_readlane((int)t, l);
                            todo &= ~__ballot(t == nx);
                            if (n_done % STORE_WAVES == wave && ncls <= 64u) {
#pragma unroll
                                for (int k = 0; k < SHARE; k++) mine[k] = n_mine == (uint32_t)k ? nx : mine[k];
                                n_mine++;
                            }
                            n_done++;
                        }
                        uint32_t t2[SHARE];                  // the rows' loads travel together
#pragma unroll
                        for (int k = 0; k < SHARE; k++) {
                            t2[k] = AT_NONE;
                            if ((uint32_t)k < n_mine && lane < ncls) t2[k] = __hip_atomic_load(&G.trans[mine[k] * ncls + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                        }
#pragma unroll
                        for (int k = 0; k < SHARE; k++) {
                            const uint32_t k2 = mine[k] * ncls + lane;
                            if ((uint32_t)k < n_mine && lane < ncls && t_final(t2[k]) && t2[k] != AT_FAIL)
                                __hip_atomic_store(&lc[(k2 * 0x9E3779B1u) >> (32 - LC_BITS)], ((unsigned long long)k2 << 32) | t2[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                        }
                    }
                }
            };
            warm_row(root);
        }
    };
    // One token of a batch: where its verdict goes, and its string (requested here, used a batch later).
    struct Tok { uint32_t slot, bit, len, token; Str16 c16; bool live; };
    uint32_t incl = 0, want = 0;                             // of the segment in hand: running bit counts of its words, undecided bits
    auto fetch = [&](uint32_t g, uint32_t b0, uint32_t total) -> Tok {
        Tok k;
        const uint32_t i = b0 + lane;
        k.live = i < total;
        k.slot = 0;                                          // the word that holds the lane's token: the first whose running count exceeds i (by bisection)
        for (uint32_t half = slots >> 1; half; half >>= 1) k.slot += i >= (uint32_t)__shfl((int)incl, (int)(k.slot + half - 1u)) ? half : 0u;
        const uint32_t before = (uint32_t)__shfl((int)incl, (int)(k.slot ? k.slot - 1 : 0));
        const uint32_t bits = (uint32_t)__shfl((int)want, (int)k.slot);
        uint32_t n = i - (k.slot ? before : 0u);             // the n-th set bit of the word, by halving
        k.bit = 0;
#pragma unroll
        for (int sh = 16; sh >= 1; sh >>= 1) {
            const uint32_t low = (uint32_t)__popc(bits & (((1u << sh) - 1u) << k.bit));
            if (n >= low) { n -= low; k.bit += (uint32_t)sh; }
        }
        k.token = (g * sw + k.slot) * 32u + k.bit;
        k.len = 0;
        k.c16 = Str16{{0, 0, 0, 0}};
        if (k.live) { k.len = D.tok_len[k.token]; k.c16 = D.tok16[k.token]; }   // requested here, looked at a batch later: nothing below waits for them
        return k;
    };
    bool root_ok = false;
    // the first pass runs even for a wavefront without a segment (the row's first wavefront reports the row's state)
    for (uint32_t g = unit, first = 1; first || g < n_seg; g += n_units, first = 0) {
        const uint32_t w = slot16 < sw && g < n_seg ? g * sw + slot16 : 0xFFFFFFFFu;
        uint32_t vn = 0, cn = 0;
        request(g + n_units, vn, cn);                        // the next segment's words travel while this one's tokens are checked
        u32x4 l_nxt[2];
        logits_ahead(g + n_units, l_nxt);                    // and so do its logits
        uint32_t pieces;
        size_t l_at;
        logits_of(g, pieces, l_at);
        const u32x4 *l_src = reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint8_t *>(a.apply_logits) + l_at);
        if (slots_log2 <= 4u) { v |= __shfl_xor(v, 16); c |= __shfl_xor(c, 16); }
        if (slots_log2 <= 5u) { v |= __shfl_xor(v, 32); c |= __shfl_xor(c, 32); }
        want = c & ~v;
        {
            const uint32_t t0 = w * 32u;
            if (w >= W || t0 >= (uint32_t)D.V) want = 0;
            else if ((uint32_t)D.V - t0 < 32u) want &= (1u << ((uint32_t)D.V - t0)) - 1u;
        }
        // ---- one lane per undecided token through the table.  The undecided tokens of the segment's words are numbered
        // through (prefix sum of the words' bit counts) and taken 64 at a time, so that a batch is full whatever the
        // pattern of the bits; verdicts go back to their words through LDS.  The strings of a batch are requested one
        // batch ahead; those of the first batch travel while the row's current state is worked out ----
        incl = (uint32_t)__popc(want);                       // every copy holds the same words
        // running sums over each copy's lanes by data-parallel-primitive moves (a row of 16 lanes shifts by 1, 2, 4, 8 with
        // zeros coming in; then the last lane of a row is broadcast into the next row, of the lower half into the upper half):
        // six vector instructions where shuffles would be six trips through LDS
        incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x111, 0xF, 0xF, true);   // row_shr:1
        incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x112, 0xF, 0xF, true);   // row_shr:2
        incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x114, 0xF, 0xF, true);   // row_shr:4
        incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x118, 0xF, 0xF, true);   // row_shr:8
        if (slots_log2 >= 5u) incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
        if (slots_log2 >= 6u) incl += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)incl, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
        uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, (int)(slots - 1u));
        Tok nxt = fetch(g, 0, total);
        if (first) { find_root(); root_ok = root < AT_FAIL; }   // AT_SINK: nothing can follow; AT_FAIL: the call fails
        if (!root_ok) { total = 0; v = 0; }                  // no token can follow a finished sentence
        undecided += total;
        if (lane < slots) lds_store(&vbuf[lane], 0u);
        for (uint32_t b0 = 0; b0 < total; b0 += 64) {
            const Tok cur = nxt;
            if (b0 + 64 < total) nxt = fetch(g, b0 + 64, total);
            const uint32_t slot = cur.slot, bit = cur.bit;
            uint32_t soff = 0, len = cur.len;
            const Str16 c16 = cur.c16;
            const bool long_one = cur.live & (len == (uint32_t)TOK_LEN_LONG);   // longer than the 16 classes at hand: the rest is with the string's rank
            if (__ballot(long_one)) {
                if (long_one) {
                    const uint32_t rank = D.rank_of[cur.token];
                    soff = D.str_off[rank]; len = D.str_off[rank + 1] - soff;
                }
            }
            // Where a lane stands with its string, in ONE register: the loop below carries no per-lane truth value from one
            // round to the next.  (Carried truth values live in scalar register pairs, and every one of them costs three
            // scalar instructions per round to merge; the four vector units of a compute unit share one scalar unit, which
            // was what bounded the walk.)
            enum : uint32_t { PH_GO = 0,      // takes a step in the next round
                              PH_NONE = 1,    // waits: nobody has computed the entry it needs
                              PH_BUSY = 2,    // waits: somebody is computing it
                              PH_FAR = 3,     // beyond the 16 bytes at hand: the next byte has to be fetched
                              PH_OK = 4,      // done: the whole string went through (codes from here on: done)
                              PH_DEAD = 5,    // done: the string cannot follow
                              PH_FAIL = 6 };  // done: no room, or a wait that did not end
            // what a step that found no state makes of a lane, a nibble per special value (~value = 0 .. 4): not computed,
            // dead, nothing can follow (the one string that ends right here is picked out below), being computed, no room
            constexpr uint32_t PH_OF_SPECIAL = (PH_NONE << 0) | (PH_DEAD << 4) | (PH_DEAD << 8) | (PH_BUSY << 12) | (PH_FAIL << 16);
            static_assert(AT_NONE == ~0u && AT_DEAD == ~1u && AT_SINK == ~2u && AT_BUSY == ~3u && AT_FAIL == ~4u, "the nibbles above");
            uint32_t ph = cur.live && len > 0 ? (uint32_t)PH_GO : (uint32_t)PH_DEAD;
            uint32_t s = root, pos = 0, spins = 0, rounds = 0;
            uint32_t c_far = 0;                              // class of the byte at `pos` of a string beyond the 16 at hand (fetched while the lane is PH_FAR)
            const uint32_t w0 = c16.w[0], w1 = c16.w[1], w2 = c16.w[2], w3 = c16.w[3];
            auto class_at = [&](uint32_t at) -> uint32_t {  // byte `at` of the sixteen at hand: the half that holds it, then one byte permute
                const bool upper = (at & 8u) != 0;
                const uint32_t c_near = __builtin_amdgcn_perm(upper ? w3 : w1, upper ? w2 : w0, (at & 7u) | 0x0C0C0C00u);
                return at >= 16u ? c_far : c_near;
            };
            for (;;) {
                // Every lane follows its own string as far as the table goes: all lanes that can move take a step together,
                // written without branches on per-lane conditions (selects; an entry that is not in the block's LDS cache
                // sits behind a wavefront-uniform test).  No result of a load from device memory is used on the way round
                // when every lane finds its entry: the loop never waits for what was requested ahead (the next batch's
                // strings, the next segment's words and logits).
                ph = ph == PH_NONE || ph == PH_BUSY ? (uint32_t)PH_GO : ph;   // those that waited look again
                for (;;) {
                    const bool go = ph == PH_GO;
                    if (!__builtin_amdgcn_ballot_w64(go)) break;
                    const uint32_t c_new = class_at(pos);
                    const uint32_t key = __umul24(s, ncls) + c_new;          // a state has at most 18 bits, a class 8
                    const uint32_t lslot = go ? (key * 0x9E3779B1u) >> (32 - LC_BITS) : 0u;
                    const unsigned long long e = __hip_atomic_load(&lc[lslot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    const bool hit = (uint32_t)(e >> 32) == key;
                    uint32_t t_new = hit ? (uint32_t)e : (uint32_t)AT_NONE;
                    const bool miss = go & !hit;
                    if (__builtin_amdgcn_ballot_w64(miss)) {
                        if (miss) {
                            // through the caches first; an entry seen unfinished is asked of device memory only on the
                            // way back from the claim below, which is itself a fresh read of the entry it claims
                            t_new = __hip_atomic_load(&G.trans[key], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                            if (!t_final(t_new) && rounds) t_new = g_load(&G.trans[key]);
                            if (t_final(t_new) && t_new != AT_FAIL) __hip_atomic_store(&lc[lslot], ((unsigned long long)key << 32) | t_new, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                        }
                    }
                    const bool state = t_new < AT_FAIL;      // a state: the lane moves on
                    const uint32_t pos1 = pos + 1u;
                    const bool ends = pos1 == len;
                    uint32_t nx = __builtin_amdgcn_ubfe(PH_OF_SPECIAL, (~t_new) << 2, 4u);
                    nx = state ? (pos1 >= 16u ? (uint32_t)PH_FAR : (uint32_t)PH_GO) : nx;
                    nx = ((state | (t_new == AT_SINK)) & ends) ? (uint32_t)PH_OK : nx;   // (& and | on purpose: && and || would ask for a branch apiece)
                    const bool adv = go & state;
                    s = adv ? t_new : s;
                    pos = adv ? pos1 : pos;
                    ph = go ? nx : ph;
                }
                if (!__builtin_amdgcn_ballot_w64(ph < PH_OK)) break;
                {
                    const bool fetch_far = ph == PH_FAR;
                    if (__builtin_amdgcn_ballot_w64(fetch_far)) {   // strings beyond 16 bytes: the next byte's class, then round again
                        if (fetch_far) {
                            c_far = D.str_cls[soff + pos];
                            asm volatile("" : "+v"(c_far));  // waited for here, not at the top of the loop above
                            ph = PH_GO;
                        }
                        continue;
                    }
                }
                rounds++;
                // one of the waiting lanes' transitions is claimed and computed here; the other lanes look again afterwards
                const unsigned long long missing = __builtin_amdgcn_ballot_w64(ph == PH_NONE);
                bool progress = false;
                if (missing) {
                    const int l = __ffsll((long long)missing) - 1;
                    const uint32_t rs = (uint32_t)__builtin_amdgcn_readlane((int)s, l), rc = (uint32_t)__builtin_amdgcn_readlane((int)class_at(pos), l);
                    uint32_t old = 0;
                    if (lane == 0) old = atomicCAS(&G.trans[rs * ncls + rc], (uint32_t)AT_NONE, (uint32_t)AT_BUSY);
                    old = (uint32_t)__builtin_amdgcn_readfirstlane((int)old);
                    if (old == AT_NONE) {
                        const uint32_t r = store_transition(T, G, sc, stg, errors, rs, rc, lane);
                        steps++;
                        if (lane == 0) g_store_release(&G.trans[rs * ncls + rc], r);   // everything the transition wrote, then the entry
                        progress = true;
                    } else progress = old != AT_BUSY;        // somebody else has it, or has finished it meanwhile
                }
                if (progress) spins = 0;
                else {
                    poll_pause(spins);
                    if (++spins > (uint32_t)AUT_SPIN_LIMIT) ph = ph < PH_OK ? (uint32_t)PH_FAIL : ph;   // bounded wait
                }
                // Nothing this slow path asked of device memory is outstanding when the walk above starts again (vmcnt 0; the
                // other two counters left alone).  Said explicitly, because the compiler otherwise has to assume that one of
                // the loads in here may still be on its way to a register the walk reuses, and waits at the top of the walk on
                // every round -- for the strings, words and logits requested ahead as well.
                __builtin_amdgcn_s_waitcnt(0x0F70);
            }
            if (ph == PH_OK) atomicOr(&vbuf[slot], 1u << bit);
            const unsigned long long fm = __builtin_amdgcn_ballot_w64(ph == PH_FAIL);    // no room in the scratch or the store, or a wait that did not end
            if (lane == 0 && fm) atomicAdd(errors, (uint32_t)__popcll(fm));
        }
        if (total) v |= lds_load(&vbuf[slot16]);             // LDS serves one wavefront's accesses in issue order
        if (lane < slots && w < W) out_row[w] = v;
        if (a.apply_out && g < n_seg) {
            // Logit masking (Section 3.3) of the segment's tokens, right here: 16-byte pieces, consecutive lanes on consecutive
            // pieces, the mask word from the lane that holds it.  Allowed logits are copied bit for bit, the others become -inf.
            uint8_t *dst = reinterpret_cast<uint8_t *>(a.apply_out) + l_at;
            auto mask_piece = [&](uint32_t p, u32x4 x) {     // all lanes call it together: the shuffle is for all of them
                const uint32_t t_in = p * tp;
                const uint32_t mb = (uint32_t)__shfl((int)v, (int)((t_in >> 5) & 63u)) >> (t_in & 31u);
                if (p < pieces) {
                    if (a.apply_dtype) {
#pragma unroll
                        for (int k = 0; k < 4; k++) {
                            uint32_t e = x[k];
                            if (!((mb >> (2 * k)) & 1u)) e = (e & 0xFFFF0000u) | 0xFF80u;
                            if (!((mb >> (2 * k + 1)) & 1u)) e = (e & 0x0000FFFFu) | 0xFF800000u;
                            x[k] = e;
                        }
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; k++) if (!((mb >> k) & 1u)) x[k] = 0xFF800000u;
                    }
                    __builtin_nontemporal_store(x, reinterpret_cast<u32x4 *>(dst) + p);
                }
            };
            mask_piece(lane, l_pre[0]);
            if (pieces > 64u) mask_piece(64u + lane, l_pre[1]);
            for (uint32_t p0 = 128; p0 < pieces; p0 += 256) {   // what was not requested ahead: four pieces per lane in flight
                u32x4 x[4];
#pragma unroll
                for (int u = 0; u < 4; u++) { const uint32_t p = p0 + (uint32_t)u * 64u + lane; x[u] = u32x4{0, 0, 0, 0}; if (p < pieces) x[u] = __builtin_nontemporal_load(l_src + p); }
#pragma unroll
                for (int u = 0; u < 4; u++) if (p0 + (uint32_t)u * 64u < pieces) mask_piece(p0 + (uint32_t)u * 64u + lane, x[u]);
            }
        }
        v = vn; c = cn;
        l_pre[0] = l_nxt[0]; l_pre[1] = l_nxt[1];
    }
    if (lane == 0 && steps) atomicAdd(&a.counters[3], steps);
    if (lane == 0 && undecided) atomicAdd(&block_undecided, undecided);   // LDS: the block's sum travels with its ticket
    }
    }
    // the call's status goes to the host from the block that finishes last (a failed look-up counts up to the end)
    __syncthreads();
    hand_over(a, blockIdx.x, gridDim.x, true, block_undecided, !a.handoff_in_store);
}

// Clear the store: every transition unknown, every header unpublished, the hash table empty; then the
// state of the empty prefix, whose items started in that very set.
__global__ __launch_bounds__(256) void store_clear_kernel(StoreView G, uint32_t ncls, const uint2 *root_items, uint32_t n_root) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    for (size_t k = i; k < (size_t)G.cap_states * ncls; k += stride) G.trans[k] = AT_NONE;
    for (size_t k = i; k < G.cap_states; k += stride) G.hdr[k] = k == STORE_ROOT ? make_uint2(0, n_root) : make_uint2(0, UNPUBLISHED);
    for (size_t k = i; k <= G.intern_mask; k += stride) G.intern[k] = 0;
    for (size_t k = i; k < n_root; k += stride) G.arena[k] = make_uint2(root_items[k].x, STORE_ROOT);
    if (i == 0) { G.ctl[0] = STORE_ROOT + 1; G.ctl[1] = n_root; G.ctl[2] = 0; G.ctl[3] = 0; }
}

// Bring rows whose state the store does not know (after the store was cleared, or after more bytes than
// a call carries) in from their host charts: every set of the packed chart becomes a state of its own,
// origins renamed from set indices to the new names.  One block per such row.
__global__ __launch_bounds__(256) void store_import_kernel(MaskArgs a, const uint32_t *import_rows, uint32_t n_import) {
    const StoreView &G = a.store;
    __shared__ uint32_t base[2];
    const uint32_t r = import_rows[blockIdx.x];
    const RowChart rc = a.rows[blockIdx.x];
    if (threadIdx.x == 0) { base[0] = atomicAdd(&G.ctl[0], rc.n_sets); base[1] = atomicAdd(&G.ctl[1], rc.n_items); }
    __syncthreads();
    const uint32_t id0 = base[0], at0 = base[1];
    if (id0 > G.cap_states - rc.n_sets || id0 + rc.n_sets > G.cap_states || at0 > G.cap_items - rc.n_items || rc.n_items > G.cap_items) {
        if (threadIdx.x == 0) { atomicAdd(&G.ctl[2], 1u); atomicAdd(&a.counters[2], 1u); a.store_import_root[r] = AT_FAIL; }
        return;
    }
    const uint32_t *so = a.set_off + rc.set_base;
    const uint2 *it = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
    for (uint32_t k = threadIdx.x; k < rc.n_items; k += 256) { const uint2 x = it[k]; G.arena[at0 + k] = make_uint2(x.x, id0 + x.y); }
    for (uint32_t k = threadIdx.x; k < rc.n_sets; k += 256) G.hdr[id0 + k] = make_uint2(at0 + so[k], so[k + 1] - so[k]);
    if (threadIdx.x == 0) a.store_import_root[r] = id0 + rc.n_sets - 1;
    (void)n_import;
}

}  // namespace

hipError_t prepare_store_kernels() {
    const int max_lds = STORE_LDS_MAX;
    hipError_t e;
#define SET_ATTR(k) if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k), hipFuncAttributeMaxDynamicSharedMemorySize, max_lds)) != hipSuccess) return e
    SET_ATTR(mask_store_kernel<0>); SET_ATTR(mask_store_kernel<1>); SET_ATTR(mask_store_kernel<2>);
#undef SET_ATTR
    return hipSuccess;
}

uint32_t store_lds_bytes(const DeviceTables &t, int mode, int scratch) {
    return table_bytes(t, mode) + 256 + LC_ENTRIES * 8 + 32 + STORE_WAVES * 64 * 4 +
           STORE_WAVES * ((uint32_t)scratch * 8 + aut_hash_places((uint32_t)scratch) * 4);
}

// Blocks of the kernel one compute unit holds at once (registers and the LDS the call asks for decide); asked of the runtime once
// per LDS size.
int store_blocks_per_cu(const DeviceTables &t, int mode, int scratch) {
    static thread_local uint32_t known_lds[3] = {0, 0, 0};
    static thread_local int known[3] = {0, 0, 0};
    const uint32_t lds = store_lds_bytes(t, mode, scratch);
    const int m = mode < 0 ? 0 : (mode > 2 ? 2 : mode);
    if (known[m] && known_lds[m] == lds) return known[m];
    int n = 0;
    hipError_t e;
    if (m == 0) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_store_kernel<0>, STORE_BLOCK, lds);
    else if (m == 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_store_kernel<1>, STORE_BLOCK, lds);
    else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_store_kernel<2>, STORE_BLOCK, lds);
    if (e != hipSuccess || n < 1) { (void)hipGetLastError(); n = 1; }
    known[m] = n; known_lds[m] = lds;
    return n;
}

hipError_t launch_mask_store(const MaskArgs &a, const StoreMiniRows &mini, hipStream_t s) {
    const uint32_t lds = store_lds_bytes(a.tab, a.mode, a.aut_scratch);
    dim3 grid(a.store_uniform_parts ? (uint32_t)a.store_uniform_parts * (uint32_t)a.batch : (uint32_t)a.store_first_block[a.batch]);
    if (a.mode == 0) hipLaunchKernelGGL(mask_store_kernel<0>, grid, dim3(STORE_BLOCK), lds, s, a, mini);
    else if (a.mode == 1) hipLaunchKernelGGL(mask_store_kernel<1>, grid, dim3(STORE_BLOCK), lds, s, a, mini);
    else hipLaunchKernelGGL(mask_store_kernel<2>, grid, dim3(STORE_BLOCK), lds, s, a, mini);
    return hipGetLastError();
}

hipError_t launch_store_clear(const StoreView &G, uint32_t ncls, const void *root_items, uint32_t n_root, hipStream_t s) {
    hipLaunchKernelGGL(store_clear_kernel, dim3(2048), dim3(256), 0, s, G, ncls, (const uint2 *)root_items, n_root);
    return hipGetLastError();
}

hipError_t launch_store_import(const MaskArgs &a, const uint32_t *import_rows, uint32_t n_import, hipStream_t s) {
    if (n_import == 0) return hipSuccess;
    hipLaunchKernelGGL(store_import_kernel, dim3(n_import), dim3(256), 0, s, a, import_rows, n_import);
    return hipGetLastError();
}

}  // namespace zf
