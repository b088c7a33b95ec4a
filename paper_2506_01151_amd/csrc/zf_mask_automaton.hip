// Mask kernel, default (zf_options.walk_mode = 0): mask_automaton_kernel.  What does not fit its LDS budgets goes to
// the fallback pass of the call's closing kernel (finish_kernel, zf_mask_walk.hip).
#include "zf_kernel_common.h"
#include "zf_aut_step.h"

namespace zf {
namespace {

//
// The Earley set reached after a byte is a function of the set it came from, of the sets that
// set's items point back to, and of the byte's equivalence class -- not of the token that is
// being checked.  So the sets met while checking one row's tokens are the states of a
// deterministic automaton over byte classes, and with a pruned chart (Section 4.2) it is tiny: a
// few states, a few dozen transitions, while thousands of tokens need a verdict (Section 4.1).
// A block builds the automaton of its row lazily in LDS: a transition is computed by one
// wavefront-cooperative Earley byte step (Scan + Complete, tabulated Predict: Section 3.2) the
// first time a string needs it and looked up from then on; sets are interned by content, so a
// terminal that loops in place is a self loop (the state-cache idea of Section 5.2 inside one
// mask).  Every lane then walks its own string through the transition table.
//
// An item of a state is (item word, origin reference); an origin reference is the index of a set
// of the row's chart, or AUT_REF | id of another state of this automaton.  State 0 is the row's
// current set and is read from the chart.
struct Aut {               // one block's automaton; every pointer leads into LDS
    uint32_t *trans;       // [states_cap][ncls] next state or AT_*
    uint2 *hdr;            // [states_cap] (first item in arena, item count); count 0xFFFFFFFF = not written yet
    uint32_t *hash;        // [states_cap] signature of the content (filter for the interning compare)
    uint2 *arena;          // [arena_cap] items of all states
    uint32_t *ctl;         // [0] states handed out, [1] arena items handed out, [2] next batch of strings, [3] number of batches,
                           // [4] help-queue places handed out, [5] help-queue places taken, [6] batches finished
    uint32_t *hq;          // [AUT_HELP_QUEUE] transitions that wait for a free wavefront: HQ_VALID | state << 8 | class
    const uint8_t *rep;    // [ncls] one byte of each class
    uint32_t states_cap, arena_cap, ncls;
};

static const uint32_t HQ_VALID = 0x80000000u;


template <class BaseT>
struct AutSets {           // resolves origin references
    const BaseT &B;
    const Aut &A;
    __device__ __forceinline__ void view(uint32_t ref, uint64_t &h, uint32_t &n) const {   // the handle is the address of the set's first item
        if (ref & AUT_REF) { const uint2 hd = A.hdr[ref & ~AUT_REF]; h = (uint64_t)(uintptr_t)(A.arena + hd.x); n = hd.y; }
        else { const uint32_t lo = B.so[ref]; h = (uint64_t)(uintptr_t)(B.it + lo); n = B.so[ref + 1] - lo; }
    }
    __device__ __forceinline__ uint2 item(uint64_t h, uint32_t i) const { return reinterpret_cast<const uint2 *>((uintptr_t)h)[i]; }
};

// The transition of state s on class cl: take the byte step, then find the state that holds the
// resulting set (sets are interned by content: the same items in the same order are the same
// state) or make a new one.  Returns a state id or AT_DEAD / AT_SINK / AT_FAIL.
template <bool WIDE, class BaseT>
__device__ __forceinline__ uint32_t aut_transition(const TV &T, const BaseT &B, const Aut &A, uint32_t *sc_w, uint32_t *sc_o, uint32_t *sc_h, uint32_t sc_cap,
                                                   uint32_t s, uint32_t byte, uint32_t cl, uint32_t lane) {
    const AutSets<BaseT> S{B, A};
    const uint32_t cur = s == 0 ? B.m - 1 : (AUT_REF | s);   // the source set; also what items predicted in it get as origin
    uint32_t nnew = 0, kept = 0;
    uint64_t src_p;
    uint32_t src_n;
    S.view(cur, src_p, src_n);
    int st = WIDE && src_n > (uint32_t)AUT_NARROW_SET_MAX ? AUT_WIDE : aut_step_narrow<WIDE>(T, S, sc_w, sc_o, sc_cap, cur, byte, cl, lane, nnew, kept);   // a wide source set rarely leaves a narrow one
    if (st == AUT_WIDE) st = WIDE ? aut_step_wide(T, S, sc_w, sc_o, sc_h, sc_cap, cur, byte, cl, lane, nnew, kept) : (int)AUT_OVER;
    if (st != AUT_OK) return AT_FAIL;
    if (nnew == 0) return AT_DEAD;
    if (kept == 0) return AT_SINK;
    // a cheap signature (first and last item) filters the candidates of the content compare
    const uint32_t h = (sc_w[0] * 0x9E3779B1u) ^ (sc_o[0] * 0x85EBCA77u) ^ (sc_w[kept - 1] * 0xC2B2AE3Du) ^ sc_o[kept - 1];
    uint32_t n_st = lds_load(&A.ctl[0]);
    n_st = n_st < A.states_cap ? n_st : A.states_cap;
    for (uint32_t j0 = 1; j0 < n_st; j0 += 64) {
        const uint32_t j = j0 + lane;
        bool cand = false;
        if (j < n_st) { const uint2 hj = A.hdr[j]; cand = hj.y == kept && A.hash[j] == h; }   // a state that is still being written has count 0xFFFFFFFF
        unsigned long long m = __ballot(cand);
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t id = j0 + (uint32_t)l;
            const uint2 hj = A.hdr[id];
            unsigned long long diff = 0;
            for (uint32_t i0 = 0; i0 < kept; i0 += 64) {
                bool ne = false;
                if (i0 + lane < kept) { const uint2 x = A.arena[hj.x + i0 + lane]; ne = x.x != sc_w[i0 + lane] || x.y != sc_o[i0 + lane]; }
                diff |= __ballot(ne);
            }
            if (!diff) return id;
        }
    }
    uint32_t id = 0, at = 0;
    if (lane == 0) { id = atomicAdd(&A.ctl[0], 1u); at = atomicAdd(&A.ctl[1], kept); }
    id = (uint32_t)__builtin_amdgcn_readfirstlane((int)id);
    at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
    if (id >= A.states_cap || at + kept > A.arena_cap) return AT_FAIL;
    for (uint32_t i0 = 0; i0 < kept; i0 += 64)
        if (i0 + lane < kept) A.arena[at + i0 + lane] = make_uint2(sc_w[i0 + lane], sc_o[i0 + lane]);
    aut_mark_dead<WIDE>(T, A.ncls, A.rep, [&](uint32_t i) { return sc_w[i]; }, kept, lane, [&](uint32_t c) { A.trans[id * A.ncls + c] = AT_DEAD; });
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // items before the hash, the hash before the header that makes the state visible
    if (lane == 0) A.hash[id] = h;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) A.hdr[id] = make_uint2(at, kept);
    return id;
}

// Compute the transition of state s on class cl (the caller owns it: its entry is AT_BUSY) and publish it.
template <bool WIDE, class BaseT>
__device__ __forceinline__ void aut_resolve(const TV &T, const BaseT &B, const Aut &A, uint32_t *sc_w, uint32_t *sc_o, uint32_t *sc_h, uint32_t sc_cap,
                                            uint32_t s, uint32_t cl, uint32_t lane) {
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");   // the states this step reads were published by other wavefronts
    const uint32_t r = aut_transition<WIDE>(T, B, A, sc_w, sc_o, sc_h, sc_cap, s, A.rep[cl], cl, lane);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // the new state before the transition that leads to it
    if (lane == 0) lds_store(&A.trans[s * A.ncls + cl], r);
}

// A wavefront whose strings miss several transitions at once computes one and leaves the others in
// the help queue; wavefronts that wait or have run out of strings take them from there.  Takes one
// request (s, cl) if there is one.  Uniform over the wavefront.
enum { AUT_HQ_EMPTY = 0, AUT_HQ_GOT = 1, AUT_HQ_AGAIN = 2 /* another wavefront was faster: look again */ };
__device__ __forceinline__ int aut_help_take(const Aut &A, uint32_t lane, uint32_t &s, uint32_t &cl) {
    uint32_t tail = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&A.ctl[4]));
    tail = tail < (uint32_t)AUT_HELP_QUEUE ? tail : (uint32_t)AUT_HELP_QUEUE;
    const uint32_t head = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&A.ctl[5]));
    if (head >= tail) return AUT_HQ_EMPTY;
    uint32_t got = 0;
    if (lane == 0) got = atomicCAS(&A.ctl[5], head, head + 1u) == head ? 1u : 0u;
    if (!__builtin_amdgcn_readfirstlane((int)got)) return AUT_HQ_AGAIN;
    uint32_t e = 0;
    for (int tries = 0; tries < AUT_SPIN_LIMIT; tries++) {    // the entry is written right after its place was handed out
        e = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&A.hq[head]));
        if (e & HQ_VALID) break;
        __builtin_amdgcn_s_sleep(1);
    }
    if (!(e & HQ_VALID)) return AUT_HQ_AGAIN;                // cannot happen: places below the end of the queue are always filled
    s = (e & ~HQ_VALID) >> 8;
    cl = e & 0xFFu;
    return AUT_HQ_GOT;
}

__host__ __device__ inline uint32_t aut_round16(uint32_t x) { return (x + 15u) & ~15u; }

// Grid (parts, rows).  A block takes slices of AUT_SUB_WORDS words of its row's rank-ordered bitmap in
// turn: it merges the token-mask cache rows of the row's current set (Section 4.3: strings a terminal
// swallows whole are valid at once), lists the strings that need the parser, and its wavefronts
// take the list in batches of 64 strings, one lane per string.  The verdicts of a slice are
// collected in LDS and stored once: no atomics on global memory and nothing to clear beforehand.
// MODE: which grammar tables are staged in LDS (0 all, 1 the small ones, 2 none).  WIDE: the build that
// holds the wide variant of the byte step and its hash table; the build without it is for charts whose
// sets are all small (the host knows: it packs them), where a set of more than 64 items fails over to the
// fallback pass.  Keeping the wide variant out of that build keeps the narrow path's registers and code small.
template <int MODE, bool WIDE>
__global__ __launch_bounds__(AUT_BLOCK) void mask_automaton_kernel(MaskArgs a) {
    extern __shared__ __align__(16) uint8_t smem[];
    const DeviceTables &D = a.tab;
    const uint32_t tid = threadIdx.x, row = blockIdx.y, wave = tid >> 6, lane = tid & 63;
    const uint32_t Wr = (uint32_t)D.Wr, n_strings = (uint32_t)D.n_strings;
    if (blockIdx.x >= (Wr + AUT_GROUP_WORDS - 1) / AUT_GROUP_WORDS) return;
    // Everything a block needs from global memory before it can start is requested at once (tables,
    // the row's chart, its token-mask-cache rows) and written to LDS afterwards: one memory latency.
    TV T;
    uint32_t off = table_view<MODE>(D, smem, T);
    const uint32_t n16 = off / 16;
    static_assert(AUT_TABLE_LOADS <= 7, "the staging below holds at most seven 16-byte pieces per thread");
    const uint4 *blob = reinterpret_cast<const uint4 *>(D.table_blob);
    uint4 tb0 = make_uint4(0, 0, 0, 0), tb1 = tb0, tb2 = tb0, tb3 = tb0, tb4 = tb0, tb5 = tb0, tb6 = tb0;   // named registers: an indexed array ends up in scratch memory
#define ZF_STAGE_LOAD(u) if (tid + (u) * AUT_BLOCK < n16) tb##u = blob[tid + (u) * AUT_BLOCK];
    ZF_STAGE_LOAD(0) ZF_STAGE_LOAD(1) ZF_STAGE_LOAD(2) ZF_STAGE_LOAD(3) ZF_STAGE_LOAD(4) ZF_STAGE_LOAD(5) ZF_STAGE_LOAD(6)
#undef ZF_STAGE_LOAD
    Aut A;
    A.ncls = (uint32_t)D.n_cls; A.states_cap = (uint32_t)a.aut_states; A.arena_cap = (uint32_t)a.aut_arena;
    const uint32_t sc_cap = (uint32_t)a.aut_scratch;
    A.trans = reinterpret_cast<uint32_t *>(smem + off); off += aut_round16(A.states_cap * A.ncls * 4);
    A.hdr = reinterpret_cast<uint2 *>(smem + off); off += aut_round16(A.states_cap * 8);
    A.hash = reinterpret_cast<uint32_t *>(smem + off); off += aut_round16(A.states_cap * 4);
    A.ctl = reinterpret_cast<uint32_t *>(smem + off); off += 32;
    A.hq = reinterpret_cast<uint32_t *>(smem + off); off += AUT_HELP_QUEUE * 4;
    const uint32_t base_sets_cap = (uint32_t)a.aut_base_sets, base_items_cap = (uint32_t)a.aut_base_items;
    uint32_t *l_so = reinterpret_cast<uint32_t *>(smem + off); off += aut_round16((base_sets_cap + 1) * 4);
    uint2 *l_it = reinterpret_cast<uint2 *>(smem + off); off += aut_round16(base_items_cap * 8);
    uint32_t *l_ent = reinterpret_cast<uint32_t *>(smem + off); off += AUT_ENT_LDS * 4;
    uint8_t *l_rep = smem + off; off += 256;
    A.rep = l_rep;
    uint32_t *vslice = reinterpret_cast<uint32_t *>(smem + off); off += AUT_SUB_WORDS * 4;
    uint32_t *cslice = reinterpret_cast<uint32_t *>(smem + off); off += AUT_SUB_WORDS * 4;
    uint8_t *pairs = smem + off; off += AUT_SUB_WORDS / 2;   // slots of the word pairs that hold undecided strings
    A.arena = reinterpret_cast<uint2 *>(smem + off); off += aut_round16(A.arena_cap * 8);
    uint32_t *sc_w = reinterpret_cast<uint32_t *>(smem + off) + (size_t)wave * (2 * sc_cap + (WIDE ? aut_hash_places(sc_cap) : 0u));   // the hash table belongs to the wide byte step
    uint32_t *sc_o = sc_w + sc_cap, *sc_h = sc_o + sc_cap;
    // the row's chart: its LDS copy when it is small, else global memory (generic pointers either way).  When every
    // row has the same room in the upload (strides), the pieces are requested before the row's header is known.
    uint32_t so_v = 0, ent_v = 0;
    uint2 it_v = make_uint2(0, 0);
    const bool strided = a.so_stride != 0;
    if (strided) {
        if (tid < a.so_stride && tid <= base_sets_cap) so_v = (a.set_off + (size_t)row * a.so_stride)[tid];
        if (tid < a.it_stride && tid < base_items_cap) it_v = (reinterpret_cast<const uint2 *>(a.items) + (size_t)row * a.it_stride)[tid];
        if (tid < a.ent_stride && tid < (uint32_t)AUT_ENT_LDS) ent_v = (a.entries + (size_t)row * a.ent_stride)[tid];
    }
    const RowChart rc = a.rows[row];
    const uint32_t *g_so = a.set_off + rc.set_base;
    const uint2 *g_it = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
    const uint32_t *g_ent = a.entries + rc.ent_base;
    const bool base_fits = rc.n_sets <= base_sets_cap && rc.n_items <= base_items_cap;
    const bool ent_fits = rc.n_ent <= AUT_ENT_LDS;
    if (!WIDE && !(base_fits && ent_fits)) {                               // never launched like this; if it were, the call must fail loudly
        if (tid == 0) atomicAdd(&a.counters[2], 1u);
        return;
    }
    if (!strided) {
        if (base_fits && tid <= rc.n_sets) so_v = g_so[tid];
        if (base_fits && tid < rc.n_items) it_v = g_it[tid];
        if (ent_fits && tid < rc.n_ent) ent_v = g_ent[tid];
    }
    const uint8_t rep_v = tid < A.ncls ? D.cls_rep[tid] : (uint8_t)0;
#define ZF_STAGE_STORE(u) if (tid + (u) * AUT_BLOCK < n16) reinterpret_cast<uint4 *>(smem)[tid + (u) * AUT_BLOCK] = tb##u;
    ZF_STAGE_STORE(0) ZF_STAGE_STORE(1) ZF_STAGE_STORE(2) ZF_STAGE_STORE(3) ZF_STAGE_STORE(4) ZF_STAGE_STORE(5) ZF_STAGE_STORE(6)
#undef ZF_STAGE_STORE
    if (base_fits && tid <= rc.n_sets) l_so[tid] = so_v;
    if (base_fits && tid < rc.n_items) l_it[tid] = it_v;
    if (ent_fits && tid < rc.n_ent) l_ent[tid] = ent_v;
    if (tid < 256) l_rep[tid] = rep_v;
    if (base_fits) {                                         // a long chart: what the first load per thread did not cover
        for (uint32_t k = tid + AUT_BLOCK; k <= rc.n_sets; k += AUT_BLOCK) l_so[k] = g_so[k];
        for (uint32_t k = tid + AUT_BLOCK; k < rc.n_items; k += AUT_BLOCK) l_it[k] = g_it[k];
    }
    for (uint32_t k = tid; k < A.states_cap * A.ncls; k += AUT_BLOCK) A.trans[k] = AT_NONE;
    for (uint32_t k = tid; k < A.states_cap; k += AUT_BLOCK) A.hdr[k] = make_uint2(0, 0xFFFFFFFFu);
    for (uint32_t k = tid; k < (uint32_t)AUT_HELP_QUEUE; k += AUT_BLOCK) A.hq[k] = 0;
    if (tid == 0) { A.ctl[0] = 1; A.ctl[1] = 0; A.ctl[4] = 0; A.ctl[5] = 0; }
    const uint32_t *b_ent = (!WIDE || ent_fits) ? l_ent : g_ent;   // without the wide step: sets of at most AUT_NARROW_SET_MAX items, so at most that many cache rows
    const uint32_t *b_so = (!WIDE || base_fits) ? l_so : g_so;   // the build without the wide step is launched only when every chart fits:
    const uint2 *b_it = (!WIDE || base_fits) ? l_it : g_it;      // its chart pointers are LDS addresses at compile time
    uint32_t steps = 0;
    const uint32_t cr = (uint32_t)D.chunk_ranks;
    // The words of the row's bitmap are dealt to the blocks in groups of AUT_GROUP_WORDS, round robin:
    // undecided strings come in runs of thousands of neighbouring ranks (everything that begins
    // with a quote, say), and every block should get its share of each run.
    const uint32_t n_groups = (Wr + AUT_GROUP_WORDS - 1) / AUT_GROUP_WORDS, groups_per_pass = AUT_SUB_WORDS / AUT_GROUP_WORDS;
    for (uint32_t j0 = 0; blockIdx.x + j0 * gridDim.x < n_groups; j0 += groups_per_pass) {
        auto word_of = [&](uint32_t t) -> uint32_t {         // the bitmap word slot t of this pass stands for, or Wr and more if none
            const uint32_t grp = blockIdx.x + (j0 + t / AUT_GROUP_WORDS) * gridDim.x;
            return grp < n_groups ? grp * AUT_GROUP_WORDS + t % AUT_GROUP_WORDS : 0xFFFFFF00u;
        };
        if (tid == 0) { A.ctl[2] = 0; A.ctl[3] = 0; A.ctl[6] = 0; }
        if (tid < AUT_SUB_WORDS) { vslice[tid] = 0; cslice[tid] = rc.n_ent == 0 ? 0xFFFFFFFFu : 0u; }
        __syncthreads();                                     // also: tables, chart and automaton set-up are in place
        // ---- merge the token-mask cache rows (all threads: word slot tid % SUB, cache rows tid / SUB, + 4, ...) ----
        {
            const uint32_t t = tid % AUT_SUB_WORDS, w = word_of(t);
            uint32_t v = 0, c = 0;
            if (w < Wr)
                for (uint32_t k = tid / AUT_SUB_WORDS; k < rc.n_ent; k += AUT_BLOCK / AUT_SUB_WORDS) {
                    const size_t r = (size_t)b_ent[k] * Wr + w;
                    v |= D.ci_valid[r]; c |= D.ci_cd[r];
                }
            if (v) atomicOr(&vslice[t], v);
            if (c) atomicOr(&cslice[t], c);
        }
        __syncthreads();
        // ---- the undecided strings, and the word pairs (64 ranks) that hold any: one wavefront, one ballot ----
        if (tid < AUT_SUB_WORDS / 2) {                       // the first wavefront
            uint32_t want[2];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t w = word_of(2 * tid + h), r0 = w * 32u;
                want[h] = cslice[2 * tid + h] & ~vslice[2 * tid + h];
                if (w >= Wr || r0 >= n_strings) want[h] = 0;                 // strings beyond the last one do not exist
                else if (n_strings - r0 < 32u) want[h] &= (1u << (n_strings - r0)) - 1u;
                cslice[2 * tid + h] = want[h];
            }
            const unsigned long long nz = __ballot((want[0] | want[1]) != 0);
            if (want[0] | want[1]) pairs[__popcll(nz & ((1ull << lane) - 1ull))] = (uint8_t)tid;
            uint32_t cnt = (uint32_t)(__popc(want[0]) + __popc(want[1]));
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d);
            if (lane == 0) { A.ctl[3] = (uint32_t)__popcll(nz); if (cnt) atomicAdd(&a.counters[1], cnt); }
        }
        const BaseG B{b_so, b_it, rc.n_sets, b_so[rc.n_sets - 1], rc.n_items};
        if (j0 == 0 && wave == AUT_WAVES - 1)                // meanwhile the last wavefront settles the dead transitions of the row's current set
            aut_mark_dead<WIDE>(T, A.ncls, A.rep, [&](uint32_t i) { return B.it[B.last_lo + i].x; }, B.last_hi - B.last_lo, lane, [&](uint32_t c) { A.trans[c] = AT_DEAD; });
        __syncthreads();
        const uint32_t n_pairs = A.ctl[3];
        // ---- one lane per string through the automaton, 64 neighbouring ranks at a time.  A wavefront that finds
        // no batch left stays in the same loop (the byte step is expanded in one place only) and serves the
        // help queue until every batch of the block is finished ----
        for (;;) {
            uint32_t b = 0;
            if (lane == 0) b = atomicAdd(&A.ctl[2], 1u);
            b = (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
            const bool batch = b < n_pairs;
            const uint32_t pair = batch ? pairs[b] : 0u;
            const uint32_t rank = word_of(2 * pair) * 32u + lane;            // a pair lies inside one group: consecutive ranks
            bool live = batch && ((cslice[2 * pair + (lane >> 5)] >> (lane & 31u)) & 1u);
            uint32_t soff = 0, len = 0;
            Str16 c16{{0, 0, 0, 0}};
            if (live) { soff = D.str_off[rank]; len = D.str_off[rank + 1] - soff; c16 = D.str16[rank]; }
            live = live && len > 0;
            uint32_t s = 0, pos = 0, c = 0, spins = 0, t = AT_BUSY;
            bool ok = false, fail = false;
            for (;;) {
                bool have = false, progress = false;         // a transition to compute here; something this wavefront waits for has moved
                uint32_t rs = 0, rc = 0;
                if (batch) {
                    while (live) {                           // every lane follows its own string as far as the table goes
                        if (pos < 16u) {
                            const uint32_t q = pos >> 2;
                            const uint32_t word = q == 0 ? c16.w[0] : (q == 1 ? c16.w[1] : (q == 2 ? c16.w[2] : c16.w[3]));
                            c = (word >> ((pos & 3u) * 8u)) & 0xFFu;
                        } else c = D.str_cls[soff + pos];
                        t = lds_load(&A.trans[s * A.ncls + c]);
                        if (t < AT_FAIL) { s = t; pos++; if (pos == len) { ok = true; live = false; } }
                        else if (t == AT_DEAD) live = false;
                        else if (t == AT_SINK) { ok = pos + 1 == len; live = false; }
                        else if (t == AT_FAIL) { fail = true; live = false; }
                        else break;                          // not there yet
                    }
                    if (!__ballot(live)) break;
                    // Every waiting lane tries to claim the transition it misses, all at once (among lanes that miss
                    // the same one, one wins).  The first claim is computed here, the others are left in the
                    // help queue for wavefronts that have nothing to do.
                    uint32_t old = AT_BUSY;                  // lanes that found the transition being computed need not ask again
                    if (live && t == AT_NONE) old = atomicCAS(&A.trans[s * A.ncls + c], (uint32_t)AT_NONE, (uint32_t)AT_BUSY);
                    const unsigned long long won = __ballot(live && old == AT_NONE);
                    progress = won != 0 || __ballot(live && old != AT_NONE && old != AT_BUSY) != 0;   // claimed, or published meanwhile
                    if (won) {
                        const int first = __ffsll((long long)won) - 1;
                        const unsigned long long rest = won & ~(1ull << first);
                        if (rest) {
                            uint32_t at = 0;
                            if (lane == 0) at = atomicAdd(&A.ctl[4], (uint32_t)__popcll(rest));
                            at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
                            if ((rest >> lane) & 1ull) {
                                const uint32_t k = at + (uint32_t)__popcll(rest & ((1ull << lane) - 1ull));
                                if (k < (uint32_t)AUT_HELP_QUEUE) lds_store(&A.hq[k], HQ_VALID | (s << 8) | c);
                                else lds_store(&A.trans[s * A.ncls + c], (uint32_t)AT_NONE);   // no room in the queue: the claim is given back
                            }
                        }
                        have = true;
                        rs = (uint32_t)__builtin_amdgcn_readlane((int)s, first);
                        rc = (uint32_t)__builtin_amdgcn_readlane((int)c, first);
                    }
                }
                int q = AUT_HQ_EMPTY;
                if (!have && !progress) {                    // nothing of its own to compute: lend a hand
                    q = aut_help_take(A, lane, rs, rc);
                    have = q == AUT_HQ_GOT;
                }
                if (have) {
                    aut_resolve<WIDE>(T, B, A, sc_w, sc_o, sc_h, sc_cap, rs, rc, lane);
                    steps++;
                    if (!batch) spins = 0;
                } else if (!progress && q == AUT_HQ_EMPTY) { // everything this wavefront waits for is being computed by others
                    if (!batch && (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&A.ctl[6])) >= n_pairs) break;   // all batches finished, nothing queued
                    __builtin_amdgcn_s_sleep(4);
                    if (++spins > (uint32_t)AUT_SPIN_LIMIT) {   // bounded wait: hand the strings to the fallback
                        if (!batch) break;
                        fail = fail || live;
                        live = false;
                    }
                }
            }
            if (!batch) break;
            if (lane == 0) atomicAdd(&A.ctl[6], 1u);
            const unsigned long long okb = __ballot(ok);     // this wavefront is the only one that touches the pair's two words
            if (lane == 0 && okb) { vslice[2 * pair] |= (uint32_t)okb; vslice[2 * pair + 1] |= (uint32_t)(okb >> 32); }
            // strings this block could not decide: one fallback entry per trie chunk
            unsigned long long fm = __ballot(fail);
            const uint32_t my_chunk = rank / cr;
            while (fm) {
                const int l = __ffsll((long long)fm) - 1;
                const uint32_t ch = __builtin_amdgcn_readlane(my_chunk, l);
                const bool same = fail && my_chunk == ch;
                fm &= ~__ballot(same);
                uint32_t bits = same ? 1u << (rank % cr) : 0u;
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) bits |= __shfl_xor(bits, d);
                if (lane == 0) {
                    const uint32_t slot = atomicAdd(&a.counters[0], 1u);
                    if (slot < a.overflow_cap) a.overflow_list[slot] = make_uint4(row, ch, bits, 0);
                }
            }
        }
        __syncthreads();
        if (tid < AUT_SUB_WORDS) { const uint32_t w = word_of(tid); if (w < Wr) a.rank_mask[(size_t)row * Wr + w] = vslice[tid]; }
    }
    if (lane == 0 && steps) atomicAdd(&a.counters[3], steps);
}

}  // namespace

hipError_t prepare_automaton_kernels() {
    const int max_lds = 160 * 1024;
    hipError_t e;
#define SET_ATTR(k) if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k), hipFuncAttributeMaxDynamicSharedMemorySize, max_lds)) != hipSuccess) return e
    SET_ATTR((mask_automaton_kernel<0, false>)); SET_ATTR((mask_automaton_kernel<1, false>)); SET_ATTR((mask_automaton_kernel<2, false>));
    SET_ATTR((mask_automaton_kernel<0, true>)); SET_ATTR((mask_automaton_kernel<1, true>)); SET_ATTR((mask_automaton_kernel<2, true>));
#undef SET_ATTR
    return hipSuccess;
}

uint32_t automaton_lds_bytes(const DeviceTables &t, int mode, int states, int arena, int scratch, int base_sets, int base_items, bool wide) {
    return table_bytes(t, mode) + aut_round16((uint32_t)states * (uint32_t)t.n_cls * 4) + aut_round16((uint32_t)states * 8) + aut_round16((uint32_t)states * 4) + 32 + AUT_HELP_QUEUE * 4 +
           aut_round16(((uint32_t)base_sets + 1) * 4) + aut_round16((uint32_t)base_items * 8) + AUT_ENT_LDS * 4 + 256 + 2 * AUT_SUB_WORDS * 4 + AUT_SUB_WORDS / 2 + aut_round16((uint32_t)arena * 8) +
           AUT_WAVES * ((uint32_t)scratch * 8 + (wide ? aut_hash_places((uint32_t)scratch) * 4 : 0u));
}
hipError_t launch_mask_automaton(const MaskArgs &a, hipStream_t s) {
    const uint32_t lds = automaton_lds_bytes(a.tab, a.mode, a.aut_states, a.aut_arena, a.aut_scratch, a.aut_base_sets, a.aut_base_items, a.aut_wide != 0);
    dim3 grid(a.aut_parts, a.batch);
    // two builds of the kernel: without the wide variant of the byte step (its code costs the narrow path ~10 %
    // in registers and instruction fetch) for charts whose sets are all small, and with it
    if (a.aut_wide) {
        if (a.mode == 0) hipLaunchKernelGGL((mask_automaton_kernel<0, true>), grid, dim3(AUT_BLOCK), lds, s, a);
        else if (a.mode == 1) hipLaunchKernelGGL((mask_automaton_kernel<1, true>), grid, dim3(AUT_BLOCK), lds, s, a);
        else hipLaunchKernelGGL((mask_automaton_kernel<2, true>), grid, dim3(AUT_BLOCK), lds, s, a);
    } else {
        if (a.mode == 0) hipLaunchKernelGGL((mask_automaton_kernel<0, false>), grid, dim3(AUT_BLOCK), lds, s, a);
        else if (a.mode == 1) hipLaunchKernelGGL((mask_automaton_kernel<1, false>), grid, dim3(AUT_BLOCK), lds, s, a);
        else hipLaunchKernelGGL((mask_automaton_kernel<2, false>), grid, dim3(AUT_BLOCK), lds, s, a);
    }
    return hipGetLastError();
}
}  // namespace zf
