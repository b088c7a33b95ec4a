// HIP kernels for gfx950: the vocabulary-mask kernels (mask automaton, trie walk, exact fallback),
// the rank-order -> token-order bit permutation, and the logit-masking kernel.
//
// Mask path.  The distinct vocabulary strings are numbered in sorted order (their rank); verdicts
// are first produced in rank order.  The context-independent token-mask cache (Section 4.3) settles
// most strings from the terminals of the row's current Earley set alone; the strings it leaves
// undecided need the parser.  Two kernels can do that part (zf_options.walk_mode), both exact:
//   mask_automaton_kernel (default): the Earley sets met while checking one row's strings are the
//      states of a small deterministic automaton over byte classes.  A block merges the cache rows
//      of a slice of its row's bitmap, builds the automaton lazily in LDS (one wavefront-cooperative
//      Earley byte step per missing transition: Scan + Complete with tabulated Predict, Section 3.2)
//      and walks every undecided string through the transition table, one lane per string.
//   cache_merge_kernel + mask_walk_kernel: the vocabulary trie is stored in preorder, so a
//      depth-first walk is a linear scan in which a dead subtree is left through the node's skip
//      pointer and a shared prefix is scanned once.  A chunk is the node range of `chunk_ranks`
//      consecutive strings; the merge kernel queues the chunks that hold undecided strings, and a
//      persistent grid of wavefronts walks them, one Earley byte step per live trie node, on an item
//      list in LDS that holds one set per trie depth of the current path.  The step is
//      wavefront-cooperative with uniform control flow (wave_step): items of a set are spread over
//      the lanes, the set under construction is held in registers, duplicate tests are ballots.
//      (Giving every lane its own chunk was measured first: the nests of short data-dependent loops
//      of an Earley step then cost ~12,000 cycles per step per wavefront because every loop level
//      runs for its longest trip count over the 64 lanes.)  Grammar tables are staged in LDS once
//      per block.
//   mask_fallback_kernel: whatever did not fit the LDS budgets of either kernel repeats the trie
//      walk, one wavefront per chunk, with the item list in a global-memory arena.
#include <hip/hip_runtime.h>
#include "zf_launch.h"

namespace zf {
namespace {

// Table view used by the device code; the pointers lead into LDS or global memory.
struct TV {
    const uint32_t *advpq;
    const uint8_t *cls;
    const uint32_t *qinfo;
    const uint32_t *scan_off;
    const uint32_t *comp_off;
    const uint32_t *delta;
    const uint2 *scan_list;
    const uint32_t *comp_list;
    uint32_t N, ncls, end_base;
};

__device__ __forceinline__ void copy16(void *dst, const void *src, uint32_t bytes, uint32_t tid, uint32_t nthreads) {
    const uint4 *s = reinterpret_cast<const uint4 *>(src);
    uint4 *d = reinterpret_cast<uint4 *>(dst);
    for (uint32_t i = tid; i < bytes / 16; i += nthreads) d[i] = s[i];
}

// Stage the tables the MODE asks for into LDS at smem and build the view.  Returns the bytes used.
// The caller must put a barrier between this and the first use.
template <int MODE>
__device__ __forceinline__ uint32_t stage_tables(const DeviceTables &D, uint8_t *smem, TV &tv, uint32_t tid, uint32_t nthreads) {
    tv.N = D.N; tv.ncls = D.n_cls; tv.end_base = D.end_base;
    uint32_t off = 0;
    if (MODE <= 1) {
        const void *src[5] = {D.advpq, D.cls, D.qinfo, D.scan_off, D.comp_off};
        uint32_t at[5];
#pragma unroll
        for (int k = 0; k < 5; k++) { at[k] = off; copy16(smem + off, src[k], D.small_bytes[k], tid, nthreads); off += D.small_bytes[k]; }
        tv.advpq = reinterpret_cast<const uint32_t *>(smem + at[0]);
        tv.cls = smem + at[1];
        tv.qinfo = reinterpret_cast<const uint32_t *>(smem + at[2]);
        tv.scan_off = reinterpret_cast<const uint32_t *>(smem + at[3]);
        tv.comp_off = reinterpret_cast<const uint32_t *>(smem + at[4]);
    } else {
        tv.advpq = D.advpq; tv.cls = D.cls; tv.qinfo = D.qinfo; tv.scan_off = D.scan_off; tv.comp_off = D.comp_off;
    }
    if (MODE == 0) {
        const void *src[3] = {D.delta, D.scan_list, D.comp_list};
        uint32_t at[3];
#pragma unroll
        for (int k = 0; k < 3; k++) { at[k] = off; copy16(smem + off, src[k], D.big_bytes[k], tid, nthreads); off += D.big_bytes[k]; }
        tv.delta = reinterpret_cast<const uint32_t *>(smem + at[0]);
        tv.scan_list = reinterpret_cast<const uint2 *>(smem + at[1]);
        tv.comp_list = reinterpret_cast<const uint32_t *>(smem + at[2]);
    } else {
        tv.delta = D.delta; tv.scan_list = reinterpret_cast<const uint2 *>(D.scan_list); tv.comp_list = D.comp_list;
    }
    return off;
}

// The same view without the copy: the tables of the MODE are expected at the start of smem in the
// order of DeviceTables::table_blob (the caller copies that prefix).  Returns the bytes they take.
template <int MODE>
__device__ __forceinline__ uint32_t table_view(const DeviceTables &D, uint8_t *smem, TV &tv) {
    tv.N = D.N; tv.ncls = D.n_cls; tv.end_base = D.end_base;
    tv.advpq = D.advpq; tv.cls = D.cls; tv.qinfo = D.qinfo; tv.scan_off = D.scan_off; tv.comp_off = D.comp_off;
    tv.delta = D.delta; tv.scan_list = reinterpret_cast<const uint2 *>(D.scan_list); tv.comp_list = D.comp_list;
    uint32_t off = 0;
    if (MODE <= 1) {
        tv.advpq = reinterpret_cast<const uint32_t *>(smem + off); off += D.small_bytes[0];
        tv.cls = smem + off; off += D.small_bytes[1];
        tv.qinfo = reinterpret_cast<const uint32_t *>(smem + off); off += D.small_bytes[2];
        tv.scan_off = reinterpret_cast<const uint32_t *>(smem + off); off += D.small_bytes[3];
        tv.comp_off = reinterpret_cast<const uint32_t *>(smem + off); off += D.small_bytes[4];
    }
    if (MODE == 0) {
        tv.delta = reinterpret_cast<const uint32_t *>(smem + off); off += D.big_bytes[0];
        tv.scan_list = reinterpret_cast<const uint2 *>(smem + off); off += D.big_bytes[1];
        tv.comp_list = reinterpret_cast<const uint32_t *>(smem + off); off += D.big_bytes[2];
    }
    return off;
}

// ---- item-list storage policies ---------------------------------------------------------
// An item is (w, o): w = item word (see IW_* in zf_device.h), o = origin set.
struct WaveLdsStore {          // walk kernel: the wavefront's list in LDS; set starts in a register (lane d holds the start of depth d)
    uint32_t *pq;
    uint32_t *org;
    uint32_t ss_reg;
    uint32_t lane;
    uint32_t cap;
    static constexpr int max_depth = WALK_DEPTH_MAX;
    __device__ __forceinline__ void get(uint32_t i, uint32_t &p, uint32_t &o) const { p = pq[i]; o = org[i]; }
    __device__ __forceinline__ void put(uint32_t i, uint32_t p, uint32_t o) { pq[i] = p; org[i] = o; }
    __device__ __forceinline__ uint32_t start(int d) const { return (uint32_t)__builtin_amdgcn_readlane((int)ss_reg, __builtin_amdgcn_readfirstlane(d)); }
    __device__ __forceinline__ void set_start(int d, uint32_t v) { if ((int)lane == d) ss_reg = v; }
};
struct GlobalStore {           // fallback: the wavefront's list in a global-memory arena
    uint2 *items;
    uint32_t *ss;
    uint32_t cap;
    static constexpr int max_depth = FB_DEPTH_MAX;
    __device__ __forceinline__ void get(uint32_t i, uint32_t &p, uint32_t &o) const { const uint2 x = items[i]; p = x.x; o = x.y; }
    __device__ __forceinline__ void put(uint32_t i, uint32_t p, uint32_t o) { items[i] = make_uint2(p, o); }
    __device__ __forceinline__ uint32_t start(int d) const { return ss[d]; }
    __device__ __forceinline__ void set_start(int d, uint32_t v) { ss[d] = v; }
};

// One DFA step: returns next state | flags of the next state << 16, or DFA_DEAD in the low half.
__device__ __forceinline__ uint32_t dfa_next(const TV &T, uint32_t q, uint32_t byte, uint32_t cl) {
    const uint32_t info = T.qinfo[q];
    if (info & QF_LITERAL) return (((info >> 8) & 0xFFu) == byte && (info & QF_CONT)) ? ((q + 1) | (info & 0xFFFF0000u)) : (uint32_t)DFA_DEAD;
    return T.delta[(info >> 16) * T.ncls + cl];
}

enum { STEP_ALIVE = 1, STEP_KERNEL = 2, STEP_OVERFLOW = 4, STEP_WIDE = 8 /* a set wider than 64 items: redo with wave_step_big */ };

template <class SoPtr, class ItPtr>
struct Base {                  // the row's uploaded chart (LDS copy or global)
    SoPtr so;                  // set offsets, so[k] .. so[k+1]
    ItPtr it;                  // items: x = item word, y = origin
    uint32_t m;                // number of sets; set m-1 is the current one
    uint32_t last_lo, last_hi; // so[m-1], so[m]
};
typedef Base<const uint32_t *, const uint2 *> BaseG;

// One Earley byte step at trie depth d (1-based) is done by a whole wavefront with uniform control
// flow.  The source set is the row's current set for d == 1, else the wavefront's set of depth
// d-1.  On entry cnt == st.start(d); on exit the new set is stored at [cnt_in, cnt_out).
// All 64 lanes call it with identical arguments.  Lane i loads source item i, the DFA transitions of all items run in
// parallel, the set under construction lives in registers (lane j holds new item j) so that the
// duplicate test is one compare + ballot, and Complete loads S[origin] 64 items at a time.  Sets
// of more than 64 items are reported as overflow (the fallback handles them).
template <class BaseT>
__device__ __forceinline__ int wave_step(const TV &T, const BaseT &B, WaveLdsStore &st, int d, uint32_t byte, uint32_t cl, uint32_t &cnt, uint32_t lane) {
    const uint32_t nb = cnt;
    const uint32_t cur = B.m - 1 + (uint32_t)(d - 1);
    const bool from_base = d == 1;
    const uint32_t sb = from_base ? B.last_lo : st.start(d - 1);
    const uint32_t ns = (from_base ? B.last_hi : nb) - sb;
    if (ns > 64) return STEP_WIDE;
    uint32_t sw = IW_END, so = 0;                        // lanes beyond the set hold an inert item
    if (lane < ns) { if (from_base) { const uint2 x = B.it[sb + lane]; sw = x.x; so = x.y; } else st.get(sb + lane, sw, so); }
    uint32_t nw = 0xFFFFFFFFu, no = 0, nnew = 0;         // the set under construction, one item per lane (no item word is all ones)
    bool saw_end = false;
    bool failed = false;                                 // sticky: an item found no room (64 lanes, or the item budget)
    const uint32_t room = st.cap - nb < 64u ? st.cap - nb : 64u;   // nb <= cap always
    // No branch in here: an item that does not fit leaves `failed` set and the set as it is; the
    // step runs on (every loop below is bounded by the tables and by 64 items) and reports at its end.
    auto insert = [&](uint32_t w, uint32_t o) {          // uniform arguments
        const bool fresh = __ballot(nw == w && no == o) == 0;
        const bool add = fresh && nnew < room;
        failed |= fresh && !add;
        const bool mine = add && lane == nnew;
        nw = mine ? w : nw;
        no = mine ? o : no;
        nnew += add ? 1u : 0u;
    };
    auto advance = [&](uint32_t p, uint32_t o) {         // dot arrives at p: skip nullable nonterminals, canonical END item
        for (;;) {
            const uint32_t w = T.advpq[p];
            insert(w, o);
            if (w & IW_END) { saw_end = true; return; }
            if ((w & IW_TERM) || !(w & IW_NT_NULLABLE)) return;
            p++;
        }
    };
    // Scan, terminal items: all DFA steps at once, then the survivors one after the other
    uint32_t nx = DFA_DEAD, aw = 0;
    if (sw & IW_TERM) {
        aw = T.advpq[(sw & IW_POS_MASK) + 1];            // the item behind the terminal, fetched alongside the DFA step in case the terminal ends here
        nx = dfa_next(T, sw >> 16, byte, cl);
    }
    unsigned long long m = __ballot((nx & 0xFFFFu) != DFA_DEAD);
    while (m) {
        const int l = __ffsll((long long)m) - 1;
        m &= m - 1;
        const uint32_t lw = __builtin_amdgcn_readlane(sw, l), lo = __builtin_amdgcn_readlane(so, l), lnx = __builtin_amdgcn_readlane(nx, l);
        if ((lnx >> 16) & QF_CONT) insert((lw & 0xFFFFu) | (lnx << 16), lo);   // no longest match: keep matching ...
        if ((lnx >> 16) & QF_ACCEPT) {                                                                                        // ... and also finish here
            const uint32_t law = __builtin_amdgcn_readlane(aw, l);
            insert(law, lo);
            if (law & IW_END) saw_end = true;
            else if (!(law & IW_TERM) && (law & IW_NT_NULLABLE)) advance((lw & IW_POS_MASK) + 2, lo);
        }
    }
    // Scan, items that wait for a nonterminal Y: the tabulated first steps of every terminal that can begin Y
    uint32_t sk0 = 0, sk1 = 0;                           // every lane looks up the list of its own nonterminal
    if (!(sw & (IW_TERM | IW_END))) {
        const uint32_t Y = (sw >> IW_NT_SHIFT) & IW_NT_MASK;
        sk0 = T.scan_off[Y * T.ncls + cl]; sk1 = T.scan_off[Y * T.ncls + cl + 1];
    }
    m = __ballot(sk1 > sk0);
    while (m) {
        const int l = __ffsll((long long)m) - 1;
        m &= m - 1;
        const uint32_t k0 = __builtin_amdgcn_readlane(sk0, l), k1 = __builtin_amdgcn_readlane(sk1, l);
        for (uint32_t e0 = k0; e0 < k1; e0 += 64) {
            uint2 ef = make_uint2(0, 0);
            if (e0 + lane < k1) ef = T.scan_list[e0 + lane];
            const uint32_t n_e = k1 - e0 < 64 ? k1 - e0 : 64;
            for (uint32_t t = 0; t < n_e; t++) {
                const uint32_t ent = __builtin_amdgcn_readlane(ef.x, t), f = __builtin_amdgcn_readlane(ef.y, t);
                if (f & QF_CONT) insert(ent, cur);
                if (f & QF_ACCEPT) advance((ent & IW_POS_MASK) + 1, cur);
            }
        }
    }
    if (saw_end) {
        // Complete: new items are visited in order; completing may append more
        unsigned long long visited = 0;
        for (;;) {
            const unsigned long long todo = __ballot(lane < nnew && (nw & IW_END)) & ~visited;
            if (!todo) break;
            const int i = __ffsll((long long)todo) - 1;
            visited |= 1ull << i;
            const uint32_t w = __builtin_amdgcn_readlane(nw, i);
            const uint32_t X = (w & IW_POS_MASK) - T.end_base;
            if (X == T.N - 1) continue;                 // the start rule is complete: the prefix is a sentence
            const uint32_t o = __builtin_amdgcn_readlane(no, i);
            const bool in_base = o < B.m;
            uint32_t jb, je;
            if (in_base) { jb = B.so[o]; je = B.so[o + 1]; }
            else { const int dj = (int)(o - (B.m - 1)); jb = st.start(dj); je = st.start(dj + 1); }
            for (uint32_t j0 = jb; j0 < je; j0 += 64) {
                uint32_t yw = IW_END, yo = 0;
                if (j0 + lane < je) { if (in_base) { const uint2 y = B.it[j0 + lane]; yw = y.x; yo = y.y; } else st.get(j0 + lane, yw, yo); }
                const bool nt = !(yw & (IW_TERM | IW_END));
                const uint32_t Y = (yw >> IW_NT_SHIFT) & IW_NT_MASK;
                uint32_t c0 = 0, c1 = 0, cw0 = 0;
                if (nt) { c0 = T.comp_off[Y * T.N + X]; c1 = T.comp_off[Y * T.N + X + 1]; }
                if (c1 > c0) cw0 = T.comp_list[c0];     // every lane fetches the first entry of its own list
                unsigned long long mm = __ballot(nt && c1 > c0);
                while (mm) {
                    const int l = __ffsll((long long)mm) - 1;
                    mm &= mm - 1;
                    const uint32_t lc0 = __builtin_amdgcn_readlane(c0, l), lc1 = __builtin_amdgcn_readlane(c1, l);
                    for (uint32_t e = lc0; e < lc1; e++) {
                        const uint32_t cw = e == lc0 ? (uint32_t)__builtin_amdgcn_readlane(cw0, l) : T.comp_list[e];
                        if (cw != 0xFFFFFFFFu) insert(cw, o);
                        else advance((__builtin_amdgcn_readlane(yw, l) & IW_POS_MASK) + 1, __builtin_amdgcn_readlane(yo, l));   // Y itself is complete: the waiting item moves on
                    }
                }
            }
        }
    }
    if (failed) return nnew >= 64u ? STEP_WIDE : STEP_OVERFLOW;   // all lanes taken: the strip-wise step may still fit; else the budget is used up
    // completed items are needed only while their own set is processed: store the others
    const bool keep = lane < nnew && !(nw & IW_END);
    const unsigned long long kb = __ballot(keep);
    if (keep) st.put(nb + __popcll(kb & ((1ull << lane) - 1ull)), nw, no);
    cnt = nb + (uint32_t)__popcll(kb);
    st.set_start(d + 1, cnt);
    return (nnew ? STEP_ALIVE : 0) | (kb ? STEP_KERNEL : 0);
}

// The wavefront step for large sets (ambiguous grammars make sets of hundreds of items): same
// structure, but the set under construction lives in LDS only and every loop over items runs in
// strips of 64.  Slower per item than wave_step, used only when a set does not fit 64 lanes.
template <class BaseT, class S>
__device__ __forceinline__ int wave_step_big(const TV &T, const BaseT &B, S &st, int d, uint32_t byte, uint32_t cl, uint32_t &cnt, uint32_t lane) {
    const uint32_t nb = cnt;
    const uint32_t cur = B.m - 1 + (uint32_t)(d - 1);
    const bool from_base = d == 1;
    const uint32_t sb = from_base ? B.last_lo : st.start(d - 1);
    const uint32_t se = from_base ? B.last_hi : nb;
    uint32_t nnew = 0;
    bool saw_end = false, failed = false;                // failed: the item budget is used up (sticky; the step runs on and reports at its end)
    auto insert = [&](uint32_t w, uint32_t o) {
        unsigned long long dup = 0;
        for (uint32_t s0 = 0; s0 < nnew; s0 += 64) {
            uint32_t xw = 0, xo = 0xFFFFFFFFu;
            if (s0 + lane < nnew) st.get(nb + s0 + lane, xw, xo);
            dup |= __ballot(s0 + lane < nnew && xw == w && xo == o);
        }
        const bool add = !dup && nb + nnew < st.cap;
        failed |= !dup && !add;
        if (add && lane == 0) st.put(nb + nnew, w, o);
        nnew += add ? 1u : 0u;
    };
    auto advance = [&](uint32_t p, uint32_t o) {
        for (;;) {
            const uint32_t w = T.advpq[p];
            insert(w, o);
            if (w & IW_END) { saw_end = true; return; }
            if ((w & IW_TERM) || !(w & IW_NT_NULLABLE)) return;
            p++;
        }
    };
    for (uint32_t s0 = sb; s0 < se; s0 += 64) {
        uint32_t sw = IW_END, so = 0;
        if (s0 + lane < se) { if (from_base) { const uint2 x = B.it[s0 + lane]; sw = x.x; so = x.y; } else st.get(s0 + lane, sw, so); }
        uint32_t nx = DFA_DEAD;
        if (sw & IW_TERM) nx = dfa_next(T, sw >> 16, byte, cl);
        unsigned long long m = __ballot((nx & 0xFFFFu) != DFA_DEAD);
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t lw = __builtin_amdgcn_readlane(sw, l), lo = __builtin_amdgcn_readlane(so, l), lnx = __builtin_amdgcn_readlane(nx, l);
            if ((lnx >> 16) & QF_CONT) insert((lw & 0xFFFFu) | (lnx << 16), lo);
            if ((lnx >> 16) & QF_ACCEPT) advance((lw & IW_POS_MASK) + 1, lo);
        }
        m = __ballot(!(sw & (IW_TERM | IW_END)));
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t Y = (__builtin_amdgcn_readlane(sw, l) >> IW_NT_SHIFT) & IW_NT_MASK;
            const uint32_t k0 = T.scan_off[Y * T.ncls + cl], k1 = T.scan_off[Y * T.ncls + cl + 1];
            for (uint32_t e = k0; e < k1; e++) {
                const uint2 ef = T.scan_list[e];
                if (ef.y & QF_CONT) insert(ef.x, cur);
                if (ef.y & QF_ACCEPT) advance((ef.x & IW_POS_MASK) + 1, cur);
            }
        }
    }
    if (saw_end) {
        for (uint32_t i = 0; i < nnew; i++) {
            uint32_t w, o;
            st.get(nb + i, w, o);                        // every lane reads the same item
            if (!(w & IW_END)) continue;
            const uint32_t X = (w & IW_POS_MASK) - T.end_base;
            if (X == T.N - 1) continue;
            const bool in_base = o < B.m;
            uint32_t jb, je;
            if (in_base) { jb = B.so[o]; je = B.so[o + 1]; }
            else { const int dj = (int)(o - (B.m - 1)); jb = st.start(dj); je = st.start(dj + 1); }
            for (uint32_t j0 = jb; j0 < je; j0 += 64) {
                uint32_t yw = IW_END, yo = 0;
                if (j0 + lane < je) { if (in_base) { const uint2 y = B.it[j0 + lane]; yw = y.x; yo = y.y; } else st.get(j0 + lane, yw, yo); }
                const bool nt = !(yw & (IW_TERM | IW_END));
                const uint32_t Y = (yw >> IW_NT_SHIFT) & IW_NT_MASK;
                uint32_t c0 = 0, c1 = 0;
                if (nt) { c0 = T.comp_off[Y * T.N + X]; c1 = T.comp_off[Y * T.N + X + 1]; }
                unsigned long long mm = __ballot(nt && c1 > c0);
                while (mm) {
                    const int l = __ffsll((long long)mm) - 1;
                    mm &= mm - 1;
                    const uint32_t lc0 = __builtin_amdgcn_readlane(c0, l), lc1 = __builtin_amdgcn_readlane(c1, l);
                    for (uint32_t e = lc0; e < lc1; e++) {
                        const uint32_t cw = T.comp_list[e];
                        if (cw != 0xFFFFFFFFu) insert(cw, o);
                        else advance((__builtin_amdgcn_readlane(yw, l) & IW_POS_MASK) + 1, __builtin_amdgcn_readlane(yo, l));
                    }
                }
            }
        }
    }
    if (failed) return STEP_OVERFLOW;
    // drop the completed items: forward compaction, strip by strip (a strip is read before it is written)
    uint32_t kept = 0;
    for (uint32_t s0 = 0; s0 < nnew; s0 += 64) {
        uint32_t w = IW_END, o = 0;
        if (s0 + lane < nnew) st.get(nb + s0 + lane, w, o);
        const bool keep = !(w & IW_END);
        const unsigned long long kb = __ballot(keep);
        if (keep) st.put(nb + kept + __popcll(kb & ((1ull << lane) - 1ull)), w, o);
        kept += (uint32_t)__popcll(kb);
    }
    cnt = nb + kept;
    st.set_start(d + 1, cnt);
    return (nnew ? STEP_ALIVE : 0) | (kept ? STEP_KERNEL : 0);
}

// What a wavefront remembers between two chunks of the same row: which trie path its stored sets
// belong to.  A node is named by (depth, rank of its first string).  Consecutive chunks share most
// of the path above their first node, so the next walk replays only what differs.
struct PathMemo {
    uint32_t rank_at;          // lane d: the node whose live set is stored at depth d (valid for 1 <= d <= valid)
    int valid;                 // depths 1..valid hold live sets of one root path
    int dead_depth;            // the node (dead_depth, dead_rank) below that path is known to leave no item: its subtree is dead
    uint32_t dead_rank;
    __device__ __forceinline__ void reset() { rank_at = 0; valid = 0; dead_depth = 0; dead_rank = 0; }
    __device__ __forceinline__ void note(int d, uint32_t rank, bool live, uint32_t lane) {   // a step was taken at depth d
        if (live) { valid = d; dead_depth = 0; if ((int)lane == d) rank_at = rank; }
        else { valid = d - 1; dead_depth = d; dead_rank = rank; }
    }
};

// Walk the nodes of one chunk.  anc(j) gives the first node's ancestor at depth j+1.  Returns
// false on overflow (the memo is then unusable); otherwise *bits_out holds the chunk's verdicts.
// `want` marks the strings of the chunk that still need a verdict (the others are decided by the
// token-mask cache); subtrees without such a string are skipped without a byte step.
template <class S, class Step, class Anc, class Nodes>
__device__ __forceinline__ bool walk_chunk(const DeviceTables &D, S &st, Step step, uint32_t chunk, uint32_t want,
                                           uint32_t begin, uint32_t end, Anc anc, Nodes node, uint32_t *bits_out,
                                           PathMemo &memo, uint32_t lane) {
    uint32_t i = begin;
    const uint32_t rank0 = chunk * (uint32_t)D.chunk_ranks;
    uint32_t bits = 0, cnt = 0;
    st.set_start(1, 0);
    TrieNode nd = node(i);
    const int n_anc = nd.depth - 1;                      // the path above the chunk's first node: reused or replayed
    if (nd.depth > S::max_depth) return false;
    int j = 0;
    while (j < n_anc && j < memo.valid && (uint32_t)__builtin_amdgcn_readlane((int)memo.rank_at, j + 1) == anc(j).rank) j++;
    if (j < n_anc && memo.dead_depth == j + 1 && j == memo.valid) {
        const TrieNode dn = anc(j);
        if (dn.rank == memo.dead_rank) {                 // the chunk starts inside a subtree known to be dead
            i = dn.skip; j = n_anc;
            if (i < end) nd = node(i);
        }
    } else if (j < memo.valid) { memo.valid = j; memo.dead_depth = 0; }
    cnt = st.start(j + 1);
    for (;;) {                                           // one loop, one call site of the byte step (keeps the code small)
        const bool warm = j < n_anc;
        const uint32_t nxt = i + 1;
        TrieNode cur, nx = nd;
        uint32_t rel = 0;
        bool do_step = true;
        if (warm) cur = anc(j);
        else {
            if (i >= end) break;
            cur = nd;
            if (nxt < end) nx = node(nxt);               // issued before the step so that it overlaps it
            rel = cur.rank - rank0;
            const uint32_t span = (cur.n_sub >= 32u ? 0xFFFFFFFFu : ((1u << cur.n_sub) - 1u)) << rel;
            do_step = (span & want) != 0;                // nothing to decide below this node: skip it without a step
            if (do_step) {
                if (cur.depth > S::max_depth) return false;
                cnt = st.start(cur.depth);               // forget the sets of the deeper path we came from
            }
        }
        int r = 0;
        if (do_step) {
            const int d = warm ? j + 1 : (int)cur.depth;
            r = step(d, cur.byte, cur.cls, cnt);
            if (r & STEP_OVERFLOW) return false;
            memo.note(d, cur.rank, (r & STEP_KERNEL) != 0, lane);
        }
        if (warm) {
            if (r & STEP_KERNEL) { j++; continue; }
            i = cur.skip; cnt = st.start(j + 1); j = n_anc;   // that whole subtree is dead
            if (i < end) nd = node(i);
            continue;
        }
        if (cur.has_string && (r & STEP_ALIVE)) bits |= 1u << rel;
        const uint32_t ni = (r & STEP_KERNEL) ? nxt : cur.skip;
        if (ni == nxt) nd = nx;
        else if (ni < end) nd = node(ni);
        i = ni;
    }
    *bits_out = bits;
    return true;
}

__device__ __forceinline__ uint32_t load_bits(const DeviceTables &D, const uint32_t *bitmap_row, uint32_t chunk) {
    const uint8_t *rowp = reinterpret_cast<const uint8_t *>(bitmap_row);
    if (D.chunk_ranks == 32) return reinterpret_cast<const uint32_t *>(rowp)[chunk];
    if (D.chunk_ranks == 16) return reinterpret_cast<const uint16_t *>(rowp)[chunk];
    return rowp[chunk];
}

__device__ __forceinline__ void store_bits(const DeviceTables &D, uint32_t *rank_mask, uint32_t row, uint32_t chunk, uint32_t bits) {
    uint8_t *rowp = reinterpret_cast<uint8_t *>(rank_mask + (size_t)row * D.Wr);
    if (D.chunk_ranks == 32) reinterpret_cast<uint32_t *>(rowp)[chunk] = bits;
    else if (D.chunk_ranks == 16) reinterpret_cast<uint16_t *>(rowp)[chunk] = (uint16_t)bits;
    else rowp[chunk] = (uint8_t)bits;
}
// several walks may add verdicts to the same word of the rank-ordered bitmap: atomic OR
__device__ __forceinline__ void or_bits(const DeviceTables &D, uint32_t *rank_mask, uint32_t row, uint32_t chunk, uint32_t bits) {
    if (!bits) return;
    const uint32_t byte_off = chunk * ((uint32_t)D.chunk_ranks >> 3);
    atomicOr(rank_mask + (size_t)row * D.Wr + (byte_off >> 2), bits << ((byte_off & 3u) * 8u));
}

// Token-mask cache (Section 4.3): merge the cached bitsets of every item of the row's current set,
// store the strings some terminal swallows whole, and queue the chunks that hold strings which
// need the parser.  One lane per 64 ranks (two words of the rank-ordered bitmap, 64 / chunk_ranks
// chunks); a wavefront appends its chunks to the queue in chunk order with one atomic, so that
// neighbours in the queue are mostly neighbours in the trie (the walk reuses shared paths).
__global__ __launch_bounds__(256) void cache_merge_kernel(MaskArgs a) {
    const DeviceTables &D = a.tab;
    const uint32_t t = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y, lane = threadIdx.x & 63;
    const RowChart rc = a.rows[row];
    const uint32_t w0 = 2 * t, Wr = (uint32_t)D.Wr, cr = (uint32_t)D.chunk_ranks;
    const bool has0 = w0 < Wr, has1 = w0 + 1 < Wr;
    uint32_t v0 = 0, v1 = 0, c0 = 0, c1 = 0;
    if (has0) {
        if (rc.n_ent == 0) { c0 = 0xFFFFFFFFu; c1 = has1 ? 0xFFFFFFFFu : 0u; }
        for (uint32_t k = 0; k < rc.n_ent; k++) {
            const size_t r = (size_t)a.entries[rc.ent_base + k] * Wr + w0;
            v0 |= D.ci_valid[r]; c0 |= D.ci_cd[r];
            if (has1) { v1 |= D.ci_valid[r + 1]; c1 |= D.ci_cd[r + 1]; }
        }
        a.rank_mask[(size_t)row * Wr + w0] = v0;
        if (has1) a.rank_mask[(size_t)row * Wr + w0 + 1] = v1;
    }
    const unsigned long long want = ((unsigned long long)(c1 & ~v1) << 32) | (c0 & ~v0);
    const uint32_t per_lane = 64u / cr, chunk0 = t * per_lane;
    const unsigned long long cm = cr == 32 ? 0xFFFFFFFFull : ((1ull << cr) - 1ull);
    uint32_t n_mine = 0;
    for (uint32_t k = 0; k < per_lane; k++) n_mine += ((want >> (k * cr)) & cm) != 0 && chunk0 + k < (uint32_t)D.n_chunks;
    if (!__ballot(n_mine != 0)) return;
    uint32_t incl = n_mine;                                  // inclusive prefix sum over the lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) { const uint32_t up = __shfl_up(incl, d); if ((int)lane >= d) incl += up; }
    uint32_t base = 0;
    if (lane == 63) base = atomicAdd(&a.counters[1], incl);
    base = __shfl(base, 63);
    uint32_t at = base + incl - n_mine;
    for (uint32_t k = 0; k < per_lane; k++) {
        const uint32_t wk = (uint32_t)((want >> (k * cr)) & cm), chunk = chunk0 + k;
        if (!wk || chunk >= (uint32_t)D.n_chunks) continue;
        const uint32_t begin = D.chunk_begin[chunk], n_nodes = D.chunk_end[chunk] - begin;
        a.work[at++] = make_uint4(row | (n_nodes > 0xFFFFu ? 0xFFFF0000u : n_nodes << 16), chunk, wk, begin);
    }
}

// The packed charts of a call, a few KB, from pinned host memory to device memory: launched like
// the kernels behind it (the runtime's copy path costs the host several times as long per call).
__global__ __launch_bounds__(256) void upload_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, uint32_t n16) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

static const uint32_t BASE_LDS_BYTES = (BASE_SETS_LDS + 1) * 4 + BASE_ITEMS_LDS * 8;
__host__ __device__ inline uint32_t wave_region_bytes(uint32_t cap) {
    // prefetched nodes, ancestor nodes, the row's chart, item words, origins; a multiple of 16
    return (WALK_NODES_LDS + CHUNK_ANC) * 16 + BASE_LDS_BYTES + (cap * 8 + 15) / 16 * 16;
}

struct ParentAnc {             // ancestor node at depth j+1 through the parent links
    const TrieNode *nodes; const uint32_t *parent; uint32_t first; int d0;
    __device__ __forceinline__ TrieNode operator()(int j) const {
        uint32_t x = first;
        for (int k = d0; k > j + 1; k--) x = parent[x];
        return nodes[x];
    }
};

__device__ __forceinline__ BaseG global_base(const MaskArgs &a, uint32_t row) {
    const RowChart rc = a.rows[row];
    BaseG B;
    B.so = a.set_off + rc.set_base;
    B.it = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
    B.m = rc.n_sets;
    B.last_lo = B.so[rc.n_sets - 1];
    B.last_hi = B.so[rc.n_sets];
    return B;
}

// The parser walk.  Persistent blocks; every wavefront takes queued chunks g, g + stride, ...
template <int MODE>
__global__ __launch_bounds__(WALK_BLOCK) __attribute__((amdgpu_waves_per_eu(6))) void mask_walk_kernel(MaskArgs a) {
    extern __shared__ __align__(16) uint8_t smem[];
    const DeviceTables &D = a.tab;
    const uint32_t tid = threadIdx.x;
    const uint32_t n_work = a.counters[1];
    // The queue is dealt to the blocks in tiles, round robin; a tile is WALK_WAVES runs of `run`
    // consecutive items, and inside a block the wavefronts take the next run of the block's share
    // whenever they are free (LDS counter), so that one long walk does not hold up the items behind
    // it.  Items of a run are mostly neighbouring chunks of one row: the wavefront keeps its path
    // (PathMemo) from one to the next.  Short queues are dealt item by item so that all wavefronts work.
    uint32_t run = n_work / (gridDim.x * WALK_WAVES);
    run = run < 1 ? 1 : (run > WALK_RUN_MAX ? WALK_RUN_MAX : run);
    const uint32_t tile = run * WALK_WAVES;
    if (blockIdx.x * tile >= n_work) return;            // uniform: not even the block's first tile exists
    TV T;
    uint32_t off = stage_tables<MODE>(D, smem, T, tid, WALK_BLOCK);
    uint32_t *next_item = reinterpret_cast<uint32_t *>(smem + off);   // the block's counter of items handed out
    off += 16;
    if (tid == 0) *next_item = 0;
    __syncthreads();                                     // the only block-wide barrier; below, wavefronts run on their own
    const uint32_t wave = tid >> 6, lane = tid & 63;
    const uint32_t cap = (uint32_t)a.lane_cap;
    uint8_t *region = smem + off + wave * wave_region_bytes(cap);
    TrieNode *l_nodes = reinterpret_cast<TrieNode *>(region);
    TrieNode *l_anc = l_nodes + WALK_NODES_LDS;
    uint32_t *l_so = reinterpret_cast<uint32_t *>(region + (WALK_NODES_LDS + CHUNK_ANC) * 16);
    uint2 *l_it = reinterpret_cast<uint2 *>(l_so + BASE_SETS_LDS + 1);
    WaveLdsStore st;
    st.pq = reinterpret_cast<uint32_t *>(l_it + BASE_ITEMS_LDS);
    st.org = st.pq + cap;
    st.ss_reg = 0;
    st.lane = lane;
    st.cap = cap;
    PathMemo memo;
    memo.reset();
    uint32_t memo_row = 0xFFFFFFFFu;
    for (;;) {
        uint32_t k = 0;
        if (lane == 0) k = atomicAdd(next_item, 1u);
        k = (uint32_t)__builtin_amdgcn_readfirstlane((int)k);
        const uint32_t t_base = ((k / WALK_WAVES) * gridDim.x + blockIdx.x) * tile;
        if (t_base >= n_work) break;                    // this and every later tile of this block lie beyond the queue
        const uint32_t g0 = t_base + (k % WALK_WAVES) * run;
        for (uint32_t g = g0; g < g0 + run && g < n_work; g++) {
            const uint4 item = a.work[g];               // row | node count << 16, chunk, undecided strings, first node
            const uint32_t row = item.x & 0xFFFFu, n_nodes = item.x >> 16, chunk = item.y, want = item.z, begin = item.w;
            const RowChart rc = a.rows[row];
            const uint32_t *g_so = a.set_off + rc.set_base;
            const uint2 *g_it = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
            const bool base_fits = rc.n_sets <= BASE_SETS_LDS && rc.n_items <= BASE_ITEMS_LDS;
            // all 64 lanes pull the chunk's nodes, the ancestors of its first node and the row's chart into LDS
            if (n_nodes <= (uint32_t)WALK_NODES_LDS)
                for (uint32_t k2 = lane; k2 < n_nodes; k2 += 64) l_nodes[k2] = D.nodes[begin + k2];
            if (lane < CHUNK_ANC) l_anc[lane] = D.chunk_anc[(size_t)chunk * CHUNK_ANC + lane];
            if (row != memo_row) {                       // another row: its chart, and no path to reuse
                memo.reset();
                memo_row = row;
                if (base_fits) {
                    for (uint32_t k2 = lane; k2 <= rc.n_sets; k2 += 64) l_so[k2] = g_so[k2];
                    for (uint32_t k2 = lane; k2 < rc.n_items; k2 += 64) l_it[k2] = g_it[k2];
                }
            }
            // lanes read what other lanes of their own wavefront wrote: LDS serves one wavefront's
            // accesses in issue order; the fences keep the compiler from moving accesses across
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            {
                uint32_t bits = 0;
                bool ok = cap > 0 && n_nodes <= (uint32_t)WALK_NODES_LDS && l_nodes[0].depth - 1 <= CHUNK_ANC;
                if (ok) {
                    auto anc = [&](int j) { return l_anc[j]; };
                    auto node = [&](uint32_t i) { return l_nodes[i - begin]; };
                    // the row's chart through generic pointers: its LDS copy when it was staged, else global memory
                    const uint32_t *b_so = base_fits ? l_so : g_so;
                    const uint2 *b_it = base_fits ? l_it : g_it;
                    const BaseG B{b_so, b_it, rc.n_sets, b_so[rc.n_sets - 1], rc.n_items};
                    ok = walk_chunk(D, st, [&](int d, uint32_t byte, uint32_t cl, uint32_t &cnt) {
                                            const uint32_t keep = cnt;
                                            int r = wave_step(T, B, st, d, byte, cl, cnt, lane);
                                            if (r & STEP_WIDE) { cnt = keep; r = wave_step_big(T, B, st, d, byte, cl, cnt, lane); }
                                            return r; },
                                    chunk, want, begin, begin + n_nodes, anc, node, &bits, memo, lane);
                }
                if (!ok) memo.reset();
                if (lane == 0) {
                    if (!ok) {
                        const uint32_t slot = atomicAdd(&a.counters[0], 1u);
                        if (slot < a.overflow_cap) a.overflow_list[slot] = make_uint4(row, chunk, want, 0);
                    } else or_bits(D, a.rank_mask, row, chunk, bits & want);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the next round overwrites the staged data
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// Fallback: one wavefront per chunk that outgrew LDS; same walk with the strip-wise step and the
// item list in a global-memory arena.
__global__ __launch_bounds__(64) void mask_fallback_kernel(MaskArgs a) {
    const DeviceTables &D = a.tab;
    TV T;
    stage_tables<2>(D, nullptr, T, 0, 1);
    const uint32_t lane = threadIdx.x;
    uint32_t n = a.counters[0];
    if (n > a.overflow_cap) { if (blockIdx.x == 0 && lane == 0) atomicAdd(&a.counters[2], n - a.overflow_cap); n = a.overflow_cap; }
    GlobalStore st{a.fb_items + (size_t)blockIdx.x * FB_ITEMS_PER_WAVE, a.fb_set_start + (size_t)blockIdx.x * (FB_DEPTH_MAX + 2), (uint32_t)a.fb_cap};
    for (uint32_t e = blockIdx.x; e < n; e += gridDim.x) {
        const uint4 ent = a.overflow_list[e];
        const BaseG B = global_base(a, ent.x);
        const uint32_t begin = D.chunk_begin[ent.y], end = D.chunk_end[ent.y];
        ParentAnc anc{D.nodes, D.parent, begin, D.nodes[begin].depth};
        uint32_t bits = 0;
        PathMemo memo;
        memo.reset();
        const bool ok = walk_chunk(D, st, [&](int d, uint32_t byte, uint32_t cl, uint32_t &cnt) { return wave_step_big(T, B, st, d, byte, cl, cnt, lane); },
                                   ent.y, ent.z, begin, end, anc, [&](uint32_t i) { return D.nodes[i]; }, &bits, memo, lane);
        if (lane == 0) {
            if (!ok) atomicAdd(&a.counters[2], 1u);
            else or_bits(D, a.rank_mask, ent.x, ent.y, bits & ent.z);
        }
        // lanes write the arena, lane-uniform reads follow in the next round: keep the order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// ---- mask automaton ------------------------------------------------------------------------------
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
static const uint32_t AUT_REF = 0x80000000u;
enum : uint32_t { AT_NONE = 0xFFFFFFFFu,   // not computed yet
                  AT_DEAD = 0xFFFFFFFEu,   // the byte leaves no item
                  AT_SINK = 0xFFFFFFFDu,   // only completed items: the string may end here, nothing can follow
                  AT_BUSY = 0xFFFFFFFCu,   // a wavefront is computing it
                  AT_FAIL = 0xFFFFFFFBu }; // does not fit this block's budgets: such strings go to the fallback pass

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

// Transitions of state `id` that leave no item at all are settled when the state is made, for all
// byte classes at once (lane = class): an item before a terminal survives a class iff its DFA has
// an edge, an item that waits for a nonterminal iff some terminal that can begin it has one.  What
// remains for the byte step proper are the few classes that lead somewhere.  item(i) is uniform.
template <class ItemWord>
__device__ __forceinline__ void aut_mark_dead(const TV &T, const Aut &A, ItemWord item, uint32_t n, uint32_t id, uint32_t lane) {
    auto survives = [&](uint32_t w, uint32_t byte, uint32_t c) -> bool {   // no branch: both kinds of look-up are made, with safe indices
        const bool term = (w & IW_TERM) != 0, end = (w & IW_END) != 0;
        const uint32_t info = T.qinfo[term ? w >> 16 : 0u];
        const bool lit = (info & QF_LITERAL) != 0;
        const uint32_t d = T.delta[(lit ? 0u : info >> 16) * T.ncls + c];
        const bool a_term = lit ? (((info >> 8) & 0xFFu) == byte && (info & QF_CONT)) : (d & 0xFFFFu) != DFA_DEAD;
        const uint32_t Y = term || end ? 0u : (w >> IW_NT_SHIFT) & IW_NT_MASK;
        const bool a_nt = T.scan_off[Y * T.ncls + c + 1] > T.scan_off[Y * T.ncls + c];
        return !end && (term ? a_term : a_nt);
    };
    for (uint32_t c0 = 0; c0 < A.ncls; c0 += 64) {
        const uint32_t c = c0 + lane < A.ncls ? c0 + lane : A.ncls - 1;   // surplus lanes repeat the last class
        const uint32_t byte = A.rep[c];
        bool alive = false;
        for (uint32_t i = 0; i < n; i += 4) {                // four items at a time: their look-ups are independent of each other
            const uint32_t w0 = item(i), w1 = i + 1 < n ? item(i + 1) : (uint32_t)IW_END, w2 = i + 2 < n ? item(i + 2) : (uint32_t)IW_END,
                           w3 = i + 3 < n ? item(i + 3) : (uint32_t)IW_END;
            const bool a0 = survives(w0, byte, c), a1 = survives(w1, byte, c), a2 = survives(w2, byte, c), a3 = survives(w3, byte, c);
            alive |= a0 | a1 | a2 | a3;
        }
        if (!alive) A.trans[id * A.ncls + c] = AT_DEAD;
    }
}

static const uint32_t HQ_VALID = 0x80000000u;

__device__ __forceinline__ uint32_t lds_load(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
__device__ __forceinline__ void lds_store(uint32_t *p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }

// One Earley byte step from state s on byte class cl is done by a whole wavefront with uniform
// control flow (all lanes call these functions with identical arguments).  Both variants leave the
// new set, completed items dropped, in the wavefront's scratch (sc_w, sc_o) and return AUT_OK,
// AUT_WIDE (narrow variant only: more than 64 new items) or AUT_OVER (no room).
enum { AUT_OK = 0, AUT_WIDE = 1, AUT_OVER = 2 };

template <class BaseT>
struct AutSets {           // resolves origin references
    const BaseT &B;
    const Aut &A;
    __device__ __forceinline__ void view(uint32_t ref, const uint2 *&p, uint32_t &n) const {
        if (ref & AUT_REF) { const uint2 h = A.hdr[ref & ~AUT_REF]; p = A.arena + h.x; n = h.y; }
        else { const uint32_t lo = B.so[ref]; p = B.it + lo; n = B.so[ref + 1] - lo; }
    }
};

// Narrow variant: the set under construction lives in registers (lane j holds new item j), so the
// duplicate test is one compare + ballot; the source set is read in strips of 64 items.
template <class BaseT>
__device__ __forceinline__ int aut_step_narrow(const TV &T, const AutSets<BaseT> &S, uint32_t *sc_w, uint32_t *sc_o, uint32_t sc_cap,
                                               uint32_t cur, uint32_t byte, uint32_t cl, uint32_t lane, uint32_t &nnew_out, uint32_t &kept_out) {
    const uint2 *src;
    uint32_t ns;
    S.view(cur, src, ns);
    uint32_t nw = 0xFFFFFFFFu, no = 0, nnew = 0;             // no item word is all ones
    bool saw_end = false, failed = false;                    // failed is sticky: the step runs on and reports at its end
    const uint32_t room = sc_cap < 64u ? sc_cap : 64u;
    auto insert = [&](uint32_t w, uint32_t o) {              // uniform arguments; no branch
        const bool fresh = __ballot(nw == w && no == o) == 0;
        const bool add = fresh && nnew < room;
        failed |= fresh && !add;
        const bool mine = add && lane == nnew;
        nw = mine ? w : nw;
        no = mine ? o : no;
        nnew += add ? 1u : 0u;
    };
    auto advance = [&](uint32_t p, uint32_t o) {             // dot arrives at p: skip nullable nonterminals, canonical END item
        for (;;) {
            const uint32_t w = T.advpq[p];
            insert(w, o);
            if (w & IW_END) { saw_end = true; return; }
            if ((w & IW_TERM) || !(w & IW_NT_NULLABLE)) return;
            p++;
        }
    };
    for (uint32_t s0 = 0; s0 < ns; s0 += 64) {
        uint32_t sw = IW_END, so = 0;                        // lanes beyond the set hold an inert item
        if (s0 + lane < ns) { const uint2 x = src[s0 + lane]; sw = x.x; so = x.y; }
        // Scan, terminal items: all DFA steps at once, then the survivors one after the other
        uint32_t nx = DFA_DEAD, aw = 0;
        if (sw & IW_TERM) {
            aw = T.advpq[(sw & IW_POS_MASK) + 1];            // the item behind the terminal, fetched alongside the DFA step
            nx = dfa_next(T, sw >> 16, byte, cl);
        }
        unsigned long long m = __ballot((nx & 0xFFFFu) != DFA_DEAD);
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t lw = __builtin_amdgcn_readlane(sw, l), lo = __builtin_amdgcn_readlane(so, l), lnx = __builtin_amdgcn_readlane(nx, l);
            if ((lnx >> 16) & QF_CONT) insert((lw & 0xFFFFu) | (lnx << 16), lo);   // no longest match: keep matching ...
            if ((lnx >> 16) & QF_ACCEPT) {                                         // ... and also finish here
                const uint32_t law = __builtin_amdgcn_readlane(aw, l);
                insert(law, lo);
                if (law & IW_END) saw_end = true;
                else if (!(law & IW_TERM) && (law & IW_NT_NULLABLE)) advance((lw & IW_POS_MASK) + 2, lo);
            }
        }
        // Scan, items that wait for a nonterminal Y: the tabulated first steps of every terminal that can begin Y
        uint32_t sk0 = 0, sk1 = 0;
        if (!(sw & (IW_TERM | IW_END))) {
            const uint32_t Y = (sw >> IW_NT_SHIFT) & IW_NT_MASK;
            sk0 = T.scan_off[Y * T.ncls + cl]; sk1 = T.scan_off[Y * T.ncls + cl + 1];
        }
        m = __ballot(sk1 > sk0);
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t k0 = __builtin_amdgcn_readlane(sk0, l), k1 = __builtin_amdgcn_readlane(sk1, l);
            for (uint32_t e0 = k0; e0 < k1; e0 += 64) {
                uint2 ef = make_uint2(0, 0);
                if (e0 + lane < k1) ef = T.scan_list[e0 + lane];
                const uint32_t n_e = k1 - e0 < 64 ? k1 - e0 : 64;
                for (uint32_t t = 0; t < n_e; t++) {
                    const uint32_t ent = __builtin_amdgcn_readlane(ef.x, t), f = __builtin_amdgcn_readlane(ef.y, t);
                    if (f & QF_CONT) insert(ent, cur);
                    if (f & QF_ACCEPT) advance((ent & IW_POS_MASK) + 1, cur);
                }
            }
        }
    }
    if (saw_end) {
        // Complete: new items are visited in order; completing may append more
        unsigned long long visited = 0;
        for (;;) {
            const unsigned long long todo = __ballot(lane < nnew && (nw & IW_END)) & ~visited;
            if (!todo) break;
            const int i = __ffsll((long long)todo) - 1;
            visited |= 1ull << i;
            const uint32_t w = __builtin_amdgcn_readlane(nw, i);
            const uint32_t X = (w & IW_POS_MASK) - T.end_base;
            if (X == T.N - 1) continue;                      // the start rule is complete: the prefix is a sentence
            const uint32_t o = __builtin_amdgcn_readlane(no, i);
            const uint2 *yp;
            uint32_t yn;
            S.view(o, yp, yn);
            for (uint32_t j0 = 0; j0 < yn; j0 += 64) {
                uint32_t yw = IW_END, yo = 0;
                if (j0 + lane < yn) { const uint2 y = yp[j0 + lane]; yw = y.x; yo = y.y; }
                const bool nt = !(yw & (IW_TERM | IW_END));
                const uint32_t Y = (yw >> IW_NT_SHIFT) & IW_NT_MASK;
                uint32_t c0 = 0, c1 = 0, cw0 = 0;
                if (nt) { c0 = T.comp_off[Y * T.N + X]; c1 = T.comp_off[Y * T.N + X + 1]; }
                if (c1 > c0) cw0 = T.comp_list[c0];          // every lane fetches the first entry of its own list
                unsigned long long mm = __ballot(nt && c1 > c0);
                while (mm) {
                    const int l = __ffsll((long long)mm) - 1;
                    mm &= mm - 1;
                    const uint32_t lc0 = __builtin_amdgcn_readlane(c0, l), lc1 = __builtin_amdgcn_readlane(c1, l);
                    for (uint32_t e = lc0; e < lc1; e++) {
                        const uint32_t cw = e == lc0 ? (uint32_t)__builtin_amdgcn_readlane(cw0, l) : T.comp_list[e];
                        if (cw != 0xFFFFFFFFu) insert(cw, o);
                        else advance((__builtin_amdgcn_readlane(yw, l) & IW_POS_MASK) + 1, __builtin_amdgcn_readlane(yo, l));   // Y itself is complete: the waiting item moves on
                    }
                }
            }
        }
    }
    if (failed) return nnew >= 64u ? AUT_WIDE : AUT_OVER;
    // completed items are needed only while their own set is processed: store the others
    const bool keep = lane < nnew && !(nw & IW_END);
    const unsigned long long kb = __ballot(keep);
    if (keep) { const uint32_t at = (uint32_t)__popcll(kb & ((1ull << lane) - 1ull)); sc_w[at] = nw; sc_o[at] = no; }
    nnew_out = nnew;
    kept_out = (uint32_t)__popcll(kb);
    return AUT_OK;
}

// Wide variant (ambiguous grammars make sets of hundreds of items): the set under construction lives
// in the scratch and every loop over its items runs in strips of 64.
template <class BaseT>
__device__ __forceinline__ int aut_step_wide(const TV &T, const AutSets<BaseT> &S, uint32_t *sc_w, uint32_t *sc_o, uint32_t sc_cap,
                                             uint32_t cur, uint32_t byte, uint32_t cl, uint32_t lane, uint32_t &nnew_out, uint32_t &kept_out) {
    const uint2 *src;
    uint32_t ns;
    S.view(cur, src, ns);
    uint32_t nnew = 0;
    bool saw_end = false, failed = false;
    auto insert = [&](uint32_t w, uint32_t o) {              // uniform arguments
        unsigned long long dup = 0;
        for (uint32_t s0 = 0; s0 < nnew; s0 += 64) {
            const bool in = s0 + lane < nnew;
            uint32_t xw = 0, xo = 0;
            if (in) { xw = sc_w[s0 + lane]; xo = sc_o[s0 + lane]; }
            dup |= __ballot(in && xw == w && xo == o);
        }
        const bool add = !dup && nnew < sc_cap;
        failed |= !dup && !add;
        if (add && lane == 0) { sc_w[nnew] = w; sc_o[nnew] = o; }
        nnew += add ? 1u : 0u;
    };
    auto advance = [&](uint32_t p, uint32_t o) {
        for (;;) {
            const uint32_t w = T.advpq[p];
            insert(w, o);
            if (w & IW_END) { saw_end = true; return; }
            if ((w & IW_TERM) || !(w & IW_NT_NULLABLE)) return;
            p++;
        }
    };
    for (uint32_t s0 = 0; s0 < ns; s0 += 64) {
        uint32_t sw = IW_END, so = 0;
        if (s0 + lane < ns) { const uint2 x = src[s0 + lane]; sw = x.x; so = x.y; }
        uint32_t nx = DFA_DEAD;
        if (sw & IW_TERM) nx = dfa_next(T, sw >> 16, byte, cl);
        unsigned long long m = __ballot((nx & 0xFFFFu) != DFA_DEAD);
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t lw = __builtin_amdgcn_readlane(sw, l), lo = __builtin_amdgcn_readlane(so, l), lnx = __builtin_amdgcn_readlane(nx, l);
            if ((lnx >> 16) & QF_CONT) insert((lw & 0xFFFFu) | (lnx << 16), lo);
            if ((lnx >> 16) & QF_ACCEPT) advance((lw & IW_POS_MASK) + 1, lo);
        }
        uint32_t sk0 = 0, sk1 = 0;
        if (!(sw & (IW_TERM | IW_END))) {
            const uint32_t Y = (sw >> IW_NT_SHIFT) & IW_NT_MASK;
            sk0 = T.scan_off[Y * T.ncls + cl]; sk1 = T.scan_off[Y * T.ncls + cl + 1];
        }
        m = __ballot(sk1 > sk0);
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t k0 = __builtin_amdgcn_readlane(sk0, l), k1 = __builtin_amdgcn_readlane(sk1, l);
            for (uint32_t e = k0; e < k1; e++) {
                const uint2 ef = T.scan_list[e];
                if (ef.y & QF_CONT) insert(ef.x, cur);
                if (ef.y & QF_ACCEPT) advance((ef.x & IW_POS_MASK) + 1, cur);
            }
        }
    }
    if (saw_end) {
        for (uint32_t i = 0; i < nnew; i++) {
            const uint32_t w = sc_w[i], o = sc_o[i];         // every lane reads the same item
            if (!(w & IW_END)) continue;
            const uint32_t X = (w & IW_POS_MASK) - T.end_base;
            if (X == T.N - 1) continue;
            const uint2 *yp;
            uint32_t yn;
            S.view(o, yp, yn);
            for (uint32_t j0 = 0; j0 < yn; j0 += 64) {
                uint32_t yw = IW_END, yo = 0;
                if (j0 + lane < yn) { const uint2 y = yp[j0 + lane]; yw = y.x; yo = y.y; }
                const bool nt = !(yw & (IW_TERM | IW_END));
                const uint32_t Y = (yw >> IW_NT_SHIFT) & IW_NT_MASK;
                uint32_t c0 = 0, c1 = 0;
                if (nt) { c0 = T.comp_off[Y * T.N + X]; c1 = T.comp_off[Y * T.N + X + 1]; }
                unsigned long long mm = __ballot(nt && c1 > c0);
                while (mm) {
                    const int l = __ffsll((long long)mm) - 1;
                    mm &= mm - 1;
                    const uint32_t lc0 = __builtin_amdgcn_readlane(c0, l), lc1 = __builtin_amdgcn_readlane(c1, l);
                    for (uint32_t e = lc0; e < lc1; e++) {
                        const uint32_t cw = T.comp_list[e];
                        if (cw != 0xFFFFFFFFu) insert(cw, o);
                        else advance((__builtin_amdgcn_readlane(yw, l) & IW_POS_MASK) + 1, __builtin_amdgcn_readlane(yo, l));
                    }
                }
            }
        }
    }
    if (failed) return AUT_OVER;
    // drop the completed items: forward compaction, strip by strip (a strip is read before it is written)
    uint32_t kept = 0;
    for (uint32_t s0 = 0; s0 < nnew; s0 += 64) {
        uint32_t w = IW_END, o = 0;
        if (s0 + lane < nnew) { w = sc_w[s0 + lane]; o = sc_o[s0 + lane]; }
        const bool keep = !(w & IW_END);
        const unsigned long long kb = __ballot(keep);
        if (keep) { const uint32_t at = kept + (uint32_t)__popcll(kb & ((1ull << lane) - 1ull)); sc_w[at] = w; sc_o[at] = o; }
        kept += (uint32_t)__popcll(kb);
    }
    nnew_out = nnew;
    kept_out = kept;
    return AUT_OK;
}

// The transition of state s on class cl: take the byte step, then find the state that holds the
// resulting set (sets are interned by content: the same items in the same order are the same
// state) or make a new one.  Returns a state id or AT_DEAD / AT_SINK / AT_FAIL.
template <class BaseT>
__device__ __forceinline__ uint32_t aut_transition(const TV &T, const BaseT &B, const Aut &A, uint32_t *sc_w, uint32_t *sc_o, uint32_t sc_cap,
                                                   uint32_t s, uint32_t byte, uint32_t cl, uint32_t lane) {
    const AutSets<BaseT> S{B, A};
    const uint32_t cur = s == 0 ? B.m - 1 : (AUT_REF | s);   // the source set; also what items predicted in it get as origin
    uint32_t nnew = 0, kept = 0;
    const uint2 *src_p;
    uint32_t src_n;
    S.view(cur, src_p, src_n);
    int st = src_n > 48u ? AUT_WIDE : aut_step_narrow(T, S, sc_w, sc_o, sc_cap, cur, byte, cl, lane, nnew, kept);   // a wide source set rarely leaves a narrow one
    if (st == AUT_WIDE) st = aut_step_wide(T, S, sc_w, sc_o, sc_cap, cur, byte, cl, lane, nnew, kept);
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
    aut_mark_dead(T, A, [&](uint32_t i) { return sc_w[i]; }, kept, id, lane);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // items before the hash, the hash before the header that makes the state visible
    if (lane == 0) A.hash[id] = h;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) A.hdr[id] = make_uint2(at, kept);
    return id;
}

// Compute the transition of state s on class cl (the caller owns it: its entry is AT_BUSY) and publish it.
template <class BaseT>
__device__ __forceinline__ void aut_resolve(const TV &T, const BaseT &B, const Aut &A, uint32_t *sc_w, uint32_t *sc_o, uint32_t sc_cap,
                                            uint32_t s, uint32_t cl, uint32_t lane) {
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");   // the states this step reads were published by other wavefronts
    const uint32_t r = aut_transition(T, B, A, sc_w, sc_o, sc_cap, s, A.rep[cl], cl, lane);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // the new state before the transition that leads to it
    if (lane == 0) lds_store(&A.trans[s * A.ncls + cl], r);
}

// A wavefront whose strings miss several transitions at once computes one and leaves the others in
// the help queue; wavefronts that wait or have run out of strings take them from there.  Serves one
// request if there is one; returns false when the queue is empty.  Uniform over the wavefront.
template <class BaseT>
__device__ __forceinline__ bool aut_help(const TV &T, const BaseT &B, const Aut &A, uint32_t *sc_w, uint32_t *sc_o, uint32_t sc_cap, uint32_t lane, uint32_t &steps) {
    uint32_t tail = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&A.ctl[4]));
    tail = tail < (uint32_t)AUT_HELP_QUEUE ? tail : (uint32_t)AUT_HELP_QUEUE;
    const uint32_t head = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&A.ctl[5]));
    if (head >= tail) return false;
    uint32_t got = 0;
    if (lane == 0) got = atomicCAS(&A.ctl[5], head, head + 1u) == head ? 1u : 0u;
    if (!__builtin_amdgcn_readfirstlane((int)got)) return true;            // another wavefront took it: look again
    uint32_t e = 0;
    for (int tries = 0; tries < AUT_SPIN_LIMIT; tries++) {    // the entry is written right after its place was handed out
        e = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&A.hq[head]));
        if (e & HQ_VALID) break;
        __builtin_amdgcn_s_sleep(1);
    }
    if (!(e & HQ_VALID) || (e & 0x7FFFFF00u) == 0x7FFFFF00u) return true;   // a place whose request was settled before it was queued
    aut_resolve(T, B, A, sc_w, sc_o, sc_cap, (e & ~HQ_VALID) >> 8, e & 0xFFu, lane);
    steps++;
    return true;
}

__host__ __device__ inline uint32_t aut_round16(uint32_t x) { return (x + 15u) & ~15u; }

// Grid (parts, rows).  A block takes slices of AUT_SUB_WORDS words of its row's rank-ordered bitmap in
// turn: it merges the token-mask cache rows of the row's current set (Section 4.3: strings a terminal
// swallows whole are valid at once), lists the strings that need the parser, and its wavefronts
// take the list in batches of 64 strings, one lane per string.  The verdicts of a slice are
// collected in LDS and stored once: no atomics on global memory and nothing to clear beforehand.
template <int MODE>
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
    uint32_t *l_so = reinterpret_cast<uint32_t *>(smem + off); off += aut_round16((BASE_SETS_LDS + 1) * 4);
    uint2 *l_it = reinterpret_cast<uint2 *>(smem + off); off += BASE_ITEMS_LDS * 8;
    uint32_t *l_ent = reinterpret_cast<uint32_t *>(smem + off); off += AUT_ENT_LDS * 4;
    uint8_t *l_rep = smem + off; off += 256;
    A.rep = l_rep;
    uint32_t *vslice = reinterpret_cast<uint32_t *>(smem + off); off += AUT_SUB_WORDS * 4;
    uint32_t *cslice = reinterpret_cast<uint32_t *>(smem + off); off += AUT_SUB_WORDS * 4;
    uint8_t *pairs = smem + off; off += AUT_SUB_WORDS / 2;   // slots of the word pairs that hold undecided strings
    A.arena = reinterpret_cast<uint2 *>(smem + off); off += aut_round16(A.arena_cap * 8);
    uint32_t *sc_w = reinterpret_cast<uint32_t *>(smem + off) + (size_t)wave * 2 * sc_cap;
    uint32_t *sc_o = sc_w + sc_cap;
    // the row's chart: its LDS copy when it is small, else global memory (generic pointers either way)
    const RowChart rc = a.rows[row];
    const uint32_t *g_so = a.set_off + rc.set_base;
    const uint2 *g_it = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
    const uint32_t *g_ent = a.entries + rc.ent_base;
    const bool base_fits = rc.n_sets <= BASE_SETS_LDS && rc.n_items <= BASE_ITEMS_LDS;   // both limits are below the block size
    const bool ent_fits = rc.n_ent <= AUT_ENT_LDS;
    uint32_t so_v = 0, ent_v = 0;
    uint2 it_v = make_uint2(0, 0);
    if (base_fits && tid <= rc.n_sets) so_v = g_so[tid];
    if (base_fits && tid < rc.n_items) it_v = g_it[tid];
    if (ent_fits && tid < rc.n_ent) ent_v = g_ent[tid];
    const uint8_t rep_v = tid < A.ncls ? D.cls_rep[tid] : (uint8_t)0;
#define ZF_STAGE_STORE(u) if (tid + (u) * AUT_BLOCK < n16) reinterpret_cast<uint4 *>(smem)[tid + (u) * AUT_BLOCK] = tb##u;
    ZF_STAGE_STORE(0) ZF_STAGE_STORE(1) ZF_STAGE_STORE(2) ZF_STAGE_STORE(3) ZF_STAGE_STORE(4) ZF_STAGE_STORE(5) ZF_STAGE_STORE(6)
#undef ZF_STAGE_STORE
    if (base_fits && tid <= rc.n_sets) l_so[tid] = so_v;
    if (base_fits && tid < rc.n_items) l_it[tid] = it_v;
    if (ent_fits && tid < rc.n_ent) l_ent[tid] = ent_v;
    if (tid < 256) l_rep[tid] = rep_v;
    for (uint32_t k = tid; k < A.states_cap * A.ncls; k += AUT_BLOCK) A.trans[k] = AT_NONE;
    for (uint32_t k = tid; k < A.states_cap; k += AUT_BLOCK) A.hdr[k] = make_uint2(0, 0xFFFFFFFFu);
    for (uint32_t k = tid; k < (uint32_t)AUT_HELP_QUEUE; k += AUT_BLOCK) A.hq[k] = 0;
    if (tid == 0) { A.ctl[0] = 1; A.ctl[1] = 0; A.ctl[4] = 0; A.ctl[5] = 0; }
    const uint32_t *b_ent = ent_fits ? l_ent : g_ent;
    const uint32_t *b_so = base_fits ? l_so : g_so;
    const uint2 *b_it = base_fits ? l_it : g_it;
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
            aut_mark_dead(T, A, [&](uint32_t i) { return B.it[B.last_lo + i].x; }, B.last_hi - B.last_lo, 0u, lane);
        __syncthreads();
        const uint32_t n_pairs = A.ctl[3];
        // ---- one lane per string through the automaton, 64 neighbouring ranks at a time ----
        for (;;) {
            uint32_t b = 0;
            if (lane == 0) b = atomicAdd(&A.ctl[2], 1u);
            b = (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
            if (b >= n_pairs) break;
            const uint32_t pair = pairs[b];
            const uint32_t rank = word_of(2 * pair) * 32u + lane;            // a pair lies inside one group: consecutive ranks
            bool live = (cslice[2 * pair + (lane >> 5)] >> (lane & 31u)) & 1u;
            uint32_t soff = 0, len = 0;
            Str16 c16{{0, 0, 0, 0}};
            if (live) { soff = D.str_off[rank]; len = D.str_off[rank + 1] - soff; c16 = D.str16[rank]; }
            live = live && len > 0;
            uint32_t s = 0, pos = 0, c = 0, spins = 0;
            bool ok = false, fail = false;
            for (;;) {
                while (live) {                               // every lane follows its own string as far as the table goes
                    if (pos < 16u) {
                        const uint32_t q = pos >> 2;
                        const uint32_t word = q == 0 ? c16.w[0] : (q == 1 ? c16.w[1] : (q == 2 ? c16.w[2] : c16.w[3]));
                        c = (word >> ((pos & 3u) * 8u)) & 0xFFu;
                    } else c = D.str_cls[soff + pos];
                    const uint32_t t = lds_load(&A.trans[s * A.ncls + c]);
                    if (t < AT_FAIL) { s = t; pos++; if (pos == len) { ok = true; live = false; } }
                    else if (t == AT_DEAD) live = false;
                    else if (t == AT_SINK) { ok = pos + 1 == len; live = false; }
                    else if (t == AT_FAIL) { fail = true; live = false; }
                    else break;                              // not there yet
                }
                const unsigned long long pend = __ballot(live);
                if (!pend) break;
                // Claim the missing transitions that nobody is computing yet: the first one is computed here,
                // the others are left in the help queue for wavefronts that have nothing to do.
                unsigned long long m = pend;
                bool progress = false, mine = false;
                uint32_t ms = 0, mc = 0;
                while (m) {
                    const int l = __ffsll((long long)m) - 1;
                    const uint32_t ls = __builtin_amdgcn_readlane(s, l), lc = __builtin_amdgcn_readlane(c, l);
                    m &= ~__ballot(live && s == ls && c == lc);
                    uint32_t *slot = &A.trans[ls * A.ncls + lc];
                    uint32_t old = 0;
                    if (lane == 0) {
                        bool room = true;
                        uint32_t at = 0;
                        if (mine) { at = atomicAdd(&A.ctl[4], 1u); room = at < (uint32_t)AUT_HELP_QUEUE; }   // a place in the queue first ...
                        old = room ? atomicCAS(slot, (uint32_t)AT_NONE, (uint32_t)AT_BUSY) : (uint32_t)AT_BUSY;
                        // ... which is filled in any case: with the request, or with one that is already settled (takers find it done)
                        if (mine && room) lds_store(&A.hq[at], HQ_VALID | (old == AT_NONE ? (ls << 8) | lc : 0x7FFFFF00u));
                    }
                    old = (uint32_t)__builtin_amdgcn_readfirstlane((int)old);
                    if (old == AT_NONE) {
                        if (!mine) { mine = true; ms = ls; mc = lc; }
                        progress = true;
                    } else if (old != AT_BUSY) progress = true;      // it has just been published
                }
                if (mine) { aut_resolve(T, B, A, sc_w, sc_o, sc_cap, ms, mc, lane); steps++; }
                if (!progress && !aut_help(T, B, A, sc_w, sc_o, sc_cap, lane, steps)) {   // everything this wavefront waits for is being computed by others
                    __builtin_amdgcn_s_sleep(4);
                    if (++spins > (uint32_t)AUT_SPIN_LIMIT) { fail = fail || live; live = false; }   // bounded wait: hand the strings to the fallback
                }
            }
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
        // out of strings: serve the help queue until every batch of the block is finished
        for (uint32_t idle = 0; (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load(&A.ctl[6])) < n_pairs && idle < (uint32_t)AUT_SPIN_LIMIT;) {
            if (aut_help(T, B, A, sc_w, sc_o, sc_cap, lane, steps)) idle = 0;
            else { __builtin_amdgcn_s_sleep(4); idle++; }
        }
        while (aut_help(T, B, A, sc_w, sc_o, sc_cap, lane, steps)) {}       // nothing may stay marked as being computed
        __syncthreads();
        if (tid < AUT_SUB_WORDS) { const uint32_t w = word_of(tid); if (w < Wr) a.rank_mask[(size_t)row * Wr + w] = vslice[tid]; }
    }
    if (lane == 0 && steps) atomicAdd(&a.counters[3], steps);
}

// Verdicts are produced in trie order; the caller wants bit v at word v >> 5.  One lane per
// token looks its bit up and a wavefront ballot packs 64 of them into two words.
__global__ __launch_bounds__(256) void permute_kernel(MaskArgs a) {
    const DeviceTables &D = a.tab;
    const uint32_t v = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y;
    if (a.handoff_in_permute && v < 4 && row == 0) {  // the last kernel of the call: hand the counters to the host, clear the next call's set
        a.host_status[v] = a.counters[v];
        a.counters_next[v] = 0;
    }
    uint32_t bit = 0;
    if (v < (uint32_t)D.V) {
        const uint32_t r = D.rank_of[v];
        if (r != 0xFFFFFFFFu) bit = (a.rank_mask[(size_t)row * D.Wr + (r >> 5)] >> (r & 31)) & 1u;
    }
    const unsigned long long b = __ballot(bit);
    const uint32_t lane = threadIdx.x & 63;
    if ((lane & 31) == 0) {
        const uint32_t w = v >> 5;
        if (w < (uint32_t)D.W) a.out_mask[(size_t)a.dst_row[row] * D.W + w] = (uint32_t)(b >> lane);
    }
}

// State cache (Section 5.2): copy every row's finished mask from its pool slot to the caller's
// tensor.  When the cache is on this is the call's last kernel.
__global__ __launch_bounds__(256) void gather_kernel(MaskArgs a) {
    const uint32_t w = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y, W = (uint32_t)a.tab.W;
    if (w < 4 && row == 0) {
        a.host_status[w] = a.counters[w];
        a.counters_next[w] = 0;
    }
    if (w < W) a.user_mask[(size_t)row * W + w] = a.out_mask[(size_t)a.row_slot[row] * W + w];
}

// Logit masking (Section 3.3): pure copy-or-(-inf).  16-byte accesses, consecutive lanes on
// consecutive 16-byte pieces; the mask words come from L2.
static const int APPLY_UNROLL = 4;   // 16-byte pieces per thread
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <typename VecT, int EPV /* elements per 16 bytes */, typename ElemT>
__global__ __launch_bounds__(256) void apply_mask_vec_kernel(const ElemT *__restrict__ in, ElemT *__restrict__ out, int64_t stride,
                                                             int V, int W, const uint32_t *__restrict__ mask, ElemT neg_inf) {
    const int row = blockIdx.y;
    const ElemT *src = in + (size_t)row * stride;
    ElemT *dst = out + (size_t)row * stride;
    const uint32_t *mrow = mask + (size_t)row * W;
    const int n_vec = V / EPV;
    // a block covers APPLY_UNROLL * 256 consecutive pieces: all loads of a thread are issued before its first store
    const int g0 = blockIdx.x * (256 * APPLY_UNROLL) + threadIdx.x;
    VecT x[APPLY_UNROLL];
#pragma unroll
    for (int u = 0; u < APPLY_UNROLL; u++) {
        const int g = g0 + u * 256;
        if (g < n_vec) x[u] = __builtin_nontemporal_load(reinterpret_cast<const VecT *>(src) + g);
    }
#pragma unroll
    for (int u = 0; u < APPLY_UNROLL; u++) {
        const int g = g0 + u * 256;
        if (g >= n_vec) break;
        const int v0 = g * EPV;
        const uint32_t mb = mrow[v0 >> 5] >> (v0 & 31);
        ElemT *e = reinterpret_cast<ElemT *>(&x[u]);
#pragma unroll
        for (int k = 0; k < EPV; k++) if (!((mb >> k) & 1u)) e[k] = neg_inf;
        __builtin_nontemporal_store(x[u], reinterpret_cast<VecT *>(dst) + g);
    }
    // ragged tail of the row
    const int t = n_vec * EPV + blockIdx.x * 256 + threadIdx.x;
    if (t < V && blockIdx.x * 256 + threadIdx.x < EPV) {
        const bool keep = (mrow[t >> 5] >> (t & 31)) & 1u;
        dst[t] = keep ? src[t] : neg_inf;
    }
}

template <typename ElemT>
__global__ __launch_bounds__(256) void apply_mask_scalar_kernel(const ElemT *__restrict__ in, ElemT *__restrict__ out, int64_t stride,
                                                                int V, int W, const uint32_t *__restrict__ mask, ElemT neg_inf) {
    const int row = blockIdx.y;
    for (int v = blockIdx.x * 256 + threadIdx.x; v < V; v += gridDim.x * 256) {
        const bool keep = (mask[(size_t)row * W + (v >> 5)] >> (v & 31)) & 1u;
        out[(size_t)row * stride + v] = keep ? in[(size_t)row * stride + v] : neg_inf;
    }
}

uint32_t table_bytes(const DeviceTables &t, int mode) {
    uint32_t n = 0;
    if (mode <= 1) for (int k = 0; k < 5; k++) n += t.small_bytes[k];
    if (mode == 0) for (int k = 0; k < 3; k++) n += t.big_bytes[k];
    return n;
}

}  // namespace

int choose_table_mode(const DeviceTables &t) {
    if (table_bytes(t, 0) <= (uint32_t)TABLE_LDS_BUDGET) return 0;
    if (table_bytes(t, 1) <= (uint32_t)TABLE_LDS_BUDGET) return 1;
    return 2;
}

hipError_t prepare_kernels() {
    const int max_lds = 160 * 1024;
    hipError_t e;
#define SET_ATTR(k) if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k), hipFuncAttributeMaxDynamicSharedMemorySize, max_lds)) != hipSuccess) return e
    SET_ATTR(mask_walk_kernel<0>); SET_ATTR(mask_walk_kernel<1>); SET_ATTR(mask_walk_kernel<2>);
    SET_ATTR(mask_automaton_kernel<0>); SET_ATTR(mask_automaton_kernel<1>); SET_ATTR(mask_automaton_kernel<2>);
#undef SET_ATTR
    return hipSuccess;
}

hipError_t launch_upload(const void *pinned_src, void *dst, size_t bytes, hipStream_t s) {
    const uint32_t n16 = (uint32_t)((bytes + 15) / 16);
    hipLaunchKernelGGL(upload_kernel, dim3((n16 + 255) / 256), dim3(256), 0, s, (const uint4 *)pinned_src, (uint4 *)dst, n16);
    return hipGetLastError();
}
hipError_t launch_cache_merge(const MaskArgs &a, hipStream_t s) {
    dim3 grid(((a.tab.Wr + 1) / 2 + 255) / 256, a.batch);
    hipLaunchKernelGGL(cache_merge_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}
uint32_t walk_lds_bytes(const DeviceTables &t, int mode, int lane_cap) {
    return table_bytes(t, mode) + 16 + WALK_WAVES * wave_region_bytes((uint32_t)lane_cap);
}
// Blocks of the walk kernel one compute unit holds at once (registers and LDS both limit it): the
// persistent grid must not be larger, or the surplus blocks would start only after others finish.
hipError_t walk_blocks_per_cu(int mode, uint32_t lds_bytes, int *out) {
    int n = 0;
    hipError_t e;
    if (mode == 0) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_walk_kernel<0>, WALK_BLOCK, lds_bytes);
    else if (mode == 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_walk_kernel<1>, WALK_BLOCK, lds_bytes);
    else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_walk_kernel<2>, WALK_BLOCK, lds_bytes);
    *out = n < 1 ? 1 : n;
    return e;
}
hipError_t launch_mask_walk(const MaskArgs &a, hipStream_t s) {
    const uint32_t lds = walk_lds_bytes(a.tab, a.mode, a.lane_cap);
    dim3 grid(a.walk_blocks);
    if (a.mode == 0) hipLaunchKernelGGL(mask_walk_kernel<0>, grid, dim3(WALK_BLOCK), lds, s, a);
    else if (a.mode == 1) hipLaunchKernelGGL(mask_walk_kernel<1>, grid, dim3(WALK_BLOCK), lds, s, a);
    else hipLaunchKernelGGL(mask_walk_kernel<2>, grid, dim3(WALK_BLOCK), lds, s, a);
    return hipGetLastError();
}
uint32_t automaton_lds_bytes(const DeviceTables &t, int mode, int states, int arena, int scratch) {
    return table_bytes(t, mode) + aut_round16((uint32_t)states * (uint32_t)t.n_cls * 4) + aut_round16((uint32_t)states * 8) + aut_round16((uint32_t)states * 4) + 32 + AUT_HELP_QUEUE * 4 +
           aut_round16((BASE_SETS_LDS + 1) * 4) + BASE_ITEMS_LDS * 8 + AUT_ENT_LDS * 4 + 256 + 2 * AUT_SUB_WORDS * 4 + AUT_SUB_WORDS / 2 + aut_round16((uint32_t)arena * 8) +
           AUT_WAVES * (uint32_t)scratch * 8;
}
hipError_t launch_mask_automaton(const MaskArgs &a, hipStream_t s) {
    const uint32_t lds = automaton_lds_bytes(a.tab, a.mode, a.aut_states, a.aut_arena, a.aut_scratch);
    dim3 grid(a.aut_parts, a.batch);
    if (a.mode == 0) hipLaunchKernelGGL(mask_automaton_kernel<0>, grid, dim3(AUT_BLOCK), lds, s, a);
    else if (a.mode == 1) hipLaunchKernelGGL(mask_automaton_kernel<1>, grid, dim3(AUT_BLOCK), lds, s, a);
    else hipLaunchKernelGGL(mask_automaton_kernel<2>, grid, dim3(AUT_BLOCK), lds, s, a);
    return hipGetLastError();
}
hipError_t launch_mask_fallback(const MaskArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(mask_fallback_kernel, dim3(FB_WAVES), dim3(64), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_permute(const MaskArgs &a, hipStream_t s) {
    dim3 grid((a.tab.V + 255) / 256, a.batch);
    hipLaunchKernelGGL(permute_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gather(const MaskArgs &a, hipStream_t s) {
    dim3 grid((a.tab.W + 255) / 256 > 0 ? (a.tab.W + 255) / 256 : 1, a.user_batch);
    hipLaunchKernelGGL(gather_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_apply_mask(const void *logits, void *out, int dtype, int batch, int64_t row_stride, int V, int W,
                             const uint32_t *mask, hipStream_t s) {
    const size_t esz = dtype == 0 ? 4 : 2;
    const bool aligned = ((uintptr_t)logits % 16 == 0) && ((uintptr_t)out % 16 == 0) && ((row_stride * esz) % 16 == 0);
    const int epv = (int)(16 / esz);
    int blocks_x = aligned ? (V / epv + 256 * APPLY_UNROLL - 1) / (256 * APPLY_UNROLL) : (V + 255) / 256;
    if (blocks_x < 1) blocks_x = 1;
    dim3 grid(blocks_x, batch);
    if (dtype == 0) {
        const uint32_t ninf = 0xFF800000u;
        if (aligned) hipLaunchKernelGGL((apply_mask_vec_kernel<u32x4, 4, uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)logits, (uint32_t *)out, row_stride, V, W, mask, ninf);
        else hipLaunchKernelGGL((apply_mask_scalar_kernel<uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)logits, (uint32_t *)out, row_stride, V, W, mask, ninf);
    } else {
        const uint16_t ninf = 0xFF80u;
        if (aligned) hipLaunchKernelGGL((apply_mask_vec_kernel<u32x4, 8, uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)logits, (uint16_t *)out, row_stride, V, W, mask, ninf);
        else hipLaunchKernelGGL((apply_mask_scalar_kernel<uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)logits, (uint16_t *)out, row_stride, V, W, mask, ninf);
    }
    return hipGetLastError();
}

}  // namespace zf
