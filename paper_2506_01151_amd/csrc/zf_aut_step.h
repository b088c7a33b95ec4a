// The wavefront-cooperative Earley byte step (Scan + Complete with tabulated Predict, Section 3.2) that the
// mask automata are built with, in two variants, and the settling of a new state's dead transitions.  The
// functions are templates over a "sets view" S: S.view(ref, h, n) resolves an origin reference to a handle of
// the set it names (a 64-bit word: lanes pass it round by shuffle) and its item count, S.item(h, i) reads item
// i of that set -- so the same step serves an automaton that lives in one block's LDS, one that lives in
// device memory and is kept from call to call, and the item list of a wavefront that walks the vocabulary trie.
#pragma once
#include "zf_kernel_common.h"

namespace zf {
namespace {

static const uint32_t AUT_REF = 0x80000000u;
enum : uint32_t { AT_NONE = 0xFFFFFFFFu,   // not computed yet
                  AT_DEAD = 0xFFFFFFFEu,   // the byte leaves no item
                  AT_SINK = 0xFFFFFFFDu,   // only completed items: the string may end here, nothing can follow
                  AT_BUSY = 0xFFFFFFFCu,   // a wavefront is computing it
                  AT_FAIL = 0xFFFFFFFBu }; // does not fit this block's budgets: such strings go to the fallback pass

__device__ __forceinline__ uint32_t lds_load(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
__device__ __forceinline__ void lds_store(uint32_t *p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }

// One Earley byte step from state s on byte class cl is done by a whole wavefront with uniform
// control flow (all lanes call these functions with identical arguments).  Both variants leave the
// new set, completed items dropped, in the wavefront's scratch (sc_w, sc_o) and return AUT_OK,
// AUT_WIDE (narrow variant only: more than 64 new items, or too many candidates) or AUT_OVER (no room).
enum { AUT_OK = 0, AUT_WIDE = 1, AUT_OVER = 2 };
static const int AUT_NARROW_TRIES = 96;   // insert attempts after which the narrow variant hands the step to the wide one

// Narrow variant: the set under construction lives in registers (lane j holds new item j), so the
// duplicate test is one compare + ballot; the source set is read in strips of 64 items.  With ONE_STRIP a
// source set of more than 64 items is handed to the wide step at once (AUT_WIDE), which saves the strip
// loop's registers in a kernel that is short of them.
template <bool WIDE, bool ONE_STRIP = false, class SetsT>
__device__ __forceinline__ int aut_step_narrow(const TV &T, const SetsT &S, uint32_t *sc_w, uint32_t *sc_o, uint32_t sc_cap,
                                               uint32_t cur, uint32_t byte, uint32_t cl, uint32_t lane, uint32_t &nnew_out, uint32_t &kept_out) {
    uint64_t src;
    uint32_t ns;
    S.view(cur, src, ns);
    if (ONE_STRIP && ns > 64u) return AUT_WIDE;
    uint32_t nw = 0xFFFFFFFFu, no = 0, nnew = 0, tries = 0;  // no item word is all ones
    bool saw_end = false, failed = false;                    // failed is sticky: the step runs on and reports at its end
    const uint32_t room = sc_cap < 64u ? sc_cap : 64u;
    auto insert = [&](uint32_t w, uint32_t o) {              // uniform arguments; no branch
        tries++;
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
        if (s0 + lane < ns) { const uint2 x = S.item(src, s0 + lane); sw = x.x; so = x.y; }
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
        if (ONE_STRIP) break;
    }
    if (saw_end) {
        // Complete: new items are visited in order; completing may append more
        unsigned long long visited = 0;
        for (;;) {
            const unsigned long long todo = __ballot(lane < nnew && (nw & IW_END)) & ~visited;
            if (!todo) break;
            if (WIDE && tries > (uint32_t)AUT_NARROW_TRIES) return AUT_WIDE;   // candidates come one at a time here: an ambiguous grammar makes hundreds, mostly duplicates
            const int i = __ffsll((long long)todo) - 1;
            visited |= 1ull << i;
            const uint32_t w = __builtin_amdgcn_readlane(nw, i);
            const uint32_t X = (w & IW_POS_MASK) - T.end_base;
            if (X == T.N - 1) continue;                      // the start rule is complete: the prefix is a sentence
            const uint32_t o = __builtin_amdgcn_readlane(no, i);
            uint64_t yp;
            uint32_t yn;
            S.view(o, yp, yn);
            for (uint32_t j0 = 0; j0 < yn; j0 += 64) {
                uint32_t yw = IW_END, yo = 0;
                if (j0 + lane < yn) { const uint2 y = S.item(yp, j0 + lane); yw = y.x; yo = y.y; }
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
// in the scratch, with an open-addressing hash table over it (sc_h: 0 = free, else item index + 1;
// at least twice as many places as items).  The lanes make candidates in parallel -- one source
// item per lane in Scan, one waiting item of the completed nonterminal's origin set per lane in
// Complete -- and 64 candidates are entered at a time.  The order of the new set is fixed by strip,
// round and lane number, so the same source set always yields the same sequence of items.
__host__ __device__ inline uint32_t aut_hash_places(uint32_t sc_cap) {
    uint32_t n = 64;
    while (n < 2 * sc_cap) n <<= 1;
    return n;
}
template <class SetsT>
__device__ __forceinline__ int aut_step_wide(const TV &T, const SetsT &S, uint32_t *sc_w, uint32_t *sc_o, uint32_t *sc_h, uint32_t sc_cap,
                                             uint32_t cur, uint32_t byte, uint32_t cl, uint32_t lane, uint32_t &nnew_out, uint32_t &kept_out) {
    uint64_t src;
    uint32_t ns;
    S.view(cur, src, ns);
    const uint32_t places = aut_hash_places(sc_cap), pmask = places - 1u;
    for (uint32_t k = lane; k < places; k += 64) lds_store(&sc_h[k], 0u);
    uint32_t nnew = 0;
    bool saw_end = false, failed = false;
    const unsigned long long below = (1ull << lane) - 1ull;
    auto insert = [&](bool has, uint32_t w, uint32_t o) {    // per-lane arguments: every lane with `has` brings a candidate
        if (failed || !__ballot(has)) return;
        uint32_t h = (w * 0x9E3779B1u) ^ (o * 0x85EBCA77u);
        h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 13;
        uint32_t slot = h & pmask;
        bool fresh = has;
        while (fresh) {                                      // in the set already?  (the table always has free places: the probe ends)
            const uint32_t v = lds_load(&sc_h[slot]);
            if (v == 0u) break;
            if (lds_load(&sc_w[v - 1u]) == w && lds_load(&sc_o[v - 1u]) == o) fresh = false;
            else slot = (slot + 1u) & pmask;
        }
        unsigned long long f = __ballot(fresh);
        if (__popcll(f) > 1) {                               // the same candidate on several lanes: the lowest lane keeps it
            unsigned long long todo = f;
            while (todo) {
                const int l = __ffsll((long long)todo) - 1;
                const uint32_t lw = __builtin_amdgcn_readlane(w, l), lo = __builtin_amdgcn_readlane(o, l);
                const bool same = fresh && w == lw && o == lo;           // lane l itself included
                todo &= ~__ballot(same);
                if (same && lane != (uint32_t)l) fresh = false;
            }
            f = __ballot(fresh);
        }
        const uint32_t n_f = (uint32_t)__popcll(f);
        if (n_f > sc_cap - nnew) { failed = true; return; }
        if (fresh) {                                         // places in lane order; then into the table (distinct keys: any order will do)
            const uint32_t idx = nnew + (uint32_t)__popcll(f & below);
            lds_store(&sc_w[idx], w);
            lds_store(&sc_o[idx], o);
            while (atomicCAS(&sc_h[slot], 0u, idx + 1u) != 0u) slot = (slot + 1u) & pmask;
        }
        nnew += n_f;
        saw_end = saw_end || __ballot(fresh && (w & IW_END)) != 0;
    };
    auto chain = [&](bool on, uint32_t p, uint32_t o) {     // per lane: the dot arrives at p; skip nullable nonterminals, canonical END item
        while (__ballot(on)) {
            uint32_t w = 0;
            if (on) w = T.advpq[p];
            insert(on, w, o);
            on = on && !(w & (IW_END | IW_TERM)) && (w & IW_NT_NULLABLE);
            p++;
        }
    };
    for (uint32_t s0 = 0; s0 < ns && !failed; s0 += 64) {
        uint32_t sw = IW_END, so = 0;                        // lanes beyond the set hold an inert item
        if (s0 + lane < ns) { const uint2 x = S.item(src, s0 + lane); sw = x.x; so = x.y; }
        // Scan, terminal items
        uint32_t nx = DFA_DEAD;
        if (sw & IW_TERM) nx = dfa_next(T, sw >> 16, byte, cl);
        const bool hit = (nx & 0xFFFFu) != DFA_DEAD;
        insert(hit && ((nx >> 16) & QF_CONT), (sw & 0xFFFFu) | (nx << 16), so);        // no longest match: keep matching ...
        chain(hit && ((nx >> 16) & QF_ACCEPT), (sw & IW_POS_MASK) + 1, so);             // ... and also finish here
        // Scan, items that wait for a nonterminal Y: the tabulated first steps of every terminal that can begin Y
        uint32_t sk0 = 0, sk1 = 0;
        if (!(sw & (IW_TERM | IW_END))) {
            const uint32_t Y = (sw >> IW_NT_SHIFT) & IW_NT_MASK;
            sk0 = T.scan_off[Y * T.ncls + cl]; sk1 = T.scan_off[Y * T.ncls + cl + 1];
        }
        while (__ballot(sk0 < sk1)) {
            const bool on = sk0 < sk1;
            uint2 ef = make_uint2(0, 0);
            if (on) ef = T.scan_list[sk0];
            insert(on && (ef.y & QF_CONT), ef.x, cur);
            chain(on && (ef.y & QF_ACCEPT), (ef.x & IW_POS_MASK) + 1, cur);
            if (on) sk0++;
        }
    }
    if (saw_end) {
        // Complete: the new items are visited in order, up to 64 at a time (completing appends more).  The
        // completed items of a strip sit on their lanes; the items of their origin sets -- the ones that
        // may wait for the completed nonterminal -- are numbered through and dealt to the lanes 64 at
        // a time, so that short origin sets (a pruned chart's sets hold a handful of items) still fill the wavefront.
        uint32_t done = 0;
        while (done < nnew && !failed) {
            const uint32_t hi = nnew - done < 64u ? nnew : done + 64u;
            uint32_t w = 0, o = 0;
            if (done + lane < hi) { w = lds_load(&sc_w[done + lane]); o = lds_load(&sc_o[done + lane]); }
            const uint32_t X = (w & IW_POS_MASK) - T.end_base;
            const bool is_end = (w & IW_END) && X != T.N - 1;                  // the start rule complete: the prefix is a sentence
            uint64_t yp = 0;
            uint32_t yn = 0;
            if (is_end) S.view(o, yp, yn);
            uint32_t incl = yn;                                                // running total of the origin sets' sizes
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) { const uint32_t up = __shfl_up(incl, d); if (lane >= (uint32_t)d) incl += up; }
            const uint32_t excl = incl - yn, total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            const uint32_t yp_lo = (uint32_t)yp, yp_hi = (uint32_t)(yp >> 32);
            unsigned long long owners = __ballot(yn > 0);                      // lanes whose origin set is not dealt out yet
            for (uint32_t t0 = 0; t0 < total && !failed; t0 += 64) {
                const uint32_t t = t0 + lane;
                uint32_t own = 0;
                for (unsigned long long scan = owners; scan;) {                // ranges come in lane order: walk the ones that reach into this strip
                    const int e = __ffsll((long long)scan) - 1;
                    scan &= scan - 1;
                    const uint32_t e_lo = __builtin_amdgcn_readlane((int)excl, e), e_hi = __builtin_amdgcn_readlane((int)incl, e);
                    if (e_lo >= t0 + 64u) break;
                    if (t >= e_lo && t < e_hi) own = (uint32_t)e;
                    if (e_hi <= t0 + 64u) owners &= ~(1ull << e);
                }
                const uint32_t oX = __shfl(X, own), oo = __shfl(o, own), o_lo = __shfl(excl, own);
                const uint64_t oyp = (uint64_t)(uint32_t)__shfl(yp_lo, own) | ((uint64_t)(uint32_t)__shfl(yp_hi, own) << 32);
                uint32_t yw = IW_END, yo = 0;
                if (t < total) { const uint2 y = S.item(oyp, t - o_lo); yw = y.x; yo = y.y; }
                const bool nt = !(yw & (IW_TERM | IW_END));
                const uint32_t Y = (yw >> IW_NT_SHIFT) & IW_NT_MASK;
                uint32_t c0 = 0, c1 = 0;
                if (nt) { c0 = T.comp_off[Y * T.N + oX]; c1 = T.comp_off[Y * T.N + oX + 1]; }
                while (__ballot(c0 < c1)) {
                    const bool on = c0 < c1;
                    uint32_t cw = 0;
                    if (on) cw = T.comp_list[c0];
                    const bool self = on && cw == 0xFFFFFFFFu;                 // Y itself is complete: the waiting item moves on
                    insert(on && !self, cw, oo);
                    chain(self, (yw & IW_POS_MASK) + 1, yo);
                    if (on) c0++;
                }
            }
            done = hi;
        }
    }
    if (failed) return AUT_OVER;
    // drop the completed items: forward compaction, strip by strip (a strip is read before it is written)
    uint32_t kept = 0;
    for (uint32_t s0 = 0; s0 < nnew; s0 += 64) {
        uint32_t w = IW_END, o = 0;
        if (s0 + lane < nnew) { w = lds_load(&sc_w[s0 + lane]); o = lds_load(&sc_o[s0 + lane]); }
        const bool keep = !(w & IW_END);
        const unsigned long long kb = __ballot(keep);
        if (keep) { const uint32_t at = kept + (uint32_t)__popcll(kb & below); lds_store(&sc_w[at], w); lds_store(&sc_o[at], o); }
        kept += (uint32_t)__popcll(kb);
    }
    nnew_out = nnew;
    kept_out = kept;
    return AUT_OK;
}

// Transitions of state `id` that leave no item at all are settled when the state is made, for all
// byte classes at once (lane = class): an item before a terminal survives a class iff its DFA has
// an edge, an item that waits for a nonterminal iff some terminal that can begin it has one.  What
// remains for the byte step proper are the few classes that lead somewhere.
// item(i): the item word of the state's i-th item; rep[c]: one byte of class c; dead(c): called by one lane for every class that leaves no item.
template <bool WIDE, class ItemWord, class Dead>
__device__ __forceinline__ void aut_mark_dead(const TV &T, uint32_t ncls, const uint8_t *rep, ItemWord item, uint32_t n, uint32_t lane, Dead dead) {
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
    if (WIDE && n > 16u) {                                   // a wide set: one item per lane, the classes in turn
        for (uint32_t c0 = 0; c0 < ncls; c0 += 64) {
            const uint32_t nc = ncls - c0 < 64u ? ncls - c0 : 64u;
            uint32_t lo = 0, hi = 0;                         // bit k: some item of this lane survives class c0 + k
            for (uint32_t i0 = 0; i0 < n; i0 += 64) {
                const uint32_t w = i0 + lane < n ? item(i0 + lane) : (uint32_t)IW_END;
                for (uint32_t k = 0; k < nc; k++) {
                    const bool al = survives(w, rep[c0 + k], c0 + k);
                    lo |= (al && k < 32u) ? 1u << (k & 31u) : 0u;
                    hi |= (al && k >= 32u) ? 1u << (k & 31u) : 0u;
                }
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) { lo |= __shfl_xor(lo, d); hi |= __shfl_xor(hi, d); }
            const uint32_t mine = lane < 32u ? lo >> lane : hi >> (lane - 32u);
            if (lane < nc && !(mine & 1u)) dead(c0 + lane);
        }
        return;
    }
    for (uint32_t c0 = 0; c0 < ncls; c0 += 64) {
        const uint32_t c = c0 + lane < ncls ? c0 + lane : ncls - 1;   // surplus lanes repeat the last class
        const uint32_t byte = rep[c];
        bool alive = false;
        for (uint32_t i = 0; i < n; i += 4) {                // four items at a time: their look-ups are independent of each other
            const uint32_t w0 = item(i), w1 = i + 1 < n ? item(i + 1) : (uint32_t)IW_END, w2 = i + 2 < n ? item(i + 2) : (uint32_t)IW_END,
                           w3 = i + 3 < n ? item(i + 3) : (uint32_t)IW_END;
            const bool a0 = survives(w0, byte, c), a1 = survives(w1, byte, c), a2 = survives(w2, byte, c), a3 = survives(w3, byte, c);
            alive |= a0 | a1 | a2 | a3;
        }
        if (!alive) dead(c);
    }
}

}  // namespace
}  // namespace zf
