// Host Earley recognizer over the compiled tables: Scan, Complete (with the tabulated
// Predict closure), and the ZapFormat Compact phase (paper Sections 3.2 and 4.2).
#include "zf_internal.h"

namespace zf {
namespace {

inline int kind(uint16_t code) { return code >> SYM_KIND_SHIFT; }

// a set holds each item once (Section 3.2)
inline void insert(Chart &c, uint32_t set_begin, Item it, int64_t *created) {
    for (size_t i = set_begin; i < c.items.size(); i++)
        if (c.items[i].p == it.p && c.items[i].q == it.q && c.items[i].o == it.o) return;
    c.items.push_back(it);
    if (created) ++*created;
}

// Add the item whose dot stands at position p (origin o) to the set under construction.  A
// nullable postdot nonterminal is also skipped; a dot at the end of the rule is recorded as the
// canonical "lhs complete since o" item.
void add_advanced(const Tables &t, Chart &c, uint32_t set_begin, uint32_t p, uint32_t o, int64_t *created) {
    for (;;) {
        uint16_t code = t.sym[p];
        if (kind(code) == SYM_END) { insert(c, set_begin, Item{t.end_pos[code & SYM_ID_MASK], 0, o}, created); return; }
        if (kind(code) == SYM_TERM) { insert(c, set_begin, Item{(uint16_t)p, t.term_start[code & SYM_ID_MASK], o}, created); return; }
        insert(c, set_begin, Item{(uint16_t)p, 0, o}, created);
        if (!(code & SYM_NULLABLE_BIT)) return;
        p++;
    }
}

}  // namespace

void chart_init(const Tables &t, Chart &c) {
    c.items.clear();
    c.set_off.assign(1, 0);
    add_advanced(t, c, 0, (uint32_t)t.start_pos, 0, nullptr);
    c.set_off.push_back((uint32_t)c.items.size());
}

StepResult earley_step(const Tables &t, Chart &c, uint8_t byte, bool keep_completed, int64_t *created) {
    const uint32_t m = c.n_sets(), last = m - 1;
    const uint32_t b = c.set_off[last], e = c.set_off[m];
    const uint32_t nb = (uint32_t)c.items.size();   // == e
    const int cl = t.cls[byte];
    const int SP = t.N - 1;
    StepResult res{false, false, false};
    // Scan: kernel items before a terminal step their DFA; kernel items before a nonterminal Y
    // stand for every predicted item of I(Y), whose first DFA step is tabulated in SCAN(Y, class).
    for (uint32_t i = b; i < e; i++) {
        Item it = c.items[i];
        uint16_t code = t.sym[it.p];
        if (kind(code) == SYM_TERM) {
            uint16_t q2 = t.delta[(size_t)it.q * t.n_cls + cl];
            if (q2 == DFA_DEAD) continue;
            uint8_t f = t.qflags[q2];
            if (f & QF_CONT) insert(c, nb, Item{it.p, q2, it.o}, created);   // no longest-match: keep matching ...
            if (f & QF_ACCEPT) add_advanced(t, c, nb, it.p + 1u, it.o, created);   // ... and also finish here
        } else if (kind(code) == SYM_NT) {
            int Y = code & SYM_ID_MASK_NT;
            for (uint32_t k = t.scan_off[(size_t)Y * t.n_cls + cl]; k < t.scan_off[(size_t)Y * t.n_cls + cl + 1]; k++) {
                uint32_t ent = t.scan_list[k];
                uint16_t p0 = ent & 0xFFFF, q2 = ent >> 16;
                uint8_t f = t.qflags[q2];
                if (f & QF_CONT) insert(c, nb, Item{p0, q2, last}, created);
                if (f & QF_ACCEPT) add_advanced(t, c, nb, p0 + 1u, last, created);
            }
        }
    }
    // Complete: "X complete since o" advances every item of S[o] that waits for X -- the kernel
    // item itself when its postdot symbol is X, and the predicted items of I(Y) that wait for X.
    // COMP(Y, X) already holds the outcome for the predicted items, including the completions
    // of their own left-hand sides that follow at the same origin.
    for (size_t i = nb; i < c.items.size(); i++) {
        Item it = c.items[i];
        uint16_t code = t.sym[it.p];
        if (kind(code) != SYM_END) continue;
        int X = code & SYM_ID_MASK;
        if (X == SP) { res.accepted = true; continue; }
        uint32_t o = it.o;
        for (uint32_t j = c.set_off[o]; j < c.set_off[o + 1]; j++) {
            Item y = c.items[j];
            uint16_t yc = t.sym[y.p];
            if (kind(yc) != SYM_NT) continue;
            int Y = yc & SYM_ID_MASK_NT;
            for (uint32_t k = t.comp_off[(size_t)Y * t.N + X]; k < t.comp_off[(size_t)Y * t.N + X + 1]; k++) {
                const uint16_t p = t.comp_list[k];
                if (p == COMP_ADVANCE_WAITING) add_advanced(t, c, nb, y.p + 1u, y.o, created);   // Y itself is complete since y's set
                else insert(c, nb, Item{p, kind(t.sym[p]) == SYM_TERM ? t.term_start[t.sym[p] & SYM_ID_MASK] : (uint16_t)0, o}, created);
            }
        }
    }
    res.alive = c.items.size() > nb;
    // Completed items only matter while their own set is being processed (Figure 3, first rule).
    size_t w = nb;
    for (size_t i = nb; i < c.items.size(); i++) {
        bool done = kind(t.sym[c.items[i].p]) == SYM_END;
        if (!done) res.kernel_nonempty = true;
        if (!done || keep_completed) c.items[w++] = c.items[i];
    }
    c.items.resize(w);
    c.set_off.push_back((uint32_t)c.items.size());
    return res;
}

// Compact (Section 4.2.3).  The only time Earley reads an earlier set is Complete, which looks
// in S[origin] for items that wait for the completed nonterminal.  So the items still needed are
// those of the last set plus, transitively, for every needed item (X -> ..., o) the items of
// S[o] whose postdot nonterminal can start with X.  Everything else is dropped, sets that become
// empty disappear and origins are renumbered.
void chart_compact(const Tables &t, Chart &c) {
    const uint32_t m = c.n_sets();
    if (m <= 1) return;
    std::vector<uint8_t> mark(c.items.size(), 0);
    std::vector<uint32_t> stack;
    for (uint32_t i = c.set_off[m - 1]; i < c.set_off[m]; i++) { mark[i] = 1; stack.push_back(i); }
    while (!stack.empty()) {
        Item x = c.items[stack.back()];
        stack.pop_back();
        int X = t.lhs_of[x.p];
        for (uint32_t j = c.set_off[x.o]; j < c.set_off[x.o + 1]; j++) {
            if (mark[j]) continue;
            uint16_t yc = t.sym[c.items[j].p];
            if (kind(yc) != SYM_NT) continue;
            if (t.reach[(size_t)(yc & SYM_ID_MASK_NT) * t.N + X]) { mark[j] = 1; stack.push_back(j); }
        }
    }
    std::vector<uint32_t> new_index(m, 0xFFFFFFFFu);
    std::vector<uint32_t> new_off{0};
    size_t w = 0;
    uint32_t n_new = 0;
    for (uint32_t k = 0; k < m; k++) {
        size_t before = w;
        for (uint32_t i = c.set_off[k]; i < c.set_off[k + 1]; i++) if (mark[i]) c.items[w++] = c.items[i];
        if (w > before || k == m - 1) { new_index[k] = n_new++; new_off.push_back((uint32_t)w); }
    }
    c.items.resize(w);
    for (auto &it : c.items) it.o = new_index[it.o];   // a kept item's origin set holds the item it waits in, so it is kept too
    c.set_off.swap(new_off);
}

}  // namespace zf
