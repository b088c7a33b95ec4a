// Host twin of the mask-automaton kernel.
//
// The per-token check (Section 4.1: every vocabulary token at every step) feeds a token's bytes
// into the recognizer one at a time.  The set reached after a byte is a function of the set it
// came from, of the sets that set's items point back to, and of the byte's equivalence class --
// not of the token.  So the Earley sets met while checking one row's tokens form a deterministic
// automaton over byte classes, and that automaton is small: a pruned chart (Section 4.2) keeps
// few items, terminals loop in place, and thousands of tokens share the same few parser moves.
// The automaton is built lazily: a transition is computed with one Earley byte step (Scan +
// Complete, Section 3.2) the first time some token needs it and looked up from then on; sets are
// interned by content, so "the same set again" is the same state (a digit inside a number, a
// letter inside a string: self loops).  This is the state-cache idea of Section 5.2 applied
// inside one mask computation.
//
// A state's item is (dotted position, DFA state, origin reference).  An origin reference names
// the set the item's rule started in: a set of the row's chart (index < number of chart sets) or
// another automaton state (AUT_REF | id).  The root state is the row's current set.
#include <algorithm>
#include <cstring>
#include <map>
#include "zf_internal.h"
#include "zf_host_automaton.h"

namespace zf {
namespace {

const uint32_t AUT_REF = 0x80000000u;
enum : uint32_t { T_NONE = 0xFFFFFFFFu, T_DEAD = 0xFFFFFFFEu, T_SINK = 0xFFFFFFFDu };   // SINK: alive, nothing left to extend

struct Automaton {
    const Tables &t;
    const Chart &base;
    uint32_t m0;
    std::vector<std::vector<Item>> sets;          // state id -> items (origin = reference); state 0 = root (items unused)
    std::vector<std::vector<uint32_t>> trans;     // state id -> [n_cls]
    std::map<std::vector<uint32_t>, uint32_t> interned;
    int64_t n_steps = 0, n_lookups = 0, max_set = 0;

    Automaton(const Tables &t_, const Chart &c) : t(t_), base(c), m0(c.n_sets()) {
        sets.emplace_back();
        trans.emplace_back(t.n_cls, T_NONE);
    }

    void closure(uint32_t s, std::vector<uint32_t> &ids) const {   // states reachable through origin references, s included
        if (s == 0 || std::find(ids.begin(), ids.end(), s) != ids.end()) return;
        ids.push_back(s);
        for (const Item &it : sets[s]) if (it.o & AUT_REF) closure(it.o & ~AUT_REF, ids);
    }

    uint32_t compute(uint32_t s, uint8_t byte) {
        // lay the sets this step may read out as a chart: the row's sets, then the referenced states, s last
        Chart c = base;
        std::vector<uint32_t> ids;
        closure(s, ids);
        std::sort(ids.begin(), ids.end());           // a state only refers to states that existed before it
        if (s != 0) { ids.erase(std::find(ids.begin(), ids.end(), s)); ids.push_back(s); }
        auto index_of = [&](uint32_t ref) -> uint32_t {
            if (!(ref & AUT_REF)) return ref;
            const uint32_t id = ref & ~AUT_REF;
            if (id == 0) return m0 - 1;
            return m0 + (uint32_t)(std::find(ids.begin(), ids.end(), id) - ids.begin());
        };
        for (uint32_t id : ids) {
            for (Item it : sets[id]) { it.o = index_of(it.o); c.items.push_back(it); }
            c.set_off.push_back((uint32_t)c.items.size());
        }
        const StepResult r = earley_step(t, c, byte, false, nullptr);
        n_steps++;
        if (!r.alive) return T_DEAD;
        if (!r.kernel_nonempty) return T_SINK;
        const uint32_t last = c.n_sets() - 1;
        std::vector<Item> out(c.items.begin() + c.set_off[last], c.items.end());
        std::vector<uint32_t> key;
        for (Item &it : out) {
            if (it.o >= m0) it.o = AUT_REF | ids[it.o - m0];   // the source state itself included: it is the last of ids
            key.push_back((uint32_t)it.p | ((uint32_t)it.q << 16));
            key.push_back(it.o);
        }
        max_set = std::max<int64_t>(max_set, (int64_t)out.size());
        auto found = interned.find(key);
        if (found != interned.end()) return found->second;
        const uint32_t id = (uint32_t)sets.size();
        sets.push_back(out);
        trans.emplace_back(t.n_cls, T_NONE);
        interned.emplace(key, id);
        return id;
    }

    bool accepts(const uint8_t *p, size_t n) {
        uint32_t s = 0;
        for (size_t i = 0; i < n; i++) {
            if (s == T_SINK) return false;
            const int cl = t.cls[p[i]];
            n_lookups++;
            uint32_t to = trans[s][cl];
            if (to == T_NONE) { to = compute(s, p[i]); trans[s][cl] = to; }
            if (to == T_DEAD) return false;
            s = to;
        }
        return true;
    }
};

}  // namespace
}  // namespace zf

using namespace zf;

extern "C" int zf_debug_host_mask_automaton(zf_engine *e, const zf_state *s, uint32_t *mask, int64_t *stats) {
    if (!e || !s || !mask || s->eng != e) { set_error("bad argument"); return ZF_ERR_INVALID_ARG; }
    const Tables &t = e->tab;
    const Trie &tr = e->trie;
    const Chart &c = chart_of(s);
    const uint32_t m0 = c.n_sets();
    // merge the token-mask cache rows of the current set (Section 4.3), as the kernels do
    std::vector<uint32_t> valid(tr.Wr, 0), want(tr.Wr, 0);
    const bool use_cache = !e->opt.disable_token_mask_cache;
    if (!use_cache) want.assign(tr.Wr, 0xFFFFFFFFu);
    else for (uint32_t i = c.set_off[m0 - 1]; i < c.set_off[m0]; i++) {
        const uint16_t code = t.sym[c.items[i].p];
        size_t row;
        if ((code >> SYM_KIND_SHIFT) == SYM_TERM) row = c.items[i].q;
        else if ((code >> SYM_KIND_SHIFT) == SYM_NT) row = (size_t)t.Q + (code & SYM_ID_MASK_NT);
        else continue;
        for (int w = 0; w < tr.Wr; w++) { valid[w] |= tr.ci_valid[row * tr.Wr + w]; want[w] |= tr.ci_cd[row * tr.Wr + w]; }
    }
    for (int w = 0; w < tr.Wr; w++) want[w] &= ~valid[w];
    Automaton a(t, c);
    int64_t n_wanted = 0;
    for (uint32_t r = 0; r < (uint32_t)tr.n_strings; r++) {
        if (!((want[r >> 5] >> (r & 31)) & 1)) continue;
        n_wanted++;
        if (a.accepts(tr.str_bytes.data() + tr.str_off[r], tr.str_off[r + 1] - tr.str_off[r])) valid[r >> 5] |= 1u << (r & 31);
    }
    memset(mask, 0, sizeof(uint32_t) * e->W);
    for (int v = 0; v < e->V; v++) {
        const uint32_t r = tr.rank_of[v];
        if (r != 0xFFFFFFFFu && ((valid[r >> 5] >> (r & 31)) & 1)) mask[v >> 5] |= 1u << (v & 31);
    }
    if (stats) { stats[0] = (int64_t)a.sets.size() - 1; stats[1] = a.n_steps; stats[2] = a.n_lookups; stats[3] = n_wanted; stats[4] = a.max_set; }
    return ZF_OK;
}

// ---- Host twin of the persistent (cross-step) automaton ------------------------------------------
//
// The same observation one level up: when every Earley set is named by its content -- its items,
// each with the NAME of the set its rule started in instead of a position in some row's chart -- the
// sets of all rows and all decode steps are the states of ONE deterministic automaton over byte
// classes.  Feeding a token (Section 4.1, the update after a decoding step) is then a walk of its
// bytes through that automaton from the row's current state, the per-step token check is the same
// walk for every vocabulary string, and a transition is computed by an Earley byte step (Section
// 3.2) once, whichever row or step needs it first; everything later is a look-up (the reuse across
// steps that Sections 4.4 and 5.2 aim at).  A state refers only to the sets its items started in,
// transitively: what ZapFormat's reachability closure (Section 4.2.3) keeps of a chart is exactly
// what a state can reach through these references, and completed items are dropped when a set is
// closed, so nothing here needs a separate Compact pass.
struct zf_twin {
    zf_engine *eng;
    zf::HostAutomaton a;
    explicit zf_twin(zf_engine *e) : eng(e), a(e->tab) {}
};

extern "C" int zf_debug_twin_new(zf_engine *e, zf_twin **out) {
    if (!e || !out) { set_error("null argument"); return ZF_ERR_INVALID_ARG; }
    *out = new zf_twin(e);
    return ZF_OK;
}
extern "C" void zf_debug_twin_destroy(zf_twin *t) { delete t; }

extern "C" int zf_debug_twin_advance(zf_twin *tw, uint32_t *state, const uint8_t *bytes, int64_t n, int32_t *accepting) {
    if (!tw || !state || (n > 0 && !bytes) || n <= 0) { set_error("bad argument"); return ZF_ERR_INVALID_ARG; }
    uint32_t s = *state == 0 ? HostAutomaton::ROOT : *state;
    bool acc = false;
    for (int64_t i = 0; i < n; i++) {
        s = tw->a.step(s, bytes[i], &acc);
        if (s == HostAutomaton::DEAD || (s == HostAutomaton::SINK && i + 1 < n)) { set_error("byte " + std::to_string(i) + " cannot extend the prefix"); return ZF_ERR_REJECTED; }
    }
    *state = s;
    if (accepting) *accepting = acc;
    return ZF_OK;
}

extern "C" int zf_debug_twin_mask(zf_twin *tw, uint32_t state, uint32_t *mask, int64_t *stats) {
    if (!tw || !mask) { set_error("bad argument"); return ZF_ERR_INVALID_ARG; }
    zf_engine *e = tw->eng;
    const Tables &t = e->tab;
    const Trie &tr = e->trie;
    HostAutomaton &a = tw->a;
    const uint32_t root = state == 0 ? HostAutomaton::ROOT : state;
    memset(mask, 0, sizeof(uint32_t) * e->W);
    const int64_t steps0 = a.n_steps;
    int64_t n_wanted = 0, n_lookups = 0;
    if (root != HostAutomaton::SINK) {
        if (root >= a.n_states) { set_error("unknown state"); return ZF_ERR_INVALID_ARG; }
        std::vector<uint32_t> valid(tr.Wr, 0), want(tr.Wr, 0);
        if (e->opt.disable_token_mask_cache) want.assign(tr.Wr, 0xFFFFFFFFu);
        else for (const Item &it : a.st(root).items) {             // the token-mask cache rows of the state's items (Section 4.3)
            const uint16_t code = t.sym[it.p];
            size_t row;
            if ((code >> SYM_KIND_SHIFT) == SYM_TERM) row = it.q;
            else if ((code >> SYM_KIND_SHIFT) == SYM_NT) row = (size_t)t.Q + (code & SYM_ID_MASK_NT);
            else continue;
            for (int w = 0; w < tr.Wr; w++) { valid[w] |= tr.ci_valid[row * tr.Wr + w]; want[w] |= tr.ci_cd[row * tr.Wr + w]; }
        }
        for (int w = 0; w < tr.Wr; w++) want[w] &= ~valid[w];
        for (uint32_t r = 0; r < (uint32_t)tr.n_strings; r++) {
            if (!((want[r >> 5] >> (r & 31)) & 1)) continue;
            n_wanted++;
            uint32_t s = root;
            bool ok = true;
            for (uint32_t k = tr.str_off[r]; k < tr.str_off[r + 1] && ok; k++) {
                n_lookups++;
                s = a.step(s, tr.str_bytes[k], nullptr);
                ok = s != HostAutomaton::DEAD;
            }
            if (ok) valid[r >> 5] |= 1u << (r & 31);
        }
        for (int v = 0; v < e->V; v++) {
            const uint32_t r = tr.rank_of[v];
            if (r != 0xFFFFFFFFu && ((valid[r >> 5] >> (r & 31)) & 1)) mask[v >> 5] |= 1u << (v & 31);
        }
    }
    if (stats) { stats[0] = (int64_t)a.n_states - 1; stats[1] = a.n_steps - steps0; stats[2] = n_lookups; stats[3] = n_wanted; stats[4] = a.n_items; }
    return ZF_OK;
}
