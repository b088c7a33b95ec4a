// The persistent automaton on the host: every Earley set named by its content, items carrying the name of the
// set their rule started in, so the sets of all rows and decode steps are the states of one deterministic
// automaton over byte classes (Sections 4.4, 5.2).  zf_advance walks a token's bytes through it (a look-up per
// byte once a transition is known, one Earley byte step -- Scan, Complete, tabulated Predict: Section 3.2 --
// the first time); the diagnostics of include/zapformat_debug.h use a second instance as the twin of the
// device's store.  A state refers only to the sets its items started in, transitively, which is what
// ZapFormat's reachability closure keeps of a chart (Section 4.2.3); completed items are dropped when a set is
// closed (Figure 3, first rule), so no separate Compact pass is needed here.
//
// Sharing.  A state's items never change once the state has a name, and states live in blocks whose addresses
// never change, so a thread that has learnt a name under the owner's lock may read that state's items without
// it (lay_out); everything that writes (record, import, clear) and every look-up of a transition runs under the
// lock.  clear() frees the blocks: the owner calls it only while no thread is between lay_out and record.
#pragma once
#include <algorithm>
#include <map>
#include <memory>
#include "zf_internal.h"

namespace zf {

struct HostAutomaton {
    const Tables &t;
    static constexpr uint32_t ROOT = 1, SINK = 0xFFFFFFFDu, DEAD = 0xFFFFFFFEu, NONE = 0xFFFFFFFFu;
    static constexpr uint32_t BLOCK = 1024, MAX_BLOCKS = 1024;     // at most BLOCK x MAX_BLOCKS states
    struct State {
        std::vector<Item> items;          // an item's origin is a state id
        std::vector<uint32_t> trans;      // [n_cls] next state, NONE, DEAD or SINK
        std::vector<uint8_t> acc;         // [n_cls] the prefix is a sentence after that byte
        uint32_t widest = 0;              // items of the largest set among the state and the sets it refers to
    };
    std::vector<std::unique_ptr<State[]>> blocks;   // room for MAX_BLOCKS pointers from the start: the array never moves
    uint32_t n_states = 0;                // ids 0 .. n_states - 1 are taken (0 is not used)
    std::map<std::vector<uint32_t>, uint32_t> interned;
    int64_t n_steps = 0, n_items = 0;

    explicit HostAutomaton(const Tables &t_) : t(t_) { blocks.reserve(MAX_BLOCKS); clear(); }

    State &st(uint32_t id) { return blocks[id / BLOCK][id % BLOCK]; }
    const State &st(uint32_t id) const { return blocks[id / BLOCK][id % BLOCK]; }
    static constexpr uint32_t IMPORT_SETS_MAX = 1u << 16;          // the largest chart import takes
    bool full() const { return n_states + IMPORT_SETS_MAX + 2 >= BLOCK * MAX_BLOCKS; }   // no room for another import

    uint32_t add(std::vector<Item> &&items, uint32_t widest) {
        const uint32_t id = n_states;
        if (id / BLOCK >= blocks.size()) blocks.emplace_back(new State[BLOCK]);
        State &s = st(id);
        s.items = std::move(items);
        s.trans.assign(t.n_cls, NONE);
        s.acc.assign(t.n_cls, 0);
        s.widest = widest;
        n_states++;
        return id;
    }

    void clear() {
        blocks.clear();
        interned.clear();
        n_states = 0; n_items = 0;
        add({}, 0);                                            // id 0 is not used
        Chart c;
        chart_init(t, c);
        std::vector<Item> root;
        for (Item it : c.items) {                              // the closure of the start item; its items started in this very set
            if ((t.sym[it.p] >> SYM_KIND_SHIFT) == SYM_END) continue;
            it.o = ROOT;
            root.push_back(it);
        }
        const uint32_t w = (uint32_t)root.size();
        add(std::move(root), w);
    }

    // A transition in three parts, so that callers that share the automaton can run the Earley byte step without
    // holding the lock: lay_out reads (the sets s refers to, transitively, as a chart whose current set is s),
    // earley_step works on that private chart, record writes.
    struct Work { std::vector<uint32_t> ids; Chart c; };
    void lay_out(uint32_t s, Work &w) const {
        // marks instead of searches: a chart of an ambiguous grammar runs to tens of thousands of items
        static thread_local std::vector<uint32_t> mark, place, todo;
        static thread_local uint32_t now = 0;
        const uint32_t room = (s / BLOCK + 1) * BLOCK;         // a state refers to older states only
        if (mark.size() < room) { mark.resize(room, 0); place.resize(room, 0); }
        if (++now == 0) { std::fill(mark.begin(), mark.end(), 0); now = 1; }
        std::vector<uint32_t> &ids = w.ids;
        ids.clear();
        todo.assign(1, s);
        mark[s] = now;
        while (!todo.empty()) {
            const uint32_t id = todo.back();
            todo.pop_back();
            ids.push_back(id);
            for (const Item &it : st(id).items) if (mark[it.o] != now) { mark[it.o] = now; todo.push_back(it.o); }
        }
        std::sort(ids.begin(), ids.end());
        ids.erase(std::lower_bound(ids.begin(), ids.end(), s));
        ids.push_back(s);                                      // the source set last: it is the chart's current set
        for (uint32_t k = 0; k < (uint32_t)ids.size(); k++) place[ids[k]] = k;
        w.c.items.clear();
        w.c.set_off.assign(1, 0);
        for (uint32_t id : ids) {
            for (Item it : st(id).items) { it.o = place[it.o]; w.c.items.push_back(it); }
            w.c.set_off.push_back((uint32_t)w.c.items.size());
        }
    }
    void record(uint32_t s, int cl, const StepResult &r, const Work &w) {
        n_steps++;
        st(s).acc[cl] = r.accepted;
        if (!r.alive) { st(s).trans[cl] = DEAD; return; }
        if (!r.kernel_nonempty) { st(s).trans[cl] = SINK; return; }
        const uint32_t last = w.c.n_sets() - 1;
        std::vector<Item> out(w.c.items.begin() + w.c.set_off[last], w.c.items.end());
        for (Item &it : out) it.o = w.ids[it.o];               // items scanned from predictions started in the source set: index last - 1 = s
        st(s).trans[cl] = intern(std::move(out));
    }

    // The state that holds exactly `items` (origins are state ids), made if it is new.
    uint32_t intern(std::vector<Item> &&items) {
        std::vector<uint32_t> key;
        key.reserve(2 * items.size());
        for (const Item &it : items) { key.push_back((uint32_t)it.p | ((uint32_t)it.q << 16)); key.push_back(it.o); }
        auto found = interned.find(key);
        if (found != interned.end()) return found->second;
        n_items += (int64_t)items.size();
        uint32_t w = (uint32_t)items.size();
        for (const Item &it : items) w = std::max(w, st(it.o).widest);
        const uint32_t id = add(std::move(items), w);
        interned.emplace(std::move(key), id);
        return id;
    }

    void compute(uint32_t s, uint8_t byte) {
        Work w;
        lay_out(s, w);
        const StepResult r = earley_step(t, w.c, byte, false, nullptr);
        record(s, t.cls[byte], r, w);
    }

    // One byte from state s; returns the next state, SINK or DEAD.
    uint32_t step(uint32_t s, uint8_t byte, bool *accepted) {
        if (s == SINK) { if (accepted) *accepted = false; return DEAD; }
        const int cl = t.cls[byte];
        if (st(s).trans[cl] == NONE) compute(s, byte);
        if (accepted) *accepted = st(s).acc[cl] != 0;
        return st(s).trans[cl];
    }

    // The state of a chart's current set: every set of the chart becomes a state (found by content when it is
    // there already), origins renamed from set indices to state names.  The chart's first set is the set of the
    // empty prefix (everything refers back to it).  A chart whose current set is empty of items stands at SINK.
    uint32_t import(const Chart &c) {
        if (full() || c.n_sets() > IMPORT_SETS_MAX) return 0;       // no room: the caller empties the automaton, or fails
        std::vector<uint32_t> name(c.n_sets(), ROOT);
        for (uint32_t k = 1; k < c.n_sets(); k++) {
            std::vector<Item> items(c.items.begin() + c.set_off[k], c.items.begin() + c.set_off[k + 1]);
            if (items.empty()) { name[k] = SINK; continue; }
            for (Item &it : items) it.o = it.o < k ? name[it.o] : ROOT;
            name[k] = intern(std::move(items));
        }
        return name[c.n_sets() - 1];
    }
};

}  // namespace zf
