// Host-side structures of the library (grammar tables, trie, chart, engine, state).
#pragma once
#include <cstdint>
#include <memory>
#include <mutex>
#include <string>
#include <vector>
#include "zf_device.h"
#include "../../include/zapformat.h"
#include "../../include/zapformat_debug.h"

namespace zf {

struct HostAutomaton;
void set_error(const std::string &msg);   // thread-local detail string

// ---- byte-level DFA of one terminal ---------------------------------------------------
struct Dfa {
    // trans[state*256 + byte] = next state or -1; state 0 is the start state.  Every state can
    // reach an accepting state (trimmed), so "alive" means "the terminal can still finish".
    std::vector<int32_t> trans;
    std::vector<uint8_t> accept;
    int n_states() const { return (int)accept.size(); }
};
// Returns false and sets the error string on a syntax error.
bool regex_to_dfa(const uint8_t *src, size_t n, Dfa &out);
void literal_to_dfa(const uint8_t *bytes, size_t n, Dfa &out);

// ---- compiled grammar tables ------------------------------------------------------------
struct Tables {
    int N = 0;                        // nonterminals kept + 1 (the added start symbol S' = N-1)
    int T = 0;                        // terminals
    int P = 0;                        // dotted positions
    int Q = 0;                        // DFA states over all terminals
    int n_cls = 0;
    int start_pos = 0;                // position of (S' -> . S)
    std::vector<uint16_t> sym;        // [P]
    std::vector<uint16_t> lhs_of;     // [P] lhs of the rule that contains the position
    std::vector<uint16_t> end_pos;    // [N]
    uint8_t cls[256];
    std::vector<uint16_t> delta;      // [Q*n_cls]
    std::vector<uint8_t> qflags;      // [Q]
    std::vector<uint32_t> advpq;      // [P] device item word to insert when the dot arrives at p
    std::vector<uint32_t> dev_scan_list;  // scan_list for the device: (item word, flags) pairs
    std::vector<uint32_t> qinfo;      // [Q] flags | literal byte << 8 | dense row << 16
    std::vector<uint32_t> delta_dense; // rows of the non-literal states only: next state | flags << 16
    int end_base = 0;                 // end_pos[X] == end_base + X
    std::vector<std::vector<uint16_t>> first_terms;   // [N] terminals that can begin a derivation of Y
    std::vector<uint16_t> term_start; // [T]
    std::vector<uint32_t> scan_off, scan_list;
    std::vector<uint32_t> comp_off;
    std::vector<uint16_t> comp_list;      // positions, COMP_ADVANCE_WAITING = "advance the waiting item itself"
    std::vector<uint32_t> dev_comp_list;  // the same as device item words (0xFFFFFFFF for the marker)
    std::vector<uint8_t> reach;       // [N*N] reach[Y*N+X] = 1 iff X can be a left corner of Y (X in PRED(Y))
    // for zf_position_info: original rule index / lhs / dot of each position (-1 for added ones)
    std::vector<int32_t> pos_rule, pos_dot, pos_lhs_orig;
    int n_rules_kept = 0;
};
bool build_tables(const zf_grammar_desc *g, Tables &t);

// ---- vocabulary trie ------------------------------------------------------------------------
struct Trie {
    std::vector<TrieNode> nodes;      // preorder
    std::vector<uint32_t> parent;
    std::vector<uint32_t> chunk_begin, chunk_end;
    std::vector<TrieNode> chunk_anc;   // [n_chunks][CHUNK_ANC]
    std::vector<uint32_t> rank_of;    // [V]
    std::vector<uint32_t> str_off;    // [n_strings + 1] the distinct strings in rank order, flat: string r is
    std::vector<uint8_t> str_bytes;   //   str_bytes[str_off[r] .. str_off[r+1])
    int n_strings = 0;
    int chunk_ranks = 32;
    int Wr = 0;                       // words per row of a rank-ordered bitmap
    std::vector<uint32_t> ci_valid, ci_cd;   // [(Q + N) * Wr]
    std::vector<uint32_t> ci_undecided;      // [Q + N] strings of the row that are in ci_cd but not in ci_valid
};
// Context-independent token-mask cache (Section 4.3): per DFA state and per nonterminal, which
// strings are decided by the terminal alone and which need the parser.
void build_token_mask_cache(const Tables &t, Trie &tr);
void build_trie(const zf_vocab_desc *v, int chunk_ranks, const uint8_t *cls, Trie &t);

// ---- chart --------------------------------------------------------------------------------------
struct Chart {
    std::vector<Item> items;
    std::vector<uint32_t> set_off{0};   // n_sets + 1 entries
    uint32_t n_sets() const { return (uint32_t)set_off.size() - 1; }
    void truncate(uint32_t n) { set_off.resize(n + 1); items.resize(set_off[n]); }
};
struct StepResult { bool alive, kernel_nonempty, accepted; };
// Scan `byte` from the last set into a new set and close it (Complete + implicit Predict).
// The new set is appended even when it ends up empty.  keep_completed keeps the end-of-rule
// items in the set (pruning off); otherwise they are dropped once the set is closed.
StepResult earley_step(const Tables &t, Chart &c, uint8_t byte, bool keep_completed, int64_t *items_created);
void chart_init(const Tables &t, Chart &c);
// ZapFormat Compact: keep only what the last set can still reach through Complete look-ups.
void chart_compact(const Tables &t, Chart &c);

}  // namespace zf

struct zf_engine {
    zf::Tables tab;
    zf::Trie trie;
    zf_options opt;
    int32_t V = 0, W = 0;
    std::vector<int64_t> voc_off;
    std::vector<uint8_t> voc_bytes;
    bool start_nullable = false;
    bool lane_cap_auto = true;          // no explicit lane_item_cap: the budget follows the rows' set sizes
    bool store_on = false;              // the mask calls go through the persistent automaton (walk_mode 2, pruning on, a device)
    // zf_advance through the persistent automaton on the host (walk_mode 2, pruning on): a token's bytes are walked through
    // the table of known transitions, an Earley byte step runs only for a transition nobody has taken before, and the
    // state's chart is brought up to date only when somebody asks for it.  One automaton per engine.
    struct zf::HostAutomaton *host_aut = nullptr;
    std::mutex host_mu;                 // look-ups and everything that writes; an Earley byte step for a new transition runs without it
    int host_walkers = 0;               // threads between reading the sets a new transition needs and recording it (the automaton is not emptied meanwhile)
    uint32_t host_epoch = 1;            // bumped when the host automaton is emptied (it is when it has grown past a bound)
    struct DeviceSide *dev = nullptr;   // null when compiled with device = -1
};

struct zf_state;
namespace zf { struct StateLink { zf_state *s; }; }   // what a mask call in flight holds of a state: cleared when the state is destroyed

struct zf_state {
    zf_engine *eng;
    std::shared_ptr<zf::StateLink> link;
    zf::Chart chart;
    bool accepting = false;
    int64_t items_created = 0, bytes_fed = 0;
    // Where the row stands in the engine's persistent automaton (walk_mode 2): the state it was last known to be in,
    // and the byte classes fed since (the next mask call walks them on the device and reports the new state).
    uint32_t dev_id = 1;                // 1 = the state of the empty prefix, valid in every epoch of the store
    uint32_t dev_epoch = 0;             // epoch of the store dev_id belongs to
    uint32_t generation = 0;            // bumped by every reset: results of calls enqueued before it no longer apply
    std::vector<uint8_t> pending;
    uint64_t fed_total = 0;             // bytes fed since the state was made; pending covers [pending_base, fed_total)
    uint64_t pending_base = 0;
    int32_t pending_token = -1;         // the token whose bytes are all of `pending`, fed in state dev_id; -1 when pending is anything else
    // Where the state stands in the engine's host automaton (when the engine has one), and the bytes fed since `chart` was last
    // brought up to date (lag_cut: where each zf_advance call's bytes end).  Everything that reads the chart goes through
    // zf::chart_of, which feeds them to the chart first.
    uint32_t host_id = 1;               // 1 = the state of the empty prefix, valid in every epoch
    uint32_t host_id_epoch = 0;
    std::vector<uint8_t> lag;
    std::vector<uint32_t> lag_cut;
};

namespace zf {
// The state's chart, brought up to date first when bytes were fed through the host automaton since it last was.
const Chart &chart_of(const zf_state *s);
}
