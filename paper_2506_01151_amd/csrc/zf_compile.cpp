// Grammar compiler: grammar clean-up (paper Section 4.5: useless rules, nullable symbols),
// per-terminal DFAs merged into one state numbering with byte equivalence classes (Section
// 4.1), the look-up tables that replace explicit Predict items, and the flattened
// vocabulary trie.
//
// Table-driven Earley used throughout the library.  Only items that have consumed at least
// one byte ("kernel" items) are stored in a set.  Everything Predict would add to a set is a
// function of the postdot nonterminals of its kernel items, so it is tabulated once:
//   PRED(Y)  = nonterminals that can start a derivation of Y (left corners, skipping nullable
//              prefixes), Y included;
//   I(Y)     = dotted positions (Z -> alpha . beta) with Z in PRED(Y) and alpha nullable;
//   SCAN(Y,c)= for positions of I(Y) that stand before a terminal t: (position, delta_t(start, c))
//              for every byte class c the terminal can start with;
//   COMP(Y,X)= what the completion of X does to the predicted items of I(Y): the positions that
//              stand behind X in I(Y), with nullable symbols skipped -- and, where such a
//              position is the end of its rule, its left-hand side counts as completed too (same
//              origin, the set that predicted it) and is followed up here, at compile time.  The
//              list holds the resulting items and, if Y itself is among the completed
//              nonterminals, a marker that tells the recognizer to advance the waiting item.
// Nullable nonterminals are handled when an item is added: the item is also added with the dot
// moved over the nullable symbol (Aycock-Horspool), so no epsilon rule survives at run time.
#include <algorithm>
#include <cstring>
#include <map>
#include <set>
#include "zf_internal.h"

namespace zf {

bool build_tables(const zf_grammar_desc *g, Tables &t) {
    if (!g || g->n_nonterminals <= 0 || g->n_rules < 0 || g->n_terminals < 0 || g->start < 0 ||
        g->start >= g->n_nonterminals || (g->n_rules && (!g->rule_lhs || !g->rhs_off)) ||
        (g->n_terminals && (!g->term_kind || !g->term_off))) {
        set_error("grammar: bad sizes or null arrays");
        return false;
    }
    const int NT0 = g->n_nonterminals, R0 = g->n_rules, T = g->n_terminals;
    for (int r = 0; r < R0; r++) {
        if (g->rule_lhs[r] < 0 || g->rule_lhs[r] >= NT0 || g->rhs_off[r + 1] < g->rhs_off[r]) { set_error("grammar: bad rule " + std::to_string(r)); return false; }
        for (int k = g->rhs_off[r]; k < g->rhs_off[r + 1]; k++) {
            int s = g->rhs_sym[k];
            if ((s >= 0 && s >= NT0) || (s < 0 && ~s >= T)) { set_error("grammar: bad symbol in rule " + std::to_string(r)); return false; }
        }
    }
    // ---- terminals -> DFAs ----
    std::vector<Dfa> dfas(T);
    for (int k = 0; k < T; k++) {
        const uint8_t *src = g->term_data + g->term_off[k];
        size_t n = (size_t)(g->term_off[k + 1] - g->term_off[k]);
        if (g->term_kind[k] == 0) literal_to_dfa(src, n, dfas[k]);
        else if (g->term_kind[k] == 1) { if (!regex_to_dfa(src, n, dfas[k])) return false; }
        else { set_error("grammar: bad terminal kind"); return false; }
        if (dfas[k].accept[0]) { set_error("grammar: terminal " + std::to_string(k) + " matches the empty string; make it optional in a rule instead"); return false; }
        bool any = false;
        for (int b = 0; b < 256; b++) any |= dfas[k].trans[b] >= 0;
        if (!any) { set_error("grammar: terminal " + std::to_string(k) + " has an empty language"); return false; }
    }
    // ---- useless-rule removal: productive, then reachable ----
    std::vector<uint8_t> productive(NT0, 0), reachable(NT0, 0);
    for (bool ch = true; ch;) {
        ch = false;
        for (int r = 0; r < R0; r++) {
            if (productive[g->rule_lhs[r]]) continue;
            bool all = true;
            for (int k = g->rhs_off[r]; k < g->rhs_off[r + 1] && all; k++) { int s = g->rhs_sym[k]; if (s >= 0 && !productive[s]) all = false; }
            if (all) { productive[g->rule_lhs[r]] = 1; ch = true; }
        }
    }
    if (!productive[g->start]) { set_error("grammar: the start symbol derives no string"); return false; }
    auto rule_ok = [&](int r) {
        if (!productive[g->rule_lhs[r]]) return false;
        for (int k = g->rhs_off[r]; k < g->rhs_off[r + 1]; k++) { int s = g->rhs_sym[k]; if (s >= 0 && !productive[s]) return false; }
        return true;
    };
    reachable[g->start] = 1;
    for (bool ch = true; ch;) {
        ch = false;
        for (int r = 0; r < R0; r++) if (rule_ok(r) && reachable[g->rule_lhs[r]])
            for (int k = g->rhs_off[r]; k < g->rhs_off[r + 1]; k++) { int s = g->rhs_sym[k]; if (s >= 0 && !reachable[s]) { reachable[s] = 1; ch = true; } }
    }
    std::vector<int> nt_new(NT0, -1);
    int N = 0;
    for (int a = 0; a < NT0; a++) if (productive[a] && reachable[a]) nt_new[a] = N++;
    const int SP = N++;   // the added start symbol S'
    if (N > (int)SYM_ID_MASK_NT) { set_error("grammar: too many nonterminals"); return false; }
    if (T > (int)SYM_ID_MASK) { set_error("grammar: too many terminals"); return false; }
    struct Rule { int lhs, orig; std::vector<int> rhs; };   // rhs: >=0 new nonterminal id, <0 terminal
    std::vector<Rule> rules;
    for (int r = 0; r < R0; r++) if (rule_ok(r) && reachable[g->rule_lhs[r]]) {
        Rule x{nt_new[g->rule_lhs[r]], r, {}};
        for (int k = g->rhs_off[r]; k < g->rhs_off[r + 1]; k++) { int s = g->rhs_sym[k]; x.rhs.push_back(s >= 0 ? nt_new[s] : s); }
        rules.push_back(x);
    }
    rules.push_back(Rule{SP, -1, {nt_new[g->start]}});
    t.n_rules_kept = (int)rules.size() - 1;
    // ---- nullable ----
    std::vector<uint8_t> nullable(N, 0);
    for (bool ch = true; ch;) {
        ch = false;
        for (auto &r : rules) if (!nullable[r.lhs]) {
            bool all = true;
            for (int s : r.rhs) if (s < 0 || !nullable[s]) { all = false; break; }
            if (all) { nullable[r.lhs] = 1; ch = true; }
        }
    }
    // ---- terminals actually used; merge DFAs into one numbering; byte classes ----
    t.T = T;
    t.term_start.assign(T, 0);
    std::vector<int> base(T, 0);
    int Q = 0;
    for (int k = 0; k < T; k++) { base[k] = Q; Q += dfas[k].n_states(); }
    if (Q >= (int)DFA_DEAD) { set_error("grammar: too many DFA states"); return false; }
    t.Q = Q;
    {   // two bytes are equivalent when every state of every DFA treats them alike
        std::map<std::vector<int32_t>, int> col_ix;
        for (int b = 0; b < 256; b++) {
            std::vector<int32_t> col;
            col.reserve(Q);
            for (int k = 0; k < T; k++) for (int s = 0; s < dfas[k].n_states(); s++) col.push_back(dfas[k].trans[s * 256 + b]);
            auto it = col_ix.find(col);
            if (it == col_ix.end()) it = col_ix.emplace(col, (int)col_ix.size()).first;
            t.cls[b] = (uint8_t)it->second;
        }
        t.n_cls = (int)col_ix.size();
    }
    t.delta.assign((size_t)Q * t.n_cls, DFA_DEAD);
    t.qflags.assign(Q, 0);
    for (int k = 0; k < T; k++) {
        t.term_start[k] = (uint16_t)base[k];
        for (int s = 0; s < dfas[k].n_states(); s++) {
            bool cont = false;
            for (int b = 0; b < 256; b++) {
                int to = dfas[k].trans[s * 256 + b];
                if (to >= 0) { t.delta[(size_t)(base[k] + s) * t.n_cls + t.cls[b]] = (uint16_t)(base[k] + to); cont = true; }
            }
            t.qflags[base[k] + s] = (dfas[k].accept[s] ? QF_ACCEPT : 0) | (cont ? QF_CONT : 0);
        }
    }
    // ---- dotted positions ----
    t.N = N;
    t.sym.clear(); t.lhs_of.clear(); t.pos_rule.clear(); t.pos_dot.clear(); t.pos_lhs_orig.clear();
    std::vector<int> rule_base(rules.size());
    std::vector<int> orig_of_new(N, -1);
    for (int a = 0; a < NT0; a++) if (nt_new[a] >= 0) orig_of_new[nt_new[a]] = a;
    for (size_t r = 0; r < rules.size(); r++) {
        rule_base[r] = (int)t.sym.size();
        for (size_t d = 0; d <= rules[r].rhs.size(); d++) {
            uint16_t code;
            if (d == rules[r].rhs.size()) code = (uint16_t)((SYM_END << SYM_KIND_SHIFT) | rules[r].lhs);
            else if (rules[r].rhs[d] < 0) code = (uint16_t)((SYM_TERM << SYM_KIND_SHIFT) | (~rules[r].rhs[d]));
            else code = (uint16_t)((SYM_NT << SYM_KIND_SHIFT) | rules[r].rhs[d] | (nullable[rules[r].rhs[d]] ? SYM_NULLABLE_BIT : 0));
            t.sym.push_back(code);
            t.lhs_of.push_back((uint16_t)rules[r].lhs);
            t.pos_rule.push_back(rules[r].orig); t.pos_dot.push_back((int)d); t.pos_lhs_orig.push_back(orig_of_new[rules[r].lhs]);
        }
    }
    t.start_pos = rule_base.back();
    t.end_pos.assign(N, 0);
    for (int a = 0; a < N; a++) {   // one canonical "X is complete" position per nonterminal
        t.end_pos[a] = (uint16_t)t.sym.size();
        t.sym.push_back((uint16_t)((SYM_END << SYM_KIND_SHIFT) | a));
        t.lhs_of.push_back((uint16_t)a);
        t.pos_rule.push_back(-1); t.pos_dot.push_back(-1); t.pos_lhs_orig.push_back(orig_of_new[a]);
    }
    t.P = (int)t.sym.size();
    if (t.P > (int)MAX_POSITIONS) { set_error("grammar: too many dotted positions"); return false; }
    t.end_base = t.end_pos[0];
    t.advpq.assign(t.P, 0);
    for (int p = 0; p < t.P; p++) {
        uint16_t code = t.sym[p];
        int k = code >> SYM_KIND_SHIFT;
        if (k == SYM_END) t.advpq[p] = (uint32_t)t.end_pos[code & SYM_ID_MASK] | IW_END;
        else if (k == SYM_TERM) t.advpq[p] = (uint32_t)p | IW_TERM | ((uint32_t)t.term_start[code & SYM_ID_MASK] << 16);
        else t.advpq[p] = (uint32_t)p | ((code & SYM_NULLABLE_BIT) ? (uint32_t)IW_NT_NULLABLE : 0u) | ((uint32_t)(code & SYM_ID_MASK_NT) << IW_NT_SHIFT);
    }
    // hybrid DFA encoding for the device: literal chains carry their byte, other states a dense row
    t.qinfo.assign(Q, 0);
    t.delta_dense.clear();
    for (int k = 0; k < T; k++) {
        const bool lit = g->term_kind[k] == 0;
        for (int s = 0; s < dfas[k].n_states(); s++) {
            int q = base[k] + s;
            uint32_t info = t.qflags[q];
            if (lit) {
                int b = 0;
                for (int x = 0; x < 256; x++) if (dfas[k].trans[s * 256 + x] >= 0) b = x;
                info |= QF_LITERAL | ((uint32_t)b << 8);
                if (s + 1 < dfas[k].n_states()) info |= (uint32_t)t.qflags[q + 1] << 16;
            } else {
                uint32_t row = (uint32_t)(t.delta_dense.size() / t.n_cls);
                for (int c = 0; c < t.n_cls; c++) {
                    uint16_t to = t.delta[(size_t)q * t.n_cls + c];
                    t.delta_dense.push_back(to == DFA_DEAD ? (uint32_t)DFA_DEAD : ((uint32_t)to | ((uint32_t)t.qflags[to] << 16)));
                }
                info |= row << 16;
            }
            t.qinfo[q] = info;
        }
    }
    // ---- PRED / I / SCAN / COMP ----
    // lead[Z] = positions of Z's rules reachable from the rule start over nullable symbols
    std::vector<std::vector<int>> lead(N);
    for (size_t r = 0; r < rules.size(); r++)
        for (size_t d = 0; d < rules[r].rhs.size(); d++) {
            lead[rules[r].lhs].push_back(rule_base[r] + (int)d);
            int s = rules[r].rhs[d];
            if (s < 0 || !nullable[s]) break;
        }
    t.reach.assign((size_t)N * N, 0);
    t.first_terms.assign(N, {});
    t.scan_off.assign((size_t)N * t.n_cls + 1, 0);
    t.comp_off.assign((size_t)N * N + 1, 0);
    t.scan_list.clear(); t.comp_list.clear();
    std::vector<std::vector<std::vector<uint32_t>>> scan_tmp(N, std::vector<std::vector<uint32_t>>(t.n_cls));
    std::vector<std::vector<std::vector<uint16_t>>> comp_tmp(N, std::vector<std::vector<uint16_t>>(N));
    for (int Y = 0; Y < N; Y++) {
        std::vector<int> stack{Y};
        t.reach[(size_t)Y * N + Y] = 1;
        std::vector<int> I;
        while (!stack.empty()) {
            int Z = stack.back(); stack.pop_back();
            for (int p : lead[Z]) {
                I.push_back(p);
                uint16_t code = t.sym[p];
                if ((code >> SYM_KIND_SHIFT) == SYM_NT) {
                    int X = code & SYM_ID_MASK_NT;
                    if (!t.reach[(size_t)Y * N + X]) { t.reach[(size_t)Y * N + X] = 1; stack.push_back(X); }
                }
            }
        }
        std::sort(I.begin(), I.end());
        for (int p : I) {
            uint16_t code = t.sym[p];
            if ((code >> SYM_KIND_SHIFT) == SYM_TERM) {
                int term = code & SYM_ID_MASK;
                if (std::find(t.first_terms[Y].begin(), t.first_terms[Y].end(), (uint16_t)term) == t.first_terms[Y].end())
                    t.first_terms[Y].push_back((uint16_t)term);
                for (int c = 0; c < t.n_cls; c++) {
                    uint16_t to = t.delta[(size_t)t.term_start[term] * t.n_cls + c];
                    if (to != DFA_DEAD) scan_tmp[Y][c].push_back((uint32_t)p | ((uint32_t)to << 16));
                }
            } else if ((code >> SYM_KIND_SHIFT) == SYM_NT) {
                comp_tmp[Y][code & SYM_ID_MASK_NT].push_back((uint16_t)(p + 1));
            }
        }
    }
    for (int Y = 0; Y < N; Y++) for (int c = 0; c < t.n_cls; c++) {
        t.scan_off[(size_t)Y * t.n_cls + c] = (uint32_t)t.scan_list.size();
        t.scan_list.insert(t.scan_list.end(), scan_tmp[Y][c].begin(), scan_tmp[Y][c].end());
    }
    t.scan_off[(size_t)N * t.n_cls] = (uint32_t)t.scan_list.size();
    for (int Y = 0; Y < N; Y++) for (int X = 0; X < N; X++) {
        t.comp_off[(size_t)Y * N + X] = (uint32_t)t.comp_list.size();
        if (!t.reach[(size_t)Y * N + X]) continue;       // no item predicted by Y waits for X or for anything X leads to
        std::vector<uint8_t> completed(N, 0);
        std::vector<int> work{X};
        std::vector<uint16_t> out;
        completed[X] = 1;
        bool y_completes = false;
        while (!work.empty()) {
            const int C = work.back(); work.pop_back();
            if (C == Y) y_completes = true;
            for (uint16_t p1 : comp_tmp[Y][C]) {
                for (int p = p1;; p++) {                   // the dot arrives at p: same walk as the recognizer's add step
                    const uint16_t code = t.sym[p];
                    const int k = code >> SYM_KIND_SHIFT;
                    if (k == SYM_END) { const int L = code & SYM_ID_MASK; if (!completed[L]) { completed[L] = 1; work.push_back(L); } break; }
                    if (std::find(out.begin(), out.end(), (uint16_t)p) == out.end()) out.push_back((uint16_t)p);
                    if (k == SYM_TERM || !(code & SYM_NULLABLE_BIT)) break;
                }
            }
        }
        std::sort(out.begin(), out.end());
        t.comp_list.insert(t.comp_list.end(), out.begin(), out.end());
        if (y_completes) t.comp_list.push_back(COMP_ADVANCE_WAITING);
    }
    t.comp_off[(size_t)N * N] = (uint32_t)t.comp_list.size();
    t.dev_comp_list.resize(t.comp_list.size());
    for (size_t k = 0; k < t.comp_list.size(); k++)
        t.dev_comp_list[k] = t.comp_list[k] == COMP_ADVANCE_WAITING ? 0xFFFFFFFFu : t.advpq[t.comp_list[k]];
    t.dev_scan_list.resize(2 * t.scan_list.size());
    for (size_t k = 0; k < t.scan_list.size(); k++) {
        t.dev_scan_list[2 * k] = t.scan_list[k] | IW_TERM;
        t.dev_scan_list[2 * k + 1] = t.qflags[t.scan_list[k] >> 16];
    }
    return true;
}

// ---- vocabulary -> flattened prefix trie ---------------------------------------------------
void build_trie(const zf_vocab_desc *v, int CHUNK_RANKS, const uint8_t *cls, Trie &t) {
    t.chunk_ranks = CHUNK_RANKS;
    const int V = v->V;
    std::vector<int> order;
    for (int i = 0; i < V; i++) if (v->off[i + 1] > v->off[i]) order.push_back(i);
    auto tok = [&](int i, const uint8_t *&p, size_t &n) { p = v->bytes + v->off[i]; n = (size_t)(v->off[i + 1] - v->off[i]); };
    std::sort(order.begin(), order.end(), [&](int a, int b) {
        const uint8_t *pa, *pb; size_t na, nb;
        tok(a, pa, na); tok(b, pb, nb);
        int c = memcmp(pa, pb, std::min(na, nb));
        if (c) return c < 0;
        if (na != nb) return na < nb;
        return a < b;
    });
    t.nodes.clear(); t.parent.clear(); t.rank_of.assign(V, 0xFFFFFFFFu);
    t.str_off.clear(); t.str_bytes.clear();
    // Walk the sorted strings; the stack holds the node indices of the current path.
    std::vector<uint32_t> path;       // path[d-1] = node index at depth d
    std::vector<uint8_t> path_bytes;
    uint32_t rank = 0;
    const uint8_t *prev = nullptr; size_t prev_n = 0;
    for (int id : order) {
        const uint8_t *p; size_t n;
        tok(id, p, n);
        if (n > (size_t)MAX_TOKEN_LEN_ON_DEVICE) n = MAX_TOKEN_LEN_ON_DEVICE;   // guarded by zf_compile
        if (prev && prev_n == n && memcmp(prev, p, n) == 0) { t.rank_of[id] = rank - 1; continue; }   // duplicate string
        size_t common = 0;
        while (common < path_bytes.size() && common < n && path_bytes[common] == p[common]) common++;
        // close the subtrees we leave
        path.resize(common); path_bytes.resize(common);
        for (size_t d = common; d < n; d++) {
            TrieNode nd{};
            nd.byte = p[d]; nd.cls = cls[p[d]]; nd.depth = (uint8_t)(d + 1); nd.has_string = (d + 1 == n); nd.rank = rank; nd.skip = 0;
            t.parent.push_back(d == 0 ? 0xFFFFFFFFu : path[d - 1]);
            path.push_back((uint32_t)t.nodes.size()); path_bytes.push_back(p[d]);
            t.nodes.push_back(nd);
        }
        t.rank_of[id] = rank++;
        t.str_off.push_back((uint32_t)t.str_bytes.size());
        t.str_bytes.insert(t.str_bytes.end(), p, p + n);
        prev = p; prev_n = n;
    }
    t.str_off.push_back((uint32_t)t.str_bytes.size());
    t.n_strings = (int)rank;
    // skip pointers: next node in preorder whose depth is <= this node's depth
    {
        const uint32_t n = (uint32_t)t.nodes.size();
        std::vector<uint32_t> open;   // stack of node indices waiting for their subtree end
        for (uint32_t i = 0; i < n; i++) {
            while (!open.empty() && t.nodes[open.back()].depth >= t.nodes[i].depth) { t.nodes[open.back()].skip = i; open.pop_back(); }
            open.push_back(i);
        }
        for (uint32_t i : open) t.nodes[i].skip = n;
        for (uint32_t i = 0; i < n; i++) {
            uint32_t end_rank = t.nodes[i].skip < n ? t.nodes[t.nodes[i].skip].rank : (uint32_t)t.n_strings;
            t.nodes[i].n_sub = end_rank - t.nodes[i].rank;
        }
    }
    // chunks of CHUNK_RANKS strings: [node that carries rank 32c, node that carries the chunk's last rank + 1)
    int n_chunks = (t.n_strings + CHUNK_RANKS - 1) / CHUNK_RANKS;
    t.chunk_begin.assign(n_chunks, 0); t.chunk_end.assign(n_chunks, 0);
    for (uint32_t i = 0; i < t.nodes.size(); i++) if (t.nodes[i].has_string) {
        uint32_t r = t.nodes[i].rank;
        if (r % CHUNK_RANKS == 0) t.chunk_begin[r / CHUNK_RANKS] = i;
        t.chunk_end[r / CHUNK_RANKS] = i + 1;
    }
    t.Wr = (n_chunks * CHUNK_RANKS + 31) / 32;
    // ancestors of each chunk's first node (top down), for the lanes that start in mid-trie
    t.chunk_anc.assign((size_t)n_chunks * CHUNK_ANC, TrieNode{});
    for (int c = 0; c < n_chunks; c++) {
        uint32_t i = t.chunk_begin[c];
        int d = t.nodes[i].depth;
        for (uint32_t a = t.parent[i]; a != 0xFFFFFFFFu; a = t.parent[a]) {
            d--;
            if (d - 1 < CHUNK_ANC) t.chunk_anc[(size_t)c * CHUNK_ANC + d - 1] = t.nodes[a];
        }
    }
}

}  // namespace zf

namespace zf {

// For every DFA state q: run the DFA alone from q down the trie.  A string the DFA survives is
// valid whatever the context (the in-progress terminal item survives or has just completed).  A
// string on which the DFA dies is hopeless for this item unless the DFA passed an accepting state
// first -- then the terminal may end there and what follows depends on the parser.  Rows of
// nonterminals are the union over the terminals that can begin them.
void build_token_mask_cache(const Tables &t, Trie &tr) {
    const int Wr = tr.Wr, rows = t.Q + t.N;
    tr.ci_valid.assign((size_t)rows * Wr, 0);
    tr.ci_cd.assign((size_t)rows * Wr, 0);
    const uint32_t n = (uint32_t)tr.nodes.size();
    auto fill = [](uint32_t *bits, uint32_t lo, uint32_t hi) {   // set bits [lo, hi)
        while (lo < hi) {
            uint32_t w = lo >> 5, b = lo & 31, cnt = std::min<uint32_t>(32 - b, hi - lo);
            bits[w] |= (cnt == 32 ? 0xFFFFFFFFu : ((1u << cnt) - 1)) << b;
            lo += cnt;
        }
    };
    std::vector<uint16_t> st(MAX_TOKEN_LEN_ON_DEVICE + 2);
    std::vector<uint8_t> acc(MAX_TOKEN_LEN_ON_DEVICE + 2);
    for (int q = 0; q < t.Q; q++) {
        if (!(t.qflags[q] & QF_CONT)) continue;   // no item ever waits in a state without outgoing edges
        uint32_t *V = &tr.ci_valid[(size_t)q * Wr], *C = &tr.ci_cd[(size_t)q * Wr];
        st[0] = (uint16_t)q; acc[0] = 0;
        for (uint32_t i = 0; i < n;) {
            const TrieNode &nd = tr.nodes[i];
            const int d = nd.depth;
            uint16_t s2 = t.delta[(size_t)st[d - 1] * t.n_cls + t.cls[nd.byte]];
            if (s2 == DFA_DEAD) {
                if (acc[d - 1]) fill(C, nd.rank, nd.rank + nd.n_sub);
                i = nd.skip;
            } else {
                st[d] = s2; acc[d] = acc[d - 1] | (t.qflags[s2] & QF_ACCEPT);
                if (nd.has_string) V[nd.rank >> 5] |= 1u << (nd.rank & 31);
                i++;
            }
        }
    }
    for (int Y = 0; Y < t.N; Y++) {
        uint32_t *V = &tr.ci_valid[(size_t)(t.Q + Y) * Wr], *C = &tr.ci_cd[(size_t)(t.Q + Y) * Wr];
        for (uint16_t term : t.first_terms[Y]) {
            const uint32_t *v = &tr.ci_valid[(size_t)t.term_start[term] * Wr], *c = &tr.ci_cd[(size_t)t.term_start[term] * Wr];
            for (int w = 0; w < Wr; w++) { V[w] |= v[w]; C[w] |= c[w]; }
        }
    }
    tr.ci_undecided.assign(rows, 0);                     // per row: strings it leaves to the parser (the host sizes a call's grid by it)
    for (int r = 0; r < rows; r++)
        for (int w = 0; w < Wr; w++) tr.ci_undecided[r] += (uint32_t)__builtin_popcount(tr.ci_cd[(size_t)r * Wr + w] & ~tr.ci_valid[(size_t)r * Wr + w]);
}

}  // namespace zf
