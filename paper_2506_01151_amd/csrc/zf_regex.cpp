// Terminals -> byte-level DFAs (paper Section 4.1: terminals are regular expressions matched
// by finite-state machines).  Dialect: literal bytes, \xHH, \n \r \t, \<other> = that byte,
// '.', classes [a-z] / [^...], grouping, '|', postfix * + ? {m} {m,} {m,n}.  Byte oriented,
// no anchors.  Pipeline: recursive-descent parse straight into a Thompson NFA, subset
// construction, Moore minimisation, removal of states that cannot reach acceptance.
#include <algorithm>
#include <bitset>
#include <map>
#include <set>
#include "zf_internal.h"

namespace zf {
namespace {

typedef std::bitset<256> ByteSet;

struct Nfa {
    struct Edge { ByteSet on; int to; };
    std::vector<std::vector<Edge>> edges;
    std::vector<std::vector<int>> eps;
    int add() { edges.emplace_back(); eps.emplace_back(); return (int)edges.size() - 1; }
};
struct Frag { int in, out; };   // one entry state, one exit state

struct Parser {
    const uint8_t *s; size_t n, i = 0;
    Nfa nfa;
    std::string err;
    bool at_end() const { return i >= n; }
    int peek() const { return i < n ? s[i] : -1; }
    bool fail(const std::string &m) { if (err.empty()) err = m + " at offset " + std::to_string(i); return false; }

    static int hexval(int c) {
        if (c >= '0' && c <= '9') return c - '0';
        if (c >= 'a' && c <= 'f') return c - 'a' + 10;
        if (c >= 'A' && c <= 'F') return c - 'A' + 10;
        return -1;
    }
    bool escape(int &out) {   // after the backslash
        if (at_end()) return fail("dangling backslash");
        int c = s[i++];
        if (c == 'x') {
            if (i + 2 > n || hexval(s[i]) < 0 || hexval(s[i + 1]) < 0) return fail("bad \\x escape");
            out = hexval(s[i]) * 16 + hexval(s[i + 1]); i += 2; return true;
        }
        out = c == 'n' ? 10 : c == 'r' ? 13 : c == 't' ? 9 : c;
        return true;
    }
    Frag lit(const ByteSet &b) { Frag f{nfa.add(), nfa.add()}; nfa.edges[f.in].push_back({b, f.out}); return f; }
    Frag empty() { Frag f{nfa.add(), nfa.add()}; nfa.eps[f.in].push_back(f.out); return f; }

    // Copying a fragment (for {m,n}) is done by re-parsing its source span.
    bool parse_alt(Frag &out) {
        Frag first;
        if (!parse_cat(first)) return false;
        if (peek() != '|') { out = first; return true; }
        Frag f{nfa.add(), nfa.add()};
        nfa.eps[f.in].push_back(first.in); nfa.eps[first.out].push_back(f.out);
        while (peek() == '|') {
            i++;
            Frag g;
            if (!parse_cat(g)) return false;
            nfa.eps[f.in].push_back(g.in); nfa.eps[g.out].push_back(f.out);
        }
        out = f; return true;
    }
    bool parse_cat(Frag &out) {
        Frag acc = empty();
        while (!at_end() && peek() != '|' && peek() != ')') {
            Frag g;
            if (!parse_postfix(g)) return false;
            nfa.eps[acc.out].push_back(g.in); acc.out = g.out;
        }
        out = acc; return true;
    }
    Frag star(Frag a) { Frag f{nfa.add(), nfa.add()}; nfa.eps[f.in] = {a.in, f.out}; nfa.eps[a.out].push_back(a.in); nfa.eps[a.out].push_back(f.out); return f; }
    Frag opt(Frag a) { Frag f{nfa.add(), nfa.add()}; nfa.eps[f.in] = {a.in, f.out}; nfa.eps[a.out].push_back(f.out); return f; }
    Frag cat(Frag a, Frag b) { nfa.eps[a.out].push_back(b.in); return Frag{a.in, b.out}; }

    bool parse_postfix(Frag &out) {
        size_t atom_begin = i;
        Frag a;
        if (!parse_atom(a)) return false;
        size_t atom_end = i;
        bool had_postfix = false;
        while (!at_end() && (peek() == '*' || peek() == '+' || peek() == '?' || peek() == '{')) {
            int c = s[i++];
            if (c == '*') a = star(a);
            else if (c == '?') a = opt(a);
            else if (c == '+') { Frag b; if (!reparse(atom_begin, atom_end, b)) return false; a = cat(a, star(b)); }
            else {
                if (had_postfix) return fail("a counted repetition after another postfix operator needs a group");
                long lo = 0, hi = -1; bool comma = false, any = false;
                while (!at_end() && peek() >= '0' && peek() <= '9') { lo = lo * 10 + (s[i++] - '0'); any = true; }
                if (!any) return fail("bad repetition");
                if (peek() == ',') { comma = true; i++; if (peek() >= '0' && peek() <= '9') { hi = 0; while (!at_end() && peek() >= '0' && peek() <= '9') hi = hi * 10 + (s[i++] - '0'); } }
                if (peek() != '}') return fail("bad repetition");
                i++;
                if (!comma) hi = lo;
                if ((hi >= 0 && hi < lo) || lo > 1000 || hi > 1000) return fail("bad repetition bounds");
                size_t after = i;
                // x{lo,hi}: lo copies, then hi-lo optional copies; x{lo,}: lo copies then x*
                Frag acc = empty();
                for (long k = 0; k < lo; k++) { Frag b; if (!reparse(atom_begin, atom_end, b)) return false; acc = cat(acc, b); }
                if (hi < 0) { Frag b; if (!reparse(atom_begin, atom_end, b)) return false; acc = cat(acc, star(b)); }
                else for (long k = lo; k < hi; k++) { Frag b; if (!reparse(atom_begin, atom_end, b)) return false; acc = cat(acc, opt(b)); }
                i = after;
                a = acc;
                // a postfix applied to a counted repetition re-parses the atom only; nesting such
                // as (x{2}){3} must use a group, which is then the atom.
                atom_begin = atom_end = 0;
            }
            had_postfix = true;
            if (atom_end == 0 && !at_end() && (peek() == '*' || peek() == '+' || peek() == '?' || peek() == '{'))
                return fail("postfix after a counted repetition needs a group");
        }
        out = a; return true;
    }
    bool reparse(size_t b, size_t e, Frag &out) {
        size_t save_i = i, save_n = n;
        i = b; n = e;
        bool ok = parse_atom(out) && i == e;
        i = save_i; n = save_n;
        return ok ? true : fail("internal: re-parse of a repeated atom failed");
    }
    bool parse_atom(Frag &out) {
        if (at_end()) return fail("unexpected end");
        int c = s[i++];
        ByteSet b;
        if (c == '(') {
            if (!parse_alt(out)) return false;
            if (peek() != ')') return fail("missing )");
            i++; return true;
        }
        if (c == ')' || c == '*' || c == '+' || c == '?' || c == '{' || c == '|') { i--; return fail("unexpected operator"); }
        if (c == '[') {
            bool neg = false, first = true;
            if (peek() == '^') { neg = true; i++; }
            for (;;) {
                if (at_end()) return fail("missing ]");
                int x = s[i++];
                if (x == ']' && !first) break;
                first = false;
                int lo = x;
                if (x == '\\' && !escape(lo)) return false;
                if (peek() == '-' && i + 1 < n && s[i + 1] != ']') {
                    i++;
                    int y = s[i++], hi = y;
                    if (y == '\\' && !escape(hi)) return false;
                    if (hi < lo) return fail("reversed range");
                    for (int k = lo; k <= hi; k++) b.set(k);
                } else b.set(lo);
            }
            if (neg) b.flip();
        } else if (c == '.') b.set();
        else if (c == '\\') { int v; if (!escape(v)) return false; b.set(v); }
        else b.set(c);
        out = lit(b); return true;
    }
};

void eps_closure(const Nfa &nfa, std::vector<int> &set) {
    std::vector<int> stack(set);
    std::set<int> seen(set.begin(), set.end());
    while (!stack.empty()) {
        int u = stack.back(); stack.pop_back();
        for (int v : nfa.eps[u]) if (seen.insert(v).second) stack.push_back(v);
    }
    set.assign(seen.begin(), seen.end());
}

// Moore minimisation + trimming of states that cannot reach acceptance.
void minimise_and_trim(Dfa &d) {
    int n = d.n_states();
    // co-accessibility
    std::vector<uint8_t> live(n, 0);
    for (int s = 0; s < n; s++) live[s] = d.accept[s];
    for (bool ch = true; ch;) {
        ch = false;
        for (int s = 0; s < n; s++) if (!live[s])
            for (int b = 0; b < 256; b++) { int t = d.trans[s * 256 + b]; if (t >= 0 && live[t]) { live[s] = 1; ch = true; break; } }
    }
    for (int s = 0; s < n; s++) for (int b = 0; b < 256; b++) { int &t = d.trans[s * 256 + b]; if (t >= 0 && !live[t]) t = -1; }
    if (!live[0]) { d.trans.assign(256, -1); d.accept.assign(1, 0); return; }   // empty language
    // partition refinement over live states
    std::vector<int> part(n, -1);
    for (int s = 0; s < n; s++) if (live[s]) part[s] = d.accept[s] ? 1 : 0;
    for (;;) {
        std::map<std::vector<int>, int> sig_ix;
        std::vector<int> np(n, -1);
        for (int s = 0; s < n; s++) if (live[s]) {
            std::vector<int> sig(257);
            sig[0] = part[s];
            for (int b = 0; b < 256; b++) { int t = d.trans[s * 256 + b]; sig[b + 1] = t < 0 ? -1 : part[t]; }
            auto it = sig_ix.find(sig);
            if (it == sig_ix.end()) it = sig_ix.emplace(sig, (int)sig_ix.size()).first;
            np[s] = it->second;
        }
        std::set<int> before, after;
        for (int s = 0; s < n; s++) if (live[s]) { before.insert(part[s]); after.insert(np[s]); }
        bool same = before.size() == after.size();
        part = np;
        if (same) break;
    }
    // renumber with the start state's block first
    std::map<int, int> renum;
    renum[part[0]] = 0;
    for (int s = 0; s < n; s++) if (live[s] && !renum.count(part[s])) { int k = (int)renum.size(); renum[part[s]] = k; }
    int m = (int)renum.size();
    Dfa out;
    out.trans.assign((size_t)m * 256, -1);
    out.accept.assign(m, 0);
    for (int s = 0; s < n; s++) if (live[s]) {
        int a = renum[part[s]];
        out.accept[a] = d.accept[s];
        for (int b = 0; b < 256; b++) { int t = d.trans[s * 256 + b]; out.trans[a * 256 + b] = t < 0 ? -1 : renum[part[t]]; }
    }
    d = out;
}

}  // namespace

bool regex_to_dfa(const uint8_t *src, size_t n, Dfa &out) {
    Parser p{src, n};
    Frag f;
    if (!p.parse_alt(f) || !p.at_end()) {
        if (p.err.empty()) p.fail("unbalanced )");
        set_error("regex: " + p.err);
        return false;
    }
    const Nfa &nfa = p.nfa;
    std::map<std::vector<int>, int> ix;
    std::vector<std::vector<int>> sets;
    std::vector<int> start{f.in};
    eps_closure(nfa, start);
    ix[start] = 0; sets.push_back(start);
    out.trans.clear(); out.accept.clear();
    for (size_t k = 0; k < sets.size(); k++) {
        if (sets.size() > 20000) { set_error("regex: automaton too large"); return false; }
        out.trans.resize((k + 1) * 256, -1);
        std::vector<int> cur = sets[k];
        out.accept.push_back(std::binary_search(cur.begin(), cur.end(), f.out) ? 1 : 0);
        // group bytes by target set
        std::vector<std::vector<int>> tgt(256);
        for (int u : cur) for (const auto &e : nfa.edges[u]) for (int b = 0; b < 256; b++) if (e.on[b]) tgt[b].push_back(e.to);
        std::map<std::vector<int>, int> local;
        for (int b = 0; b < 256; b++) {
            if (tgt[b].empty()) continue;
            std::sort(tgt[b].begin(), tgt[b].end());
            tgt[b].erase(std::unique(tgt[b].begin(), tgt[b].end()), tgt[b].end());
            auto lit = local.find(tgt[b]);
            int id;
            if (lit != local.end()) id = lit->second;
            else {
                std::vector<int> cl = tgt[b];
                eps_closure(nfa, cl);
                auto it = ix.find(cl);
                if (it == ix.end()) { it = ix.emplace(cl, (int)sets.size()).first; sets.push_back(cl); }
                id = it->second;
                local[tgt[b]] = id;
            }
            out.trans[k * 256 + b] = id;
        }
    }
    minimise_and_trim(out);
    return true;
}

void literal_to_dfa(const uint8_t *bytes, size_t n, Dfa &out) {
    out.trans.assign((n + 1) * 256, -1);
    out.accept.assign(n + 1, 0);
    for (size_t k = 0; k < n; k++) out.trans[k * 256 + bytes[k]] = (int)k + 1;
    out.accept[n] = 1;
}

}  // namespace zf
