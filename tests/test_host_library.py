"""CPU tests of the library's host side: the C boundary loads and exports what the header
declares, error paths, and the host logic (grammar compiler, DFAs, trie, Earley advance,
ZapFormat compaction) checked against the oracle through the host walk of the compiled tables.
No GPU is touched: engines are compiled with device = -1."""
import os
import re

import numpy as np
import pytest

from workloads import grammars, configs, vocab as wvocab
from workloads.grammar import Grammar, Lit, Rx
from workloads.rng import SplitMix64, stream
from tests.helpers import OracleRun, popcount, load_trajectory

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def zf():
    import paper_2506_01151_amd as zf
    zf.load_library()
    return zf


def test_library_exports_every_declared_symbol(zf):
    from paper_2506_01151_amd.binding import EXPORTS, DEBUG_EXPORTS
    lib = zf.load_library()
    for fname, names, least in (("zapformat.h", EXPORTS, 20), ("zapformat_debug.h", DEBUG_EXPORTS, 8)):
        header = open(os.path.join(ROOT, "include", fname)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared = set(re.findall(r"\b(zf_[a-z0-9_]+)\s*\(", header))
        assert len(declared) >= least
        for name in sorted(declared):
            assert hasattr(lib, name), f"{name} is declared in {fname} but not exported"
        assert declared == set(names)
        assert not any("debug" in n for n in declared) or fname == "zapformat_debug.h"


def _all_strings(alphabet, max_len):
    import itertools
    for n in range(1, max_len + 1):
        for tup in itertools.product(alphabet, repeat=n):
            yield bytes(tup)


SMALL = [(grammars.w1_grammar, b"ab"), (grammars.w2_grammar, b"ab"), (grammars.w3_grammar, b"ac+bd"),
         (grammars.parens_grammar, b"()"), (grammars.anbn_grammar, b"ab"), (grammars.palindrome_grammar, b"ab"),
         (grammars.nullable_chain_grammar, b"abcd"), (grammars.useless_grammar, b"abcux"),
         (grammars.multibyte_literal_grammar, b"abc()"), (grammars.expr_grammar, b"a1+*()")]


@pytest.mark.parametrize("pruning", [True, False])
@pytest.mark.parametrize("gram,alphabet", SMALL, ids=[s[0].__name__ for s in SMALL])
def test_small_grammars_every_prefix_every_token(gram, alphabet, pruning, zf, oracle_lib):
    """Vocabulary = every string up to length 3 over the alphabet (+ an empty token); the host
    walk must give the oracle's mask after every viable prefix up to length 4, and advance must
    succeed exactly on the allowed tokens, for pruning on and off."""
    g = gram()
    toks = [b""] + list(_all_strings(alphabet, 3 if len(alphabet) <= 4 else 2))
    off, data = wvocab.vocab_csr(toks)
    eng = zf.Engine(g, toks, device=-1, pruning=pruning)
    orc = oracle_lib.Oracle(g)
    n_checked = 0
    for p in [b""] + list(_all_strings(alphabet, 4 if len(alphabet) <= 4 else 3)):
        so = orc.new_state()
        s = eng.new_state()
        ok = so.feed_bytes(p)
        rc = s.try_advance_bytes(p)
        assert (rc == zf.ZF_OK) == ok, p
        if not ok:
            assert rc == zf.ZF_ERR_REJECTED
            continue
        assert s.accepting() == so.accepting(), p
        want = so.mask(off, data, 1)
        assert (s.debug_host_mask_cached()[0] == want).all(), (p, "token-mask cache")
        assert (s.debug_host_mask_automaton()[0] == want).all(), (p, "mask automaton")
        got = s.debug_host_mask()
        assert (got == want).all(), (p, [toks[v] for v in range(len(toks)) if ((int(got[v >> 5]) ^ int(want[v >> 5])) >> (v & 31)) & 1])
        n_checked += 1
        for v in range(0, len(toks), 3):       # advance(t) succeeds <=> bit t was 1; failure leaves the state alone
            c = s.clone()
            before = c.chart()
            rc = c.try_advance(v)
            bit = (int(want[v >> 5]) >> (v & 31)) & 1
            assert (rc == zf.ZF_OK) == bool(bit), (p, toks[v])
            if rc != zf.ZF_OK:
                assert c.chart() == before and c.accepting() == s.accepting()
    assert n_checked >= 3


REGEXES = [grammars.NUMBER_RX.pattern, grammars.STRING_RX.pattern, rb"(ab|a)(bc|c)*", rb"a{2,4}b?", rb"[^a]+|a{3}",
           rb"(a|)b{2,}", rb"x[0-9a-f]{2}\.\x41", rb"[ \t\n\r]+", rb"(a*b|ac)+d?"]


@pytest.mark.parametrize("pattern", REGEXES, ids=[r.decode("latin1")[:30] for r in REGEXES])
def test_regex_dfa_against_oracle_rules(pattern, zf, oracle_lib):
    """The library turns a regex into a DFA, the oracle into grammar rules: the two must accept
    and reject the same random strings (drawn from the pattern's own alphabet plus noise)."""
    g = grammars.regex_only_grammar(pattern)
    eng = zf.Engine(g, [b"a"], device=-1)
    orc = oracle_lib.Oracle(g)
    alphabet = sorted(set(pattern) | set(b'ab01."\\e-+\xc3\xa9\xe2\x82\xac\xf0\x9f\x98\x80 \n'))
    rs = SplitMix64(99)
    for _ in range(1500):
        w = bytes(alphabet[rs.below(len(alphabet))] for _ in range(rs.below(9)))
        so, s = orc.new_state(), eng.new_state()
        ok = so.feed_bytes(w)
        assert (s.try_advance_bytes(w) == zf.ZF_OK) == ok, w
        if ok:
            assert s.accepting() == so.accepting(), w


def test_grammar_errors(zf):
    def expect(code, g, toks=(b"a",)):
        with pytest.raises(zf.ZfError) as ei:
            zf.Engine(g, list(toks), device=-1)
        assert ei.value.code == code, ei.value

    g = Grammar(); g.set_start("S"); g.rule("S", [Rx(rb"a*")])            # terminal matches the empty string
    expect(zf.ZF_ERR_GRAMMAR, g)
    g = Grammar(); g.set_start("S"); g.rule("S", [Rx(rb"a[^\x00-\xff]")])  # empty language
    expect(zf.ZF_ERR_GRAMMAR, g)
    g = Grammar(); g.set_start("S"); g.rule("S", [Rx(rb"(ab")])            # syntax error
    expect(zf.ZF_ERR_GRAMMAR, g)
    g = Grammar(); g.set_start("S"); g.rule("S", [b"a", "S"])              # start derives nothing
    expect(zf.ZF_ERR_GRAMMAR, g)
    g = grammars.w2_grammar(); g.rules.append((0, [17]))                   # bad symbol id
    expect(zf.ZF_ERR_GRAMMAR, g)
    expect(zf.ZF_ERR_INVALID_ARG, grammars.w2_grammar(), [b"x" * 300])     # token longer than 255 bytes


def test_state_errors_and_device_less_engine(zf):
    eng = zf.Engine(grammars.w2_grammar(), [b"a", b"b", b"", b"ab"], device=-1)
    s = eng.new_state()
    assert s.try_advance(7) == zf.ZF_ERR_RANGE and s.try_advance(-1) == zf.ZF_ERR_RANGE
    assert s.try_advance(2) == zf.ZF_ERR_REJECTED          # the empty token
    assert s.try_advance(1) == zf.ZF_ERR_REJECTED
    assert s.stats().bytes_fed == 0
    s.advance(3)
    assert s.accepting() and s.stats().bytes_fed == 2
    s.reset()
    assert not s.accepting() and s.stats().bytes_fed == 0
    with pytest.raises(zf.ZfError) as ei:                    # no CPU substitute for the mask kernels
        eng.compute_mask([s], 16)
    assert ei.value.code == zf.ZF_ERR_DEVICE
    with pytest.raises(zf.ZfError) as ei:
        eng.apply_mask(16, 16, 0, 1, 8, 16)
    assert ei.value.code == zf.ZF_ERR_DEVICE
    lib = zf.load_library()
    assert lib.zf_strerror(zf.ZF_ERR_REJECTED) and lib.zf_compute_mask(None, None, 1, None, None) == zf.ZF_ERR_INVALID_ARG


def _lib_items(eng, state, names):
    """Chart of a library state as {(set, lhs name, rule, dot, origin)} for user rules."""
    items, n_sets = state.chart()
    out = set()
    for k, p, o, q in items:
        lhs, rule, dot = eng.position_info(p)
        if rule >= 0:
            out.add((k, names[lhs], rule, dot, o))
    return out, n_sets


def test_w1_pruned_chart_is_constant_and_unpruned_grows(zf):
    """Section 1 example, grammar A -> A B | B ; B -> a: with pruning the completed (B -> a .)
    disappears as soon as its set is done and nothing but the start set and the current set
    survives, however long the input; without pruning one set per byte is kept."""
    g = grammars.w1_grammar()
    pr = zf.Engine(g, [b"a"], device=-1, pruning=True)
    un = zf.Engine(g, [b"a"], device=-1, pruning=False)
    sp, su = pr.new_state(), un.new_state()
    sizes = []
    for n in range(1, 40):
        sp.advance(0)
        su.advance(0)
        assert sp.accepting() and su.accepting()
        st = sp.stats()
        sizes.append((st.n_sets, st.n_items))
        assert su.stats().n_sets == n + 1
        items, _ = _lib_items(pr, sp, g.nonterminals)
        # rule 0 is A -> A B: the only user item that must survive is (A -> A . B, origin 0) in the last set
        assert (st.n_sets - 1, "A", 0, 1, 0) in items
        assert not any(dot == 1 and lhs == "B" for _, lhs, _, dot, _ in items)      # (B -> a .) is gone
    assert len(set(sizes)) == 1 and sizes[0][0] <= 2, sizes
    assert su.stats().n_items > 5 * sp.stats().n_items


def test_hrr_only_grammar_keeps_chart_bounded(zf):
    """Rules of the forms A -> c, A -> B a, A -> eps only (Section 4.1, high-level regular rules):
    the pruned chart must not grow with the input."""
    g = Grammar(); g.set_start("L")
    g.alts("L", [], ["L", "I"])             # list of items: L -> eps | L I
    g.alts("I", [b"x"], ["P", b";"])        # I -> c | B a
    g.alts("P", [b"y"], ["P", b"y"])
    eng = zf.Engine(g, [b"x", b"y", b";"], device=-1)
    s = eng.new_state()
    rs = SplitMix64(5)
    sizes = []
    text = b""
    for _ in range(300):
        m = s.debug_host_mask()
        allowed = [v for v in range(3) if (int(m[0]) >> v) & 1]
        v = allowed[rs.below(len(allowed))]
        s.advance(v)
        sizes.append(s.stats().n_items)
    assert max(sizes) <= 8, max(sizes)


@pytest.mark.parametrize("idx,rows,steps,every", [(1, 1, 64, 1), (2, 1, 256, 8), (3, 2, 200, 25), (4, 2, 120, 20), (5, 2, 96, 12)])
def test_config_trajectories_host_walk_matches_oracle(idx, rows, steps, every, zf, oracle_lib):
    """Replay the oracle-sampled trajectory of each configuration; at sampled steps the host walk
    of the compiled tables (pruning on and off) must reproduce the oracle's mask bit for bit, and
    advance must accept exactly the tokens the oracle fed."""
    cfg = configs.CONFIGS[idx]
    toks = cfg.vocab()
    traj = load_trajectory(idx, rows, steps)
    off, data = wvocab.vocab_csr(toks)
    g = cfg.grammar()
    orc = oracle_lib.Oracle(g)
    engines = [zf.Engine(g, toks, device=-1, pruning=True), zf.Engine(g, toks, device=-1, pruning=False)]
    for b in range(rows):
        so = orc.new_state()
        ss = [e.new_state() for e in engines]
        for step, ids in enumerate(traj):
            t = ids[b]
            if t < 0:
                so = orc.new_state()
                for s in ss:
                    s.reset()
            else:
                assert so.feed_bytes(toks[t])
                for s in ss:
                    s.advance(t)
            if step % every == 0:
                want = so.mask(off, data, 8)
                for s in ss:
                    assert (s.debug_host_mask() == want).all(), (idx, b, step)
                    assert (s.debug_host_mask_cached()[0] == want).all(), (idx, b, step, "token-mask cache")
                    got, st = s.debug_host_mask_automaton()
                    assert (got == want).all(), (idx, b, step, "mask automaton")
                    assert st["steps"] <= st["lookups"] and st["states"] <= st["steps"]   # at most one Earley step per new transition
                    assert s.accepting() == so.accepting()
        assert ss[0].stats().n_items <= ss[1].stats().n_items


@pytest.mark.parametrize("idx,rows,steps,every", [(1, 1, 64, 1), (2, 1, 256, 8), (3, 4, 300, 25), (4, 3, 120, 20), (5, 2, 96, 12)])
def test_persistent_automaton_twin_matches_oracle(idx, rows, steps, every, zf, oracle_lib):
    """One automaton for all rows and steps, states named by content: feeding the trajectory's tokens is a walk
    through it, and at sampled steps the mask computed from the reached state equals the oracle's.  States and
    transitions made for one row or step serve the others."""
    cfg = configs.CONFIGS[idx]
    toks = cfg.vocab()
    traj = load_trajectory(idx, rows, steps)
    off, data = wvocab.vocab_csr(toks)
    g = cfg.grammar()
    orc = oracle_lib.Oracle(g)
    eng = zf.Engine(g, toks, device=-1)
    tw = zf.Twin(eng)
    so = [orc.new_state() for _ in range(rows)]
    st = [0] * rows
    per_mask = []
    for step, ids in enumerate(traj):
        for b in range(rows):
            t = ids[b]
            if t < 0:
                so[b], st[b] = orc.new_state(), 0
                continue
            assert so[b].feed_bytes(toks[t])
            rc, st[b], acc = tw.advance(st[b], toks[t])
            assert rc == 0 and acc == so[b].accepting(), (idx, b, step)
        if step % every == 0 or step == steps - 1:
            for b in range(rows):
                got, info = tw.mask(st[b])
                assert (got == so[b].mask(off, data, 8)).all(), (idx, b, step)
                per_mask.append(info["steps"])
    # a token the oracle rejects is rejected here too, and the state stays where it was
    want = so[0].mask(off, data, 8)
    bad = next(v for v in range(len(toks)) if toks[v] and not (want[v >> 5] >> (v & 31)) & 1)
    rc, same, _ = tw.advance(st[0], toks[bad])
    assert rc == zf.ZF_ERR_REJECTED and same == st[0]
    assert info["states"] < 40 * steps * rows and sum(per_mask) > 0


def test_advance_batch_equals_row_by_row():
    """zf_advance_batch: same charts as advancing every row on its own; negative ids reset a row;
    a rejected row is reported, left unchanged, and does not stop the others."""
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[1]
    toks = cfg.vocab()
    eng = zf.Engine(cfg.grammar(), toks, device=-1)
    traj = load_trajectory(1, 1, 40)
    one, many = eng.new_state(), zf.StateBatch([eng.new_state() for _ in range(3)])
    for ids in traj:
        t = ids[0]
        one.reset() if t < 0 else one.advance(t)
        many.advance([t, t, t])
        for s in many:
            assert s.chart() == one.chart() and s.accepting() == one.accepting()
    before = many[1].chart()
    bad = next(v for v in range(len(toks)) if one.clone().try_advance(v) == zf.ZF_ERR_REJECTED)
    good = traj[0][0]
    with pytest.raises(zf.ZfError) as ei:
        many.advance([-1, bad, -1])
    assert ei.value.code == zf.ZF_ERR_REJECTED
    assert many[1].chart() == before
    fresh = eng.new_state()
    assert many[0].chart() == fresh.chart() and many[2].chart() == fresh.chart()
    many.advance([good, -1, good])
    fresh.advance(good)
    assert many[0].chart() == fresh.chart() and many[2].chart() == fresh.chart()


def test_advance_batch_of_wide_charts_on_worker_threads():
    """A batch whose rows are expensive to feed (wide sets of the ambiguous expression grammar) is dealt to
    worker threads: same charts as row by row, over several calls; a rejected row keeps its chart, is
    reported with its own error text, and does not stop the others; a state named twice is fed twice."""
    import paper_2506_01151_amd as zf
    cfg = configs.CONFIGS[5]
    toks = cfg.vocab(3000)
    eng = zf.Engine(cfg.grammar(), toks, device=-1)
    plus, star, a, seven, close = (toks.index(t) for t in (b"+", b"*", b"a", b"7", b")"))
    rows = 12
    singles = [eng.new_state() for _ in range(rows)]
    many = zf.StateBatch([eng.new_state() for _ in range(rows)])
    for b in range(rows):
        prefix = b"x" + (b"+y" if b % 2 else b"*3") * (60 + 7 * b)
        singles[b].advance_bytes(prefix)
        many[b].advance_bytes(prefix)
    for step in range(6):
        ids = [(plus, a, star, seven, -1, a)[(step + (b % 3 == 0)) % 6] if step % 2 == 0 else (a, plus, seven, star, plus, a)[(step + (b % 3 == 0)) % 6] for b in range(rows)]
        ok = []
        for b in range(rows):
            if ids[b] < 0:
                singles[b].reset()
                ok.append(True)
            else:
                ok.append(singles[b].try_advance(ids[b]) == zf.ZF_OK)
        if all(ok):
            many.advance(ids)
        else:
            with pytest.raises(zf.ZfError) as ei:
                many.advance(ids)
            assert ei.value.code == zf.ZF_ERR_REJECTED and "cannot extend" in str(ei.value)
        for b in range(rows):
            assert many[b].chart() == singles[b].chart() and many[b].accepting() == singles[b].accepting(), (step, b)
    # a state named twice in one batch: fed twice, in order
    twice = zf.StateBatch([many[1], many[1], many[2], many[3], many[4]])
    ref = singles[1]
    t1 = plus if ref.clone().try_advance(plus) == zf.ZF_OK else a
    ref.advance(t1)
    t2 = a if ref.clone().try_advance(a) == zf.ZF_OK else plus
    ref.advance(t2)
    twice.advance([t1, t2, -1, -1, -1])
    assert many[1].chart() == ref.chart()


def test_advance_through_the_host_automaton_equals_plain_advance():
    """With walk_mode 2 zf_advance walks the token's bytes through the engine's automaton of Earley sets (a look-up per byte
    once a transition is known) and brings the chart up to date only when somebody reads it.  Same acceptance at every step,
    same charts and statistics, same rejections as the plain Scan/Complete/Compact advance of a walk_mode 0 engine: along
    sentences with long sums (wide sets, several threads at work in one batch), twice over (the second time every transition
    is known), with clones and resets on the way."""
    import paper_2506_01151_amd as zf
    from workloads.sentences import expr_sentence, cut_into_tokens
    cfg = configs.CONFIGS[5]
    toks = cfg.vocab(6000)
    rows, steps = 16, 160
    seqs = [cut_into_tokens(toks, expr_sentence(cfg.seed, f"host[{b}]", 4 * steps + 64, flat=b % 4 != 3), steps) for b in range(rows)]
    fast, plain = (zf.Engine(cfg.grammar(), toks, device=-1, walk_mode=m) for m in (2, 0))
    bad = toks.index(b")")
    for again in range(2):
        bf, bp = (zf.StateBatch([e.new_state() for _ in range(rows)]) for e in (fast, plain))
        at = [0] * rows                                            # where every row stands in its sentence
        for k in range(steps):
            ids = [seqs[b][at[b]] for b in range(rows)]
            if k == 50:
                ids[3], at[3] = -1, -1                             # a reset on the way: the row starts its sentence again
            if k == 100 + 20 * again:
                fast.clear_state_cache()                           # the automaton is emptied under the rows' feet: they come back in through their charts
            bf.advance(ids)
            bp.advance(ids)
            at = [x + 1 for x in at]
            for b in range(rows):
                assert bf[b].accepting() == bp[b].accepting(), (again, k, b)
            if k in (0, 7, 50, 51, 120, steps - 1):
                for b in range(0, rows, 3):
                    assert bf[b].chart() == bp[b].chart(), (again, k, b)
                    sf, sp = bf[b].stats(), bp[b].stats()
                    assert (sf.n_sets, sf.n_items, sf.items_created, sf.bytes_fed) == (sp.n_sets, sp.n_items, sp.items_created, sp.bytes_fed)
            if k == 90:
                cf, cp = bf[5].clone(), bp[5].clone()              # a clone goes its own way
                for t in seqs[5][at[5]:at[5] + 20]:
                    cf.advance(t)
                    cp.advance(t)
                assert cf.chart() == cp.chart() and cf.accepting() == cp.accepting()
                for t in (bad, toks.index(b"+"), toks.index(b"("), toks.index(b"7"), toks.index(b"q")):
                    rf, rp = bf[6].clone().try_advance(t), bp[6].clone().try_advance(t)   # what one refuses the other refuses ...
                    assert rf == rp, t
                # ... and a refused token moves nothing
                sf, sp = bf[7].clone(), bp[7].clone()
                first_bad = next(t for t in range(len(toks)) if sp.clone().try_advance(t) == zf.ZF_ERR_REJECTED)
                assert sf.try_advance(first_bad) == zf.ZF_ERR_REJECTED and sp.try_advance(first_bad) == zf.ZF_ERR_REJECTED
                assert sf.chart() == sp.chart() == bp[7].chart() and sf.accepting() == sp.accepting()


@pytest.mark.parametrize("seed", range(48))
def test_random_grammars_host_walk_equals_oracle(seed, zf, oracle_lib):
    """Differential test on seeded random grammars (empty rules, unit cycles, recursion of every
    kind, ambiguity): along an oracle-sampled trajectory the host walk of the compiled tables,
    with and without the token-mask cache and with pruning on and off, gives the oracle's mask,
    and advance/accepting agree."""
    from workloads import random_grammars
    g = random_grammars.random_grammar(seed)
    toks = random_grammars.random_vocab(seed)
    orc = oracle_lib.Oracle(g)
    run = OracleRun(orc, toks, [stream(seed, "random-walk")], n_threads=1)
    engines = [zf.Engine(g, toks, device=-1, pruning=p) for p in (True, False)]
    states = [e.new_state() for e in engines]
    for step in range(24):
        want = run.masks()[0]
        for s in states:
            assert (s.debug_host_mask() == want).all(), (seed, step)
            assert (s.debug_host_mask_cached()[0] == want).all(), (seed, step, "token-mask cache")
            assert (s.debug_host_mask_automaton()[0] == want).all(), (seed, step, "mask automaton")
            assert s.accepting() == run.states[0].accepting(), (seed, step)
        t = run.step(want[None, :])[0]
        for s in states:
            s.reset() if t < 0 else s.advance(t)


def test_automaton_twin_long_tokens_deep_nesting_many_classes(zf, oracle_lib):
    """The mask automaton's host twin on the inputs that stress its ends: tokens longer than 16 bytes, nesting
    deeper than any state budget, more than 64 byte classes."""
    from tests.helpers import edge_vocab_json
    g = grammars.json_grammar()
    toks = edge_vocab_json()
    off, data = wvocab.vocab_csr(toks)
    orc = oracle_lib.Oracle(g)
    eng = zf.Engine(g, toks, device=-1)
    for p in [b"", b"[", b'{"k":"', b"[1,", b'[[{"a":[', b'{"k":"v', b"[1", b'["\\']:
        o, s = orc.new_state(), eng.new_state()
        assert o.feed_bytes(p)
        s.advance_bytes(p)
        got, st = s.debug_host_mask_automaton()
        assert (got == o.mask(off, data, 4)).all(), p
        if p == b"[":
            assert st["states"] > 64      # every nesting depth is a state of its own
    g2 = grammars.many_classes_grammar(100)
    toks2 = [bytes([c]) for c in range(256)] + [bytes([32 + c, 32 + (c * 7 + 3) % 100]) for c in range(100)] + [bytes([32 + c, 32 + (c * 7 + 3) % 100, 32 + (c * 5) % 100]) for c in range(100)]
    off2, data2 = wvocab.vocab_csr(toks2)
    orc2 = oracle_lib.Oracle(g2)
    eng2 = zf.Engine(g2, toks2, device=-1)
    assert eng2.info.n_byte_classes > 64
    for p in [b"", bytes([40]), bytes([40, 32 + (8 * 7 + 3) % 100]), bytes([41, 32 + (9 * 7 + 3) % 100, 50])]:
        o, s = orc2.new_state(), eng2.new_state()
        assert o.feed_bytes(p)
        s.advance_bytes(p)
        assert (s.debug_host_mask_automaton()[0] == o.mask(off2, data2, 4)).all(), p
