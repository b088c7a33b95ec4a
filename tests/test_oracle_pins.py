"""Pins for the CPU oracle: it is checked against things other than itself.

  * the worked examples the paper prints (tests/golden/*.txt, each with its citation);
  * membership and viable prefixes by brute force: a recognizer written directly from the
    definition of derivation (least fixed point of "X derives w[i:j]"), run on EVERY string
    over a small alphabet up to a length bound;
  * the regular special case (a grammar that is one regex terminal) against Python's `re`;
  * the JSON grammar against Python's `json` in strict mode on seeded documents and mutations;
  * invariants of the mask; the closed form of logit masking.
"""
import itertools
import json
import os
import re

import numpy as np
import pytest

from workloads import grammars, vocab as wvocab
from workloads.grammar import Lit
from workloads.rng import SplitMix64, stream
from oracle import Oracle
from oracle.frontend import apply_mask, parse_regex

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------------------
# golden fixtures
def _read_golden(name):
    exact, contains, info = {}, [], {}
    mode = None
    for line in open(os.path.join(GOLDEN, name)):
        line = line.rstrip("\n")
        if not line or line.startswith("#"):
            continue
        if line.split(":")[0] in ("grammar", "input", "accept"):
            key, _, val = line.partition(":")
            info[key.strip()] = val.strip()
        elif "|" in line:
            k, lhs, rhs, dot, org = [x.strip() for x in line.split("|")]
            item = (int(k), lhs, tuple(rhs.split()), int(dot), int(org))
            (exact.setdefault(int(k), []) if mode == "exact" else contains).append(item)
        elif line.startswith("set") and "exact" in line:
            mode = "exact"
        elif "contains" in line:
            mode = "contains"
    return info, exact, contains


def _user_items(state, k):
    """Items of S[k] whose rule belongs to the user grammar, with byte symbols as text."""
    out = set()
    for lhs, rhs, dot, org in state.set_items(k):
        if lhs == "S'" or "#" in lhs:
            continue
        out.add((k, lhs, tuple(s.decode() if isinstance(s, bytes) else s for s in rhs), dot, org))
    return out


@pytest.mark.parametrize("fixture,gram", [("w1_left_recursion.txt", grammars.w1_grammar),
                                          ("w2_sequence.txt", grammars.w2_grammar),
                                          ("w3_figure1.txt", grammars.w3_grammar)])
def test_paper_worked_examples(fixture, gram, oracle_lib):
    info, exact, contains = _read_golden(fixture)
    o = Oracle(gram())
    s = o.new_state()
    for b in info["input"].encode():
        assert s.feed(b)
    for k, items in exact.items():
        assert _user_items(s, k) == set(items), f"S[{k}] differs"
    for it in contains:
        assert it in _user_items(s, it[0]), f"{it} missing"
    if info.get("accept") == "yes":
        assert s.accepting()


def test_w3_rejections(oracle_lib):
    o = Oracle(grammars.w3_grammar())
    for w, viable, accept in [(b"a+d", 1, 1), (b"c+b", 1, 1), (b"a+", 1, 0), (b"a", 1, 0), (b"", 1, 0),
                              (b"a+a", 0, 0), (b"b+d", 0, 0), (b"a+d+", 0, 0), (b"+", 0, 0)]:
        s = o.new_state()
        ok = s.feed_bytes(w)
        assert ok == bool(viable), w
        if ok:
            assert s.accepting() == bool(accept), w


# ---------------------------------------------------------------------------------------
# brute force from the definition of derivation
def _term_match(term, piece: bytes) -> bool:
    if isinstance(term, Lit):
        return piece == term.data
    return re.fullmatch(term.pattern, piece, re.DOTALL) is not None


def derives(g, w: bytes) -> bool:
    """w in L(g), by iterating 'X =>* w[i:j]' to its least fixed point."""
    n = len(w)
    T = set()
    tm = {}

    def match_sym(s, i, j):
        if s >= 0:
            return (s, i, j) in T
        key = (s, i, j)
        if key not in tm:
            tm[key] = _term_match(g.terminals[~s], w[i:j])
        return tm[key]

    changed = True
    while changed:
        changed = False
        for lhs, rhs in g.rules:
            for i in range(n + 1):
                ends = {i}
                for s in rhs:
                    ends = {k2 for k in ends for k2 in range(k, n + 1) if match_sym(s, k, k2)}
                    if not ends:
                        break
                for j in ends:
                    if (lhs, i, j) not in T:
                        T.add((lhs, i, j))
                        changed = True
    return (g.start, 0, n) in T


def _all_strings(alphabet: bytes, max_len: int):
    for n in range(max_len + 1):
        for tup in itertools.product(alphabet, repeat=n):
            yield bytes(tup)


# (grammar, alphabet, n = prefix length bound, N = n + completion bound)
BRUTE = [
    (grammars.w1_grammar, b"ab", 5, 6),
    (grammars.w2_grammar, b"ab", 3, 3),
    (grammars.parens_grammar, b"()", 5, 10),
    (grammars.anbn_grammar, b"ab", 4, 8),
    (grammars.palindrome_grammar, b"ab", 4, 8),
    (grammars.nullable_chain_grammar, b"abcd", 4, 5),
    (grammars.useless_grammar, b"abcux", 4, 5),
    (grammars.multibyte_literal_grammar, b"abc()", 2, 5),
    (grammars.expr_grammar, b"a1+(", 2, 2),   # only membership/viability up to what N covers, see below
]


@pytest.mark.parametrize("gram,alphabet,n,N", BRUTE, ids=[b[0].__name__ for b in BRUTE])
def test_membership_and_viable_prefix_brute_force(gram, alphabet, n, N, oracle_lib):
    g = gram()
    o = Oracle(g)
    if gram is grammars.expr_grammar:
        alphabet, n, N = b"a1+()", 2, 6     # "((" needs "a))": every viable prefix <= 2 completes within 6
    language = {w for w in _all_strings(alphabet, N) if derives(g, w)}
    prefixes = {w[:k] for w in language for k in range(len(w) + 1)}
    assert language, "test grammar has an empty language below the bound"
    for w in _all_strings(alphabet, N):
        s = o.new_state()
        ok = s.feed_bytes(w)
        if len(w) <= n:
            assert ok == (w in prefixes), f"viable({w!r})"
        if ok:
            assert s.accepting() == (w in language), f"accepting({w!r})"
        else:
            assert w not in language, f"oracle lost the sentence {w!r}"
    # token-level check: check(p, t) <=> p.t is a viable prefix, state untouched
    toks = [t for t in _all_strings(alphabet, 2) if t]
    for p in _all_strings(alphabet, n - 2):
        s = o.new_state()
        if not s.feed_bytes(p):
            continue
        before = (s.n_sets(), s.n_items())
        for t in toks:
            assert s.check(t) == (p + t in prefixes), (p, t)
        assert (s.n_sets(), s.n_items()) == before
        assert not s.check(b"")


def language_by_length(g, alphabet: bytes, N: int):
    """{w over the alphabet, |w| <= N : start =>* w}, as the least solution of the grammar's language
    equations L(X) = union over rules X -> s1 ... sm of L(s1) ... L(sm), iterated to its fixed point with
    every string longer than N discarded (concatenation never shortens).  Returns the set for the start symbol."""
    letters = sorted(set(alphabet))
    short = [bytes(t) for k in range(1, 4) for t in itertools.product(letters, repeat=k)]
    term_sets = []
    for t in g.terminals:
        if isinstance(t, Lit):
            term_sets.append({t.data} if len(t.data) <= N and set(t.data) <= set(letters) else set())
            continue
        # bytes that occur in some short match; longer matches are enumerated over those only (checked below for lengths <= 4)
        used = sorted({c for w in short if _term_match(t, w) for c in w})
        m = {bytes(w) for k in range(1, N + 1) for w in itertools.product(used, repeat=k) if _term_match(t, bytes(w))}
        full4 = {bytes(w) for k in range(1, 5) for w in itertools.product(letters, repeat=k) if _term_match(t, bytes(w))}
        assert {w for w in m if len(w) <= 4} == full4, "a byte of this terminal only shows up in matches longer than 3"
        term_sets.append(m)
    L = [set() for _ in g.nonterminals]
    changed = True
    while changed:
        changed = False
        for lhs, rhs in g.rules:
            cur = {b""}
            for sym in rhs:
                part = L[sym] if sym >= 0 else term_sets[~sym]
                cur = {u + v for u in cur for v in part if len(u) + len(v) <= N}
                if not cur:
                    break
            if not cur <= L[lhs]:
                L[lhs] |= cur
                changed = True
    return L[g.start]


def test_expr_grammar_brute_force_to_length_four(oracle_lib):
    """The ambiguous expression grammar, deeper than the table above reaches: every string of up to 6 bytes over
    a 1 + * ( ) through the oracle.  A viable prefix of 4 bytes is completed within 5 more ("((((" needs "a))))"), so the
    language up to 9 bytes decides viability for every prefix of up to 4 bytes exactly."""
    g = grammars.expr_grammar()
    alphabet, n, N = b"a1+*()", 4, 9
    language = language_by_length(g, alphabet, N)
    for w in _all_strings(alphabet, 5):                       # the two brute-force recognizers agree where both are affordable
        assert (w in language) == derives(g, w), w
    prefixes = {w[:k] for w in language for k in range(min(len(w), n) + 1)}
    o = Oracle(g)
    n_viable = 0
    for w in _all_strings(alphabet, 6):
        s = o.new_state()
        ok = s.feed_bytes(w)
        if len(w) <= n:
            assert ok == (w in prefixes), f"viable({w!r})"
            n_viable += ok
        if ok:
            assert s.accepting() == (w in language), f"accepting({w!r})"
        else:
            assert w not in language, f"oracle lost the sentence {w!r}"
    assert n_viable > 100
    long_ones = sorted(w for w in language if len(w) > 6)
    assert len(long_ones) > 8000
    rs = stream(17, "expr-long-sentences")
    for _ in range(4000):                                     # sentences of 7-9 bytes: sums and products of sums, many parse trees each
        w = long_ones[rs.below(len(long_ones))]
        s = o.new_state()
        assert s.feed_bytes(w) and s.accepting(), w
        bad = w[:-1] + (b")" if w[-1:] != b")" else b"+")     # one byte changed at the end: still decided by the enumerated language
        s = o.new_state()
        if s.feed_bytes(bad):
            assert s.accepting() == (bad in language), bad
        else:
            assert bad not in language, bad
    toks = [t for t in _all_strings(alphabet, 2) if t]
    for p in _all_strings(alphabet, n - 2):
        s = o.new_state()
        if not s.feed_bytes(p):
            continue
        before = (s.n_sets(), s.n_items())
        for t in toks:
            assert s.check(t) == (p + t in prefixes), (p, t)
        assert (s.n_sets(), s.n_items()) == before


def test_nullable_sets(oracle_lib):
    o = Oracle(grammars.nullable_chain_grammar())
    assert [o.nullable(x) for x in "SABC"] == [False, True, True, True]
    o = Oracle(grammars.parens_grammar())
    assert o.nullable("S")
    o = Oracle(grammars.json_grammar())
    assert o.nullable("ws") and not o.nullable("value") and not o.nullable("json")


def test_useless_rules_removed_and_unproductive_start_rejected(oracle_lib):
    o = Oracle(grammars.useless_grammar())
    s = o.new_state()
    assert not s.check(b"u")        # U never terminates: 'u' must not look viable
    assert s.check(b"a") and s.check(b"b") and not s.check(b"x")
    from workloads.grammar import Grammar
    g = Grammar()
    g.set_start("S")
    g.rule("S", [b"a", "S"])
    with pytest.raises(ValueError):
        Oracle(g)


# ---------------------------------------------------------------------------------------
# regular special case against the library regex engine
REGEXES = [
    (grammars.NUMBER_RX.pattern, b"-01.e", 5, 2),
    (grammars.INTEGER_RX.pattern, b"-01", 5, 1),
    (rb"(ab|a)(bc|c)*", b"abc", 6, 1),
    (rb"a{2,4}b?", b"ab", 6, 2),
    (rb"[^a]+|a{3}", b"ab", 5, 2),
    (rb"(a|)b{2,}", b"ab", 5, 2),
    (rb"x[0-9a-f]{2}\.\x41", b"x0f.A", 5, 4),
]


@pytest.mark.parametrize("pattern,alphabet,n,c", REGEXES, ids=[r[0].decode("latin1") for r in REGEXES])
def test_single_regex_terminal_equals_re(pattern, alphabet, n, c, oracle_lib):
    o = Oracle(grammars.regex_only_grammar(pattern))
    rx = re.compile(pattern, re.DOTALL)
    full = {w for w in _all_strings(alphabet, n + c) if rx.fullmatch(w)}
    prefixes = {w[:k] for w in full for k in range(len(w) + 1)}
    for w in _all_strings(alphabet, n):
        s = o.new_state()
        ok = s.feed_bytes(w)
        assert ok == (w in prefixes), w
        if ok:
            assert s.accepting() == (w in full), w


def test_regex_classes_match_re(oracle_lib):
    """Every class / escape form of the dialect selects the same bytes as `re` does."""
    for src in [rb'[^"\\\x00-\x1f\x80-\xff]', rb"[ \t\n\r]", rb"[-+]", rb"[a-z0-9_]", rb".", rb"\.", rb"\x7f",
                rb"[\xc2-\xdf]", rb"[^\x00-\xfe]", rb"[\]a]", rb"[a\-c]"]:
        node = parse_regex(src)
        assert node[0] == "set"
        want = {b for b in range(256) if re.fullmatch(src, bytes([b]), re.DOTALL)}
        assert set(node[1]) == want, src


# ---------------------------------------------------------------------------------------
# JSON grammar against the host JSON library (strict mode)
def _strict_json_ok(w: bytes) -> bool:
    def no_const(_):
        raise ValueError("non-finite spelling")
    try:
        json.loads(w.decode("utf-8"), parse_constant=no_const)
        return True
    except (ValueError, RecursionError):
        return False


def _rand_json(rs, depth=0):
    ws = lambda: b"".join(bytes([b" \t\n\r"[rs.below(4)]]) for _ in range(rs.below(3) if rs.below(3) == 0 else 0))
    k = rs.below(8 if depth < 3 else 6)
    if k == 0:
        return [b"true", b"false", b"null"][rs.below(3)]
    if k in (1, 2):
        parts = [b"-"] if rs.below(3) == 0 else []
        parts.append(b"0" if rs.below(4) == 0 else str(1 + rs.below(99999)).encode())
        if rs.below(3) == 0:
            parts.append(b"." + str(rs.below(1000)).encode())
        if rs.below(4) == 0:
            parts.append([b"e", b"E"][rs.below(2)] + [b"", b"+", b"-"][rs.below(3)] + str(rs.below(40)).encode())
        return b"".join(parts)
    if k in (3, 4, 5):
        out = b'"'
        for _ in range(rs.below(6)):
            c = rs.below(10)
            if c < 5:
                out += bytes([0x20 + rs.below(0x5F)]).replace(b'"', b"q").replace(b"\\", b"/")
            elif c < 7:
                out += chr(0x80 + rs.below(0x2000)).encode("utf-8")
            elif c == 7:
                out += chr(0x10000 + rs.below(0x1000)).encode("utf-8")
            elif c == 8:
                out += b"\\" + bytes([b'"\\/bfnrt'[rs.below(8)]])
            else:
                out += b"\\u" + ("%04x" % rs.below(0x10000)).encode()
        return out + b'"'
    if k == 6:
        items = [_rand_json(rs, depth + 1) for _ in range(rs.below(4))]
        return b"[" + ws() + (ws() + b"," + ws()).join(items) + ws() + b"]"
    items = [_rand_json(rs, 9) if False else (b'"k%d"' % rs.below(9)) + ws() + b":" + ws() + _rand_json(rs, depth + 1)
             for _ in range(rs.below(4))]
    return b"{" + ws() + (ws() + b"," + ws()).join(items) + ws() + b"}"


def test_json_grammar_agrees_with_json_library(oracle_lib):
    o = Oracle(grammars.json_grammar())
    rs = SplitMix64(20250601)
    docs = [_rand_json(rs) for _ in range(150)]
    pool = b'{}[]:,"\\ \n0123456789-+.eEtruefalsn\xc3\xa9\xe2\x82\xac\xf0\x9f\x98\x80\x80\xff\x1f'
    cases = list(docs)
    for d in docs:
        for _ in range(4):
            m = bytearray(d)
            op = rs.below(3)
            pos = rs.below(len(m) + 1)
            if op == 0 and m:
                del m[min(pos, len(m) - 1)]
            elif op == 1:
                m.insert(pos, pool[rs.below(len(pool))])
            elif m:
                m[min(pos, len(m) - 1)] = pool[rs.below(len(pool))]
            cases.append(bytes(m))
    cases += [bytes(pool[rs.below(len(pool))] for _ in range(1 + rs.below(6))) for _ in range(300)]
    n_yes = 0
    for w in cases:
        s = o.new_state()
        got = s.feed_bytes(w) and s.accepting()
        want = _strict_json_ok(w)
        assert got == want, w
        n_yes += want
    assert n_yes >= 150 and n_yes < len(cases) - 150     # both verdicts are exercised
    for d in docs[:40]:                                  # every prefix of a sentence is viable
        s = o.new_state()
        for b in d:
            assert s.feed(b), d


# ---------------------------------------------------------------------------------------
# mask: definition, invariants
def test_mask_bits_follow_definition_and_invariants(oracle_lib):
    g = grammars.json_grammar()
    o = Oracle(g)
    toks = wvocab.make_vocab(7, 3000, uniform_2_8=False, non_ascii=True) + [b"", b'"a', b'"', b'"ab', b'"a']
    off, data = wvocab.vocab_csr(toks)
    V = len(toks)
    for prefix in [b"", b'{"a', b'{"a":', b"[1", b'{"k": [true, ', b'"\xe2\x82']:
        s = o.new_state()
        assert s.feed_bytes(prefix)
        m = s.mask(off, data, 2)
        assert m.shape == ((V + 31) // 32,)
        bit = lambda v: (int(m[v >> 5]) >> (v & 31)) & 1
        index = {}
        for v, t in enumerate(toks):
            index.setdefault(t, []).append(v)
        for v, t in enumerate(toks):
            # the bit is the byte-at-a-time verdict on a fresh copy of the state
            c = s.clone()
            want = len(t) > 0 and all(c.feed(b) for b in t)
            assert bit(v) == int(want), (prefix, t)
            if bit(v):       # prefix closure over the vocabulary
                for k in range(1, len(t)):
                    for u in index.get(t[:k], []):
                        assert bit(u), (prefix, t, t[:k])
            assert all(bit(u) == bit(v) for u in index[t])          # duplicates agree
        for v in range(V, len(m) * 32):
            assert bit(v) == 0                                        # padding bits are zero
        # composition: allowed(p, t1 t2) = allowed(p, t1) and allowed(p t1, t2)
        for t1 in (b'"', b"1", b" ", b"[", b"a"):
            c = s.clone()
            ok1 = c.feed_bytes(t1)
            for t2 in (b"a", b'"', b",", b"0", b"]"):
                assert s.check(t1 + t2) == (ok1 and c.check(t2))


def test_toy_json_mask_after_open_brace(oracle_lib):
    """Section 3.3: after '{' of an object only '"' (a key) or '}' may follow (plus blanks here,
    because this grammar allows white space inside the braces)."""
    o = Oracle(grammars.json_grammar())
    s = o.new_state()
    assert s.feed(ord("{"))
    allowed = {b for b in range(256) if s.check(bytes([b]))}
    assert allowed == set(b'"} \t\n\r')


# ---------------------------------------------------------------------------------------
# logit masking: closed form
@pytest.mark.parametrize("dtype,neg_inf", [(np.uint32, 0xFF800000), (np.uint16, 0xFF80)])
def test_apply_mask_closed_form(dtype, neg_inf, oracle_lib):
    rng = np.random.default_rng(3)
    B, V = 3, 1000 + 13
    W = (V + 31) // 32
    logits = rng.integers(0, np.iinfo(dtype).max, size=(B, V), dtype=dtype)   # arbitrary bit patterns, NaNs included
    mask = rng.integers(0, 2**32, size=(B, W), dtype=np.uint32)
    bits = np.unpackbits(mask.view(np.uint8).reshape(B, -1), axis=1, bitorder="little")[:, :V].astype(bool)
    want = np.where(bits, logits, dtype(neg_inf))
    got = apply_mask(logits, mask)
    assert got.tobytes() == want.tobytes()
    assert apply_mask(got, mask).tobytes() == got.tobytes()                       # idempotent
    ones = np.full((B, W), 0xFFFFFFFF, dtype=np.uint32)
    assert apply_mask(logits, ones).tobytes() == logits.tobytes()                 # identity
    assert (apply_mask(logits, np.zeros((B, W), np.uint32)) == neg_inf).all()     # all -inf
    if dtype is np.uint32:
        assert np.isneginf(np.array([neg_inf], dtype=np.uint32).view(np.float32))[0]
    else:
        assert np.isneginf((np.array([neg_inf], dtype=np.uint32) << 16).view(np.float32))[0]


# ---------------------------------------------------------------------------------------
# the description of configuration 5's language that the full-length GPU test compares with (tests/expr_language.py)
def test_expr_language_description_against_the_oracle(oracle_lib):
    """tests/expr_language.py states the viable prefixes of E -> E+E | E*E | (E) | num | id directly (operands and operators
    alternate, parentheses balance).  Here the Earley oracle pins it: equal masks and equal `accepting` at every step of
    seeded sentences cut into tokens of configuration 5's vocabulary, and along the first steps of the oracle-sampled
    trajectory of configuration 5 (tokens drawn from the oracle's own masks: nested parentheses, odd token boundaries),
    every token of which the description must accept."""
    from tests.expr_language import ExprLanguage, ExprRow
    from tests.helpers import load_trajectory
    from workloads import configs
    from workloads.sentences import expr_sentence, cut_into_tokens
    cfg = configs.CONFIGS[5]
    o = Oracle(cfg.grammar())
    toks = cfg.vocab(8192)
    off, data = wvocab.vocab_csr(toks)
    lang = ExprLanguage(toks)
    for r in range(8):
        ids = cut_into_tokens(toks, expr_sentence(cfg.seed, f"pin[{r}]", 240, max_depth=3 + r), 70)
        s, row = o.new_state(), ExprRow()
        assert (s.mask(off, data, 8) == lang.mask(row.mode, row.depth)).all()
        for k, i in enumerate(ids):
            assert s.feed_bytes(toks[i]) and row.feed(toks[i]), (r, k)
            assert (s.mask(off, data, 8) == lang.mask(row.mode, row.depth)).all(), (r, k)
            assert s.accepting() == row.accepting(), (r, k)
        for bad in (b")" * (row.depth + 1), b"+*", b"1a", b"a1", b"A", b"()", b" "):      # and a few that must not follow
            t = o.new_state()
            assert t.feed_bytes(b"".join(toks[i] for i in ids))
            assert t.feed_bytes(bad) == ExprRow.feed(_copy_row(row), bad) == False, (r, bad)
    full = cfg.vocab()
    traj = load_trajectory(5, 6, 48)
    foff, fdata = wvocab.vocab_csr(full)
    flang = ExprLanguage(full)
    for b in range(6):
        s, row = o.new_state(), ExprRow()
        for k, ids in enumerate(traj):
            t = ids[b]
            if t < 0:
                s, row = o.new_state(), ExprRow()
                continue
            assert s.feed_bytes(full[t]) and row.feed(full[t]), (b, k)
            assert s.accepting() == row.accepting()
            if k % 12 == 11:
                assert (s.mask(foff, fdata, 8) == flang.mask(row.mode, row.depth)).all(), (b, k)


def _copy_row(row):
    from tests.expr_language import ExprRow
    c = ExprRow()
    c.mode, c.depth = row.mode, row.depth
    return c
