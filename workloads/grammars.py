"""The grammars of the five benchmark configurations plus small test grammars.

All identifiers (keys, enum members, predicate and entity names) are drawn
from seeded streams; nothing here comes from an external dataset.
"""
from .grammar import Grammar, Lit, Rx
from .rng import stream

# ---- shared terminal sources (tiny byte-regex dialect, see grammar.py) -------------------
WS_RX = Rx(rb'[ \t\n\r]+')
NUMBER_RX = Rx(rb'-?(0|[1-9][0-9]*)(\.[0-9]+)?([eE][-+]?[0-9]+)?')
INTEGER_RX = Rx(rb'-?(0|[1-9][0-9]*)')
# RFC 8259 string: unescaped bytes >= 0x20 except '"' and '\', well-formed UTF-8
# multi-byte sequences (RFC 3629 table), or an escape.
STRING_RX = Rx(
    rb'"('
    rb'[^"\\\x00-\x1f\x80-\xff]'
    rb'|[\xc2-\xdf][\x80-\xbf]'
    rb'|\xe0[\xa0-\xbf][\x80-\xbf]'
    rb'|[\xe1-\xec\xee\xef][\x80-\xbf][\x80-\xbf]'
    rb'|\xed[\x80-\x9f][\x80-\xbf]'
    rb'|\xf0[\x90-\xbf][\x80-\xbf][\x80-\xbf]'
    rb'|[\xf1-\xf3][\x80-\xbf][\x80-\xbf][\x80-\xbf]'
    rb'|\xf4[\x80-\x8f][\x80-\xbf][\x80-\xbf]'
    rb'|\\(["\\/bfnrt]|u[0-9a-fA-F]{4})'
    rb')*"')


def _ident(rs, lo, hi, taken):
    while True:
        n = lo + rs.below(hi - lo + 1)
        s = bytes(97 + rs.below(26) for _ in range(n))
        if s not in taken:
            taken.add(s)
            return s


def json_grammar() -> Grammar:
    """RFC 8259 at byte level; any value may be the top level; ws is a nullable nonterminal."""
    g = Grammar(name="json")
    g.set_start("json")
    g.rule("json", ["ws", "value", "ws"])
    g.alts("value", ["object"], ["array"], ["string"], ["number"], [b"true"], [b"false"], [b"null"])
    g.alts("object", [b"{", "ws", b"}"], [b"{", "ws", "members", "ws", b"}"])
    g.alts("members", ["member"], ["members", "ws", b",", "ws", "member"])
    g.rule("member", ["string", "ws", b":", "ws", "value"])
    g.alts("array", [b"[", "ws", b"]"], [b"[", "ws", "elements", "ws", b"]"])
    g.alts("elements", ["value"], ["elements", "ws", b",", "ws", "value"])
    g.rule("string", [STRING_RX])
    g.rule("number", [NUMBER_RX])
    g.alts("ws", [], [WS_RX])
    return g


def json_schema_grammar(seed: int) -> Grammar:
    """An object with 8 required keys in declared order (kinds: string, integer, number,
    boolean, enum of 5, array of <= 10 integers, nested object of 3 keys, string)."""
    rs = stream(seed, "grammar")
    taken = set()
    keys = [_ident(rs, 3, 10, taken) for _ in range(8)]
    enum = [_ident(rs, 3, 10, taken) for _ in range(5)]
    nkeys = [_ident(rs, 3, 10, taken) for _ in range(3)]
    g = Grammar(name="json_schema")
    g.set_start("root")
    kinds = ["string", "integer", "number", "boolean", "enum", "array", "nested", "string"]
    rhs = [b"{", "ws"]
    for i, (k, kind) in enumerate(zip(keys, kinds)):
        if i:
            rhs += ["ws", b",", "ws"]
        rhs += [Lit(b'"' + k + b'"'), "ws", b":", "ws", kind]
    rhs += ["ws", b"}"]
    g.rule("root", rhs)
    g.rule("string", [STRING_RX])
    g.rule("integer", [INTEGER_RX])
    g.rule("number", [NUMBER_RX])
    g.alts("boolean", [b"true"], [b"false"])
    for e in enum:
        g.rule("enum", [Lit(b'"' + e + b'"')])
    g.alts("array", [b"[", "ws", b"]"], [b"[", "ws", "ints10", "ws", b"]"])
    g.rule("ints1", ["integer"])
    for k in range(2, 11):
        g.alts(f"ints{k}", ["integer"], ["integer", "ws", b",", "ws", f"ints{k-1}"])
    g.rule("nested", [b"{", "ws",
                      Lit(b'"' + nkeys[0] + b'"'), "ws", b":", "ws", "string", "ws", b",", "ws",
                      Lit(b'"' + nkeys[1] + b'"'), "ws", b":", "ws", "integer", "ws", b",", "ws",
                      Lit(b'"' + nkeys[2] + b'"'), "ws", b":", "ws", "string", "ws", b"}"])
    g.alts("ws", [], [WS_RX])
    return g


def semantic_grammar(seed: int) -> Grammar:
    """A typed query language (select/where/and/or/not/count/argmax, parenthesised
    application) with 100 predicate and 100 entity identifier terminals."""
    rs = stream(seed, "grammar")
    taken = set()
    preds = [_ident(rs, 3, 12, taken) for _ in range(100)]
    ents = [_ident(rs, 3, 12, taken) for _ in range(100)]
    g = Grammar(name="semantic")
    g.set_start("query")
    g.rule("query", [b"answer(", "term", b")"])
    g.alts("term", ["set"], [b"count(", "set", b")"], [b"argmax(", "set", b", ", "field", b")"],
           [b"argmin(", "set", b", ", "field", b")"], [b"sum(", "set", b", ", "field", b")"],
           [b"avg(", "set", b", ", "field", b")"], [b"the(", "set", b")"])
    g.alts("set", [b"select(", "pred", b")"], [b"select(", "pred", b" where ", "cond", b")"],
           ["pred", b"(", "args", b")"], [b"all"], [b"lambda ", "var", b". ", "cond"],
           [b"largest(", "field", b", ", "set", b")"], [b"smallest(", "field", b", ", "set", b")"],
           [b"most(", "set", b", ", "pred", b")"], [b"fewest(", "set", b", ", "pred", b")"],
           [b"union(", "set", b", ", "set", b")"], [b"intersect(", "set", b", ", "set", b")"])
    g.alts("cond", ["conj"], ["cond", b" or ", "conj"])
    g.alts("conj", ["neg"], ["conj", b" and ", "neg"])
    g.alts("neg", [b"not ", "neg"], [b"(", "cond", b")"], ["rel"])
    g.alts("rel", ["pred", b"(", "args", b")"], ["field", b" ", "op", b" ", "value"],
           [b"exists(", "set", b")"], [b"in(", "value", b", ", "set", b")"], [b"true"], [b"false"])
    g.alts("args", ["arg"], ["args", b", ", "arg"])
    g.alts("arg", ["entity"], ["set"], ["value"], ["var"])
    g.alts("field", ["pred"], ["pred", b".", "pred"], ["var", b".", "pred"])
    g.alts("value", ["num"], ["entity"], [b"-", "num"])
    g.alts("op", [b"="], [b"!="], [b"<"], [b"<="], [b">"], [b">="], [b"like"])
    g.alts("var", [b"x"], [b"y"], [b"z"], [b"w"])
    g.rule("num", [Rx(rb'[0-9]+(\.[0-9]+)?')])
    for p in preds:
        g.rule("pred", [Lit(p)])
    for e in ents:
        g.rule("entity", [Lit(b"'" + e + b"'")])
    return g


def expr_grammar() -> Grammar:
    """Ambiguous, left- and right-recursive: E -> E+E | E*E | (E) | num | id."""
    g = Grammar(name="expr")
    g.set_start("E")
    g.alts("E", ["E", b"+", "E"], ["E", b"*", "E"], [b"(", "E", b")"],
           [Rx(rb'[0-9]+')], [Rx(rb'[a-z]+')])
    return g


# ---- small grammars for tests --------------------------------------------------------
def w1_grammar() -> Grammar:
    """A -> A B | B ; B -> a   (left recursion over a one-byte terminal)."""
    g = Grammar(name="w1")
    g.set_start("A")
    g.alts("A", ["A", "B"], ["B"])
    g.rule("B", [b"a"])
    return g


def w2_grammar() -> Grammar:
    """S -> A B ; A -> a ; B -> b."""
    g = Grammar(name="w2")
    g.set_start("S")
    g.rule("S", ["A", "B"])
    g.rule("A", [b"a"])
    g.rule("B", [b"b"])
    return g


def w3_grammar() -> Grammar:
    """S -> A + B ; A -> a | c ; B -> b | d."""
    g = Grammar(name="w3")
    g.set_start("S")
    g.rule("S", ["A", b"+", "B"])
    g.alts("A", [b"a"], [b"c"])
    g.alts("B", [b"b"], [b"d"])
    return g


def parens_grammar() -> Grammar:
    """Balanced parentheses, nullable start: S -> eps | S ( S )."""
    g = Grammar(name="parens")
    g.set_start("S")
    g.alts("S", [], ["S", b"(", "S", b")"])
    return g


def anbn_grammar() -> Grammar:
    """{ a^n b^n : n >= 1 }."""
    g = Grammar(name="anbn")
    g.set_start("S")
    g.alts("S", [b"a", b"b"], [b"a", "S", b"b"])
    return g


def palindrome_grammar() -> Grammar:
    """Even-length palindromes over {a,b} (inherently non-deterministic), nullable."""
    g = Grammar(name="pal")
    g.set_start("P")
    g.alts("P", [], [b"a", "P", b"a"], [b"b", "P", b"b"])
    return g


def nullable_chain_grammar() -> Grammar:
    """Heavily nullable: S -> A B C d ; A -> eps | a ; B -> eps | A b | B b ; C -> eps | c C."""
    g = Grammar(name="nullchain")
    g.set_start("S")
    g.rule("S", ["A", "B", "C", b"d"])
    g.alts("A", [], [b"a"])
    g.alts("B", [], ["A", b"b"], ["B", b"b"])
    g.alts("C", [], [b"c", "C"])
    return g


def useless_grammar() -> Grammar:
    """Has unproductive (U, never terminates) and unreachable (X) nonterminals."""
    g = Grammar(name="useless")
    g.set_start("S")
    g.alts("S", [b"a", "S"], [b"b"], ["U", b"c"])
    g.rule("U", [b"u", "U"])
    g.rule("X", [b"x"])
    return g


def regex_only_grammar(pattern: bytes) -> Grammar:
    """S -> T with a single regex terminal."""
    g = Grammar(name="regex")
    g.set_start("S")
    g.rule("S", [Rx(pattern)])
    return g


def multibyte_literal_grammar() -> Grammar:
    """Literals that share prefixes and an ambiguous split between two terminals."""
    g = Grammar(name="mblit")
    g.set_start("S")
    g.alts("S", ["K", "S"], ["K"])
    g.alts("K", [b"ab"], [b"abc"], [b"c"], [Rx(rb'ab*')], [b"(", "S", b")"])
    return g


def many_classes_grammar(n: int = 100) -> Grammar:
    """S -> T S | T ; T -> one of n two-byte literals whose first bytes are all different, so that the
    terminals' automata tell more than 64 byte classes apart."""
    g = Grammar(name=f"many_classes_{n}")
    g.set_start("S")
    g.rule("S", ["T", "S"])
    g.rule("S", ["T"])
    for c in range(n):
        g.rule("T", [bytes([32 + c, 32 + (c * 7 + 3) % n])])
    return g


def big_tables_grammar(n_words: int, word_len: int, seed: int = 11) -> Grammar:
    """S -> W | W ' ' S ; W -> one of n_words seeded lowercase literals of word_len letters: as many DFA
    states and tabulated scan entries as a test needs to outgrow the kernels' LDS budget for grammar tables."""
    rs = stream(seed, f"big-tables[{n_words},{word_len}]")
    words = set()
    while len(words) < n_words:
        words.add(bytes(97 + rs.below(26) for _ in range(word_len)))
    g = Grammar(name=f"big_tables_{n_words}x{word_len}")
    g.set_start("S")
    g.rule("S", ["W"])
    g.rule("S", ["W", b" ", "S"])
    for w in sorted(words):
        g.rule("W", [w])
    return g
