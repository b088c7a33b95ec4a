"""Seeded random context-free grammars and vocabularies for differential tests.

Shapes are drawn on purpose from the awkward corners: empty right-hand sides, unit rules and
unit cycles, left and right recursion, ambiguity, nullable prefixes before a recursive call,
literals that share prefixes, regex terminals that may end at every byte.  Every nonterminal
gets one terminal-only rule, so every symbol is productive.  No parsing logic lives here.
"""
from .grammar import Grammar, Lit, Rx
from .rng import stream

_REGEXES = [rb"[ab]+", rb"a[bc]*", rb"(ab|c)+", rb"[0-9]+", rb"b{1,3}", rb"c?a", rb"[0-9]+(\.[0-9]+)?", rb"(a|b)c*b",
            rb"[^abc0-9]", rb"a{2}|b"]
_ALPHABET = b"abc01. "


def random_grammar(seed: int) -> Grammar:
    rs = stream(seed, "random-grammar")
    n_nt = 2 + rs.below(5)
    names = [f"N{i}" for i in range(n_nt)]
    terms = []
    for _ in range(2 + rs.below(4)):
        if rs.below(3) == 0:
            terms.append(Rx(_REGEXES[rs.below(len(_REGEXES))]))
        else:
            terms.append(Lit(bytes(_ALPHABET[rs.below(len(_ALPHABET))] for _ in range(1 + rs.below(3)))))
    g = Grammar(name=f"random{seed}")
    g.set_start(names[0])
    for a in names:
        g.rule(a, [terms[rs.below(len(terms))] for _ in range(1 + rs.below(2))])      # keeps `a` productive
        for _ in range(rs.below(4)):
            rhs = []
            for _ in range(rs.below(5)):                                               # length 0 = an empty rule
                rhs.append(names[rs.below(n_nt)] if rs.below(2) else terms[rs.below(len(terms))])
            g.rule(a, rhs)
    return g


def random_vocab(seed: int, n_tokens: int = 160):
    """Single bytes of the alphabet (plus two bytes outside it) and random strings over it."""
    rs = stream(seed, "random-vocab")
    toks = [bytes([b]) for b in _ALPHABET] + [b"z", b"\xc3"]
    while len(toks) < n_tokens:
        toks.append(bytes(_ALPHABET[rs.below(len(_ALPHABET))] for _ in range(1 + rs.below(6))))
    return toks
