"""Seeded sentences of the expression language of configuration 5, cut into vocabulary tokens.

The oracle-sampled trajectory of configuration 5 ends where the oracle's cost allowed (it keeps
every Earley set).  To reach the configuration's full number of decode steps the tests also use
token sequences that are valid by construction: a seeded random expression over + * ( ) numbers
and lowercase identifiers is written out as bytes and cut greedily into the longest vocabulary
tokens that match.  Every prefix of a sentence can be completed, so every token of the sequence is
allowed where it stands.  Nothing here parses anything: strings are built from the outside in.
"""
from .rng import stream


def expr_sentence(seed: int, tag: str, min_bytes: int, max_depth: int = 5, flat: bool = True) -> bytes:
    """A sentence of at least min_bytes bytes.  flat: one long sum of operands at the top level (with an ambiguous
    grammar every operator is another way to split the sum: the sets grow with the sentence); otherwise a tree of
    parenthesised groups of two to four operands each (short sums at every level, nesting as deep as the length asks)."""
    rs = stream(seed, tag)
    digits, letters = b"0123456789", b"abcdefghijklmnopqrstuvwxyz"

    def simple() -> bytes:
        if rs.below(2):
            return bytes(digits[rs.below(10)] for _ in range(1 + rs.below(4)))
        return bytes(letters[rs.below(26)] for _ in range(1 + rs.below(5)))

    def operator() -> bytes:
        return b"+" if rs.below(2) else b"*"

    def operand(depth: int) -> bytes:
        if rs.below(10) < 2 and depth < max_depth:
            return b"(" + expr(depth + 1, 1 + rs.below(4)) + b")"
        return simple()

    def expr(depth: int, terms: int) -> bytes:
        out = operand(depth)
        for _ in range(terms - 1):
            out += operator() + operand(depth)
        return out

    def group(budget: int) -> bytes:
        terms = 2 + rs.below(3)
        out = b""
        for k in range(terms):
            share = budget // terms
            out += (operator() if k else b"") + (b"(" + group(share - 2) + b")" if share > 10 else simple())
        return out

    if not flat:
        return group(min_bytes + min_bytes // 2)
    out = operand(0)
    while len(out) < min_bytes:
        out += operator() + operand(0)
    return out


def cut_into_tokens(tokens, data: bytes, n_tokens: int):
    """Greedy longest-match cut of `data` into ids of `tokens` (the first id among duplicates); stops after n_tokens."""
    first = {}
    longest = 1
    for i, t in enumerate(tokens):
        if t and t not in first:
            first[t] = i
            longest = max(longest, len(t))
    ids, at = [], 0
    while at < len(data) and len(ids) < n_tokens:
        for n in range(min(longest, len(data) - at), 0, -1):
            i = first.get(data[at:at + n])
            if i is not None:
                ids.append(i)
                at += n
                break
        else:
            raise ValueError("no token matches: the vocabulary lacks a single byte")
    return ids
