"""CPU oracle front end -- TEST INFRASTRUCTURE ONLY (never imported by the product).

Turns a grammar description into the plain byte-class CFG that the C recognizer
(earley_oracle.c) runs on:

  * every regular-expression terminal is rewritten, straight from its syntax
    tree, into context-free rules over one-byte class terminals (x* => X -> eps |
    X x, x+ => X -> x | X x, x? => X -> eps | x, alternation => alternatives, a
    literal => one rule of single bytes).  No automaton is ever built here; a
    class terminal matches exactly one input byte (Scan, paper Section 3.2);
  * nonterminals that cannot derive any terminal string are removed (useless-rule
    removal, paper Section 4.5) so that "state set not empty" is the same as "the
    prefix can still be completed".

Everything after that (Predict / Scan / Complete, the vocabulary mask, logit
masking) is in the C file.
"""
import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile earley_oracle.c with gcc (OpenMP for the multi-threaded mask loop)."""
    src = os.path.join(_HERE, "earley_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        vp, ci, cl = ctypes.c_void_p, ctypes.c_int, ctypes.c_long
        L.orc_grammar_new.restype = vp
        L.orc_grammar_new.argtypes = [ci, ci, ci, vp, vp, vp, ci, vp]
        L.orc_grammar_free.argtypes = [vp]
        L.orc_is_nullable.argtypes = [vp, ci]
        L.orc_state_new.restype = vp
        L.orc_state_new.argtypes = [vp]
        L.orc_state_clone.restype = vp
        L.orc_state_clone.argtypes = [vp]
        L.orc_state_free.argtypes = [vp]
        L.orc_feed.argtypes = [vp, ctypes.c_uint8]
        L.orc_check.argtypes = [vp, vp, cl]
        L.orc_feed_bytes.argtypes = [vp, vp, cl]
        L.orc_accepting.argtypes = [vp]
        for f in ("orc_n_sets", "orc_n_items"):
            getattr(L, f).restype = cl
            getattr(L, f).argtypes = [vp]
        L.orc_set_size.restype = cl
        L.orc_set_size.argtypes = [vp, cl]
        L.orc_set_items.argtypes = [vp, cl, vp]
        L.orc_mask.argtypes = [vp, cl, vp, vp, vp, ci]
        L.orc_apply_mask.argtypes = [vp, vp, ci, cl, cl, cl, vp]
        _lib = L
    return _lib


# ---- regular-expression syntax tree ---------------------------------------------------
# node = ("set", frozenset of byte values) | ("cat", [nodes]) | ("alt", [nodes]) |
#        ("star", node) | ("plus", node) | ("opt", node)
_ESC = {ord("n"): 10, ord("r"): 13, ord("t"): 9}


class _P:
    def __init__(self, src: bytes):
        self.s, self.i = src, 0

    def peek(self):
        return self.s[self.i] if self.i < len(self.s) else None

    def take(self):
        c = self.s[self.i]
        self.i += 1
        return c

    def escape(self) -> int:
        c = self.take()
        if c == ord("x"):
            v = int(self.s[self.i:self.i + 2].decode(), 16)
            self.i += 2
            return v
        return _ESC.get(c, c)

    def alt(self):
        parts = [self.cat()]
        while self.peek() == ord("|"):
            self.take()
            parts.append(self.cat())
        return parts[0] if len(parts) == 1 else ("alt", parts)

    def cat(self):
        parts = []
        while self.peek() is not None and self.peek() not in b"|)":
            parts.append(self.postfix())
        return parts[0] if len(parts) == 1 else ("cat", parts)

    def postfix(self):
        a = self.atom()
        while self.peek() is not None and self.peek() in b"*+?{":
            c = self.take()
            if c == ord("*"):
                a = ("star", a)
            elif c == ord("+"):
                a = ("plus", a)
            elif c == ord("?"):
                a = ("opt", a)
            else:
                j = self.s.index(b"}", self.i)
                body = self.s[self.i:j].decode()
                self.i = j + 1
                if "," in body:
                    lo, hi = body.split(",")
                    lo = int(lo)
                    hi = None if hi == "" else int(hi)
                else:
                    lo = hi = int(body)
                # x{m,n} = m copies, then (n-m) nested optionals; x{m,} = m copies then x*
                seq = [a] * lo
                if hi is None:
                    seq.append(("star", a))
                else:
                    tail = None
                    for _ in range(hi - lo):
                        tail = ("opt", a if tail is None else ("cat", [a, tail]))
                    if tail is not None:
                        seq.append(tail)
                a = ("cat", seq)
        return a

    def atom(self):
        c = self.take()
        if c == ord("("):
            a = self.alt()
            assert self.take() == ord(")"), "unbalanced ("
            return a
        if c == ord("["):
            neg = self.peek() == ord("^")
            if neg:
                self.take()
            members = set()
            first = True
            while True:
                c = self.take()
                if c == ord("]") and not first:
                    break
                first = False
                lo = self.escape() if c == ord("\\") else c
                if self.peek() == ord("-") and self.s[self.i + 1] != ord("]"):
                    self.take()
                    c2 = self.take()
                    hi = self.escape() if c2 == ord("\\") else c2
                    members.update(range(lo, hi + 1))
                else:
                    members.add(lo)
            return ("set", frozenset(set(range(256)) - members if neg else members))
        if c == ord("."):
            return ("set", frozenset(range(256)))
        if c == ord("\\"):
            return ("set", frozenset([self.escape()]))
        return ("set", frozenset([c]))


def parse_regex(src: bytes):
    p = _P(src)
    node = p.alt()
    assert p.i == len(src), "trailing input in regex"
    return node


# ---- grammar -> byte-class CFG ------------------------------------------------------------
def desugar(grammar):
    """Return (names, rules, classes, start): rules = [(lhs, [sym])], sym >= 0 nonterminal,
    sym < 0 byte class ~sym, classes = list of frozensets of byte values."""
    from workloads.grammar import Lit
    names = list(grammar.nonterminals)
    rules = []
    classes, class_ix = [], {}

    def cls(members):
        members = frozenset(members)
        if members not in class_ix:
            class_ix[members] = len(classes)
            classes.append(members)
        return ~class_ix[members]

    def fresh(tag):
        names.append(f"{tag}#{len(names)}")
        return len(names) - 1

    def seq(node, tag):
        kind = node[0]
        if kind == "set":
            return [cls(node[1])]
        if kind == "cat":
            out = []
            for ch in node[1]:
                out += seq(ch, tag)
            return out
        x = fresh(tag)
        if kind == "alt":
            for ch in node[1]:
                rules.append((x, seq(ch, tag)))
        elif kind == "star":
            rules.append((x, []))
            rules.append((x, [x] + seq(node[1], tag)))
        elif kind == "plus":
            rules.append((x, seq(node[1], tag)))
            rules.append((x, [x] + seq(node[1], tag)))
        elif kind == "opt":
            rules.append((x, []))
            rules.append((x, seq(node[1], tag)))
        return [x]

    term_sym = []      # what stands for terminal t inside a rule
    for t, term in enumerate(grammar.terminals):
        if isinstance(term, Lit) and len(term.data) == 1:
            term_sym.append(cls(term.data))          # a one-byte literal is already a class terminal
            continue
        x = fresh(f"T{t}")
        term_sym.append(x)
        if isinstance(term, Lit):
            rules.append((x, [cls([b]) for b in term.data]))
        else:
            rules.append((x, seq(parse_regex(term.pattern), f"T{t}")))
    for lhs, rhs in grammar.rules:
        rules.append((lhs, [s if s >= 0 else term_sym[~s] for s in rhs]))

    # useless-rule removal: keep only rules whose symbols can all derive a terminal string
    productive = set()
    changed = True
    while changed:
        changed = False
        for lhs, rhs in rules:
            if lhs not in productive and all(s < 0 or s in productive for s in rhs):
                productive.add(lhs)
                changed = True
    if grammar.start not in productive:
        raise ValueError("start symbol derives no string")
    rules = [(l, r) for l, r in rules if l in productive and all(s < 0 or s in productive for s in r)]
    return names, rules, classes, grammar.start


class OracleState:
    def __init__(self, oracle, handle):
        self.o, self.h = oracle, handle

    def __del__(self):
        if _lib is not None and self.h:
            _lib.orc_state_free(self.h)
            self.h = None

    def clone(self):
        return OracleState(self.o, _lib.orc_state_clone(self.h))

    def feed(self, byte: int) -> bool:
        return bool(_lib.orc_feed(self.h, byte))

    def feed_bytes(self, data: bytes) -> bool:
        buf = (ctypes.c_uint8 * max(1, len(data))).from_buffer_copy(data or b"\0")
        return bool(_lib.orc_feed_bytes(self.h, buf, len(data)))

    def check(self, data: bytes) -> bool:
        buf = (ctypes.c_uint8 * max(1, len(data))).from_buffer_copy(data or b"\0")
        return bool(_lib.orc_check(self.h, buf, len(data)))

    def accepting(self) -> bool:
        return bool(_lib.orc_accepting(self.h))

    def n_sets(self) -> int:
        return _lib.orc_n_sets(self.h)

    def n_items(self) -> int:
        return _lib.orc_n_items(self.h)

    def set_items(self, k: int):
        """Items of S[k] as (lhs name, rhs tuple, dot, origin) with readable symbols."""
        n = _lib.orc_set_size(self.h, k)
        buf = np.zeros((max(n, 1), 3), dtype=np.int32)
        _lib.orc_set_items(self.h, k, buf.ctypes.data)
        return [self.o.describe(int(r), int(d), int(o)) for r, d, o in buf[:n]]

    def mask(self, vocab_off, vocab_bytes, n_threads: int = 0):
        V = len(vocab_off) - 1
        out = np.zeros((V + 31) // 32, dtype=np.uint32)
        vb = vocab_bytes if len(vocab_bytes) else np.zeros(1, np.uint8)
        self.o.last_threads = _lib.orc_mask(self.h, V, vocab_off.ctypes.data, vb.ctypes.data,
                                            out.ctypes.data, n_threads)
        return out


class Oracle:
    """Textbook Earley recognizer for a grammar description (see workloads.grammar)."""

    def __init__(self, grammar):
        L = _load()
        self.names, self.rules, self.classes, self.start = desugar(grammar)
        lhs = np.array([r[0] for r in self.rules], dtype=np.int32)
        off = np.zeros(len(self.rules) + 1, dtype=np.int32)
        syms = []
        for i, (_, rhs) in enumerate(self.rules):
            syms += rhs
            off[i + 1] = len(syms)
        sym = np.array(syms + [0], dtype=np.int32)
        bits = np.zeros((max(1, len(self.classes)), 32), dtype=np.uint8)
        for c, members in enumerate(self.classes):
            for b in members:
                bits[c, b >> 3] |= 1 << (b & 7)
        self._keep = (lhs, off, sym, bits)
        self.g = L.orc_grammar_new(len(self.names), self.start, len(self.rules), lhs.ctypes.data,
                                   off.ctypes.data, sym.ctypes.data, len(self.classes), bits.ctypes.data)
        self.last_threads = 1

    def __del__(self):
        if _lib is not None and getattr(self, "g", None):
            _lib.orc_grammar_free(self.g)
            self.g = None

    def new_state(self) -> OracleState:
        return OracleState(self, _lib.orc_state_new(self.g))

    def nullable(self, name: str) -> bool:
        return bool(_lib.orc_is_nullable(self.g, self.names.index(name)))

    def _sym(self, s):
        if s >= 0:
            return self.names[s]
        m = self.classes[~s]
        return bytes(sorted(m)) if len(m) <= 4 else f"<class of {len(m)}>"

    def describe(self, rule, dot, origin):
        if rule == len(self.rules):
            return ("S'", (self.names[self.start],), dot, origin)
        lhs, rhs = self.rules[rule]
        return (self.names[lhs], tuple(self._sym(s) for s in rhs), dot, origin)


def apply_mask(logits: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """logits: [B, V] array of uint32 (binary32 bits) or uint16 (bfloat16 bits); mask [B, W]."""
    L = _load()
    assert logits.dtype in (np.uint32, np.uint16) and logits.flags.c_contiguous
    mask = np.ascontiguousarray(mask, dtype=np.uint32)
    out = np.empty_like(logits)
    B, V = logits.shape
    L.orc_apply_mask(logits.ctypes.data, out.ctypes.data, logits.dtype.itemsize, B, V, V, mask.ctypes.data)
    return out
