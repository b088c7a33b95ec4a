"""A neutral description of a context-free grammar with byte-level terminals.

Terminals are either literal byte strings (``Lit``) or sources in a tiny
byte-oriented regular-expression dialect (``Rx``):

    literal bytes, ``\\xHH``, ``\\n \\r \\t``, ``\\<punct>``; ``.`` (any byte);
    classes ``[a-z0-9]`` / ``[^...]``; grouping ``( )``; alternation ``|``;
    postfix ``* + ?`` and ``{m}``, ``{m,}``, ``{m,n}``.  No anchors, no
    longest-match rule: a terminal matches any member of its language.

The container only stores symbols; interpreting them is the consumer's job.
"""
from dataclasses import dataclass, field
import numpy as np


@dataclass(frozen=True)
class Lit:
    data: bytes


@dataclass(frozen=True)
class Rx:
    pattern: bytes


@dataclass
class Grammar:
    name: str = "grammar"
    nonterminals: list = field(default_factory=list)   # names
    rules: list = field(default_factory=list)          # (lhs index, [symbols]); sym >= 0 nonterminal, < 0 terminal ~sym
    terminals: list = field(default_factory=list)      # Lit | Rx
    start: int = 0
    _nt_index: dict = field(default_factory=dict)
    _t_index: dict = field(default_factory=dict)

    def nt(self, name: str) -> int:
        if name not in self._nt_index:
            self._nt_index[name] = len(self.nonterminals)
            self.nonterminals.append(name)
        return self._nt_index[name]

    def term(self, t) -> int:
        if t not in self._t_index:
            self._t_index[t] = len(self.terminals)
            self.terminals.append(t)
        return self._t_index[t]

    def rule(self, lhs: str, rhs):
        """Add lhs -> rhs; rhs items are nonterminal names (str), Lit, Rx or bytes (= Lit)."""
        syms = []
        for s in rhs:
            if isinstance(s, str):
                syms.append(self.nt(s))
            else:
                if isinstance(s, (bytes, bytearray)):
                    s = Lit(bytes(s))
                syms.append(~self.term(s))
        self.rules.append((self.nt(lhs), syms))
        return self

    def alts(self, lhs: str, *alternatives):
        for a in alternatives:
            self.rule(lhs, a)
        return self

    def set_start(self, name: str):
        self.start = self.nt(name)
        return self

    # flat CSR arrays in the layout the C boundary takes
    def csr(self):
        lhs = np.array([r[0] for r in self.rules], dtype=np.int32)
        off = np.zeros(len(self.rules) + 1, dtype=np.int32)
        sym = []
        for i, (_, rhs) in enumerate(self.rules):
            sym.extend(rhs)
            off[i + 1] = len(sym)
        sym = np.array(sym, dtype=np.int32) if sym else np.zeros(0, dtype=np.int32)
        kind = np.array([0 if isinstance(t, Lit) else 1 for t in self.terminals], dtype=np.uint8)
        toff = np.zeros(len(self.terminals) + 1, dtype=np.int64)
        data = bytearray()
        for i, t in enumerate(self.terminals):
            data += t.data if isinstance(t, Lit) else t.pattern
            toff[i + 1] = len(data)
        tdata = np.frombuffer(bytes(data), dtype=np.uint8).copy() if data else np.zeros(0, dtype=np.uint8)
        return dict(n_nonterminals=len(self.nonterminals), start=self.start, rule_lhs=lhs,
                    rhs_off=off, rhs_sym=sym, term_kind=kind, term_off=toff, term_data=tdata)
