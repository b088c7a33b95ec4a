"""The viable prefixes of configuration 5's expression language, from its definition (test infrastructure).

The language of E -> E+E | E*E | (E) | num | id with num = [0-9]+ and id = [a-z]+ is the set of
strings in which operands (a number, an identifier, or a parenthesised expression) and the
operators + and * alternate, starting and ending with an operand, with balanced parentheses.  A
string is a prefix of a sentence exactly when a left-to-right scan never has to reject a byte: it
can always be completed by finishing the operand in hand and closing the open parentheses.  So a
token's verdict after a prefix depends on two facts about the prefix only -- what the scan expects
next and how many parentheses are open -- and on the token alone for the rest: per start situation,
whether the token scans at all and how many open parentheses it needs.  That makes the mask of every
row at every decode step computable at the full vocabulary and any prefix length, where the Earley
oracle (which keeps every set of an ambiguous grammar) needs minutes per mask.  The Earley oracle
pins this description on short prefixes (tests/test_oracle_pins.py).
"""
import numpy as np

OPERAND, IN_NUM, IN_ID, CLOSED = 0, 1, 2, 3      # what the scan has just seen: nothing usable yet / digits / letters / a closing parenthesis
NEVER = 1 << 30


def scan(mode: int, data: bytes):
    """Scan `data` from `mode`.  Returns (end mode, opened - closed, parentheses that must already be open),
    or None when some byte cannot follow."""
    net, need = 0, 0
    for b in data:
        c = chr(b)
        if c.isdigit() and c.isascii():
            if mode in (OPERAND, IN_NUM):
                mode = IN_NUM
            else:
                return None
        elif "a" <= c <= "z":
            if mode in (OPERAND, IN_ID):
                mode = IN_ID
            else:
                return None
        elif c == "(":
            if mode != OPERAND:
                return None
            net += 1
        elif c == ")":
            if mode == OPERAND:
                return None
            net -= 1
            need = max(need, -net)
            mode = CLOSED
        elif c in "+*":
            if mode == OPERAND:
                return None
            mode = OPERAND
        else:
            return None
    return mode, net, need


class ExprLanguage:
    def __init__(self, tokens):
        self.tokens = tokens
        self.W = (len(tokens) + 31) // 32
        self.need = np.full((4, self.W * 32), NEVER, dtype=np.int64)   # [start mode][token] open parentheses the token needs
        for m in range(4):
            for v, t in enumerate(tokens):
                if not t:
                    continue                                           # the empty token is never allowed
                r = scan(m, t)
                if r is not None:
                    self.need[m, v] = r[2]

    def mask(self, mode: int, depth: int) -> np.ndarray:
        bits = (self.need[mode] <= depth).astype(np.uint8)
        return np.packbits(bits, bitorder="little").view(np.uint32)


class ExprRow:
    """One query: where the scan stands after the bytes fed so far."""

    def __init__(self):
        self.mode, self.depth = OPERAND, 0

    def feed(self, data: bytes) -> bool:
        r = scan(self.mode, data)
        if r is None or r[2] > self.depth or not data:
            return False
        self.mode, self.depth = r[0], self.depth + r[1]
        return True

    def accepting(self) -> bool:
        return self.depth == 0 and self.mode != OPERAND
